// Per-example weight gradient of the LSTM layer (Section 1, item 2a):  G_b = [x_t | h_{t-1} | 1]^T dgates_t summed
// over the time steps, a (Din + H + 1) x 4H matrix per example in the layer's parameter layout (W_ih, W_hh, b),
// its squared norm for the clip factor (item 2b), and optionally the matrix itself for the weighted sum that forms
// the clipped sum (item 3).
//
// Two workgroups of eight waves own one example, each one half of the columns and all rows: with 16x16 blocks of
// v_mfma_f32_16x16x4_f32 the 201 x 400 matrix of the benchmark networks is 13 x 25 blocks with 3.5 % padding (tiles
// of 32-row MFMA blocks pad it by 43 %).  Wave (wm, wn) holds up to 7 x 4 blocks in registers; the time axis is
// walked in chunks of 32 steps staged in LDS ([t][row] for both operands, row lengths that put the four k-lanes of
// an MFMA operand on different banks), two buffers, one barrier per chunk; the next chunk travels in registers
// meanwhile.  Staging addresses are fixed per thread and computed once.
// A workgroup is PERSISTENT: it keeps its half of the columns and walks over examples blockIdx.x, blockIdx.x +
// gridDim.x, ...; the chunk pipeline runs on across examples (the next example's first chunk is on its way during the
// current one's last), and the stores of an example's gradient are issued after the next chunk has been staged and
// its successor requested, right before that chunk's multiplies -- so the wait that precedes the following staging,
// which the compiler cannot make finer than "everything", comes a whole chunk of multiplies after them.  The squared
// norm leaves the kernel as one partial per wave (16 slots per example), which needs no barrier.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

typedef float lwg_f32x4 __attribute__((ext_vector_type(4)));

#define LWG_THREADS 512
#define LWG_BK 32      // time steps per chunk
#define LWG_MB 13      // 16-row blocks of the output (rows: Din + H + 1 <= 208)
#define LWG_NH 13      // 16-column blocks per half (columns: 4H <= 416)
#define LWG_LD 208     // LDS row length of both operands: 208 % 64 = 16, so rows t .. t+3 start 16 banks apart
#define LWG_TM 7       // blocks per wave: rows [0, 7) / [7, 13); columns 4, 3, 3, 3 of the half's 13
#define LWG_TN 4
#define LWG_ITEMS 4    // groups of four floats a thread stages per operand and chunk: 32 * 52 / 512 rounded up

struct LstmWgArgs {
  const float *x;      // [B][T][Din]
  const float *hs;     // [B][T][H]   h_t; row t of the operand uses h_{t-1} (zero for t = 0)
  const float *dg;     // [B][T][4H]  gate gradients
  float *slots;        // squared norms, one partial per wave: slots[(slot0 + half * 8 + wave) * slot_stride + b]
  long slot_stride; int slot0;
  float *gstore;       // [B][gstride] or null
  long gstride;
  int B, T, Din, H;
};

static inline bool lstm_wgrad_fits(int Din, int H, int T) {
  return Din >= 4 && H >= 4 && (Din & 3) == 0 && (H & 3) == 0 && Din + H + 1 <= LWG_MB * 16 && 4 * H <= 2 * LWG_NH * 16 && T >= 1;
}
static inline size_t lstm_wgrad_lds_bytes() { return sizeof(float) * (2 * LWG_BK * 2 * LWG_LD); }
#define LWG_SLOTS 16 // slots per example: 2 halves x 8 waves

__global__ __launch_bounds__(LWG_THREADS) void lstm_wgrad_kernel(const LstmWgArgs a) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63, i16 = lane & 15, kq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // waves w and w + 4 share a SIMD: the second row of waves takes the column groups in rotated order, so that the
  // SIMD that hosts the widest group of the upper rows hosts a narrow one of the lower rows
  const int wm = wave >> 2, wn = (wave + 2 * wm) & 3;
  const int half = blockIdx.y;
  const int Din = a.Din, H = a.H, T = a.T, G = 4 * H, M = Din + H + 1;
  const int n_half0 = half * (LWG_NH * 16);              // first column of this workgroup
  const int n_cols = min(G - n_half0, LWG_NH * 16);      // its columns (a multiple of 4)
  const int m_blk0 = wm * 7, m_cnt = wm == 0 ? 7 : 6;
  // the half's column blocks dealt to the four column groups: 13 -> 4, 3, 3, 3; 12 -> 3, 3, 3, 3; ...
  const int nb_total = (n_cols + 15) >> 4, nb_base = nb_total >> 2, nb_rem = nb_total & 3;
  const int n_cnt = nb_base + (wn < nb_rem ? 1 : 0), n_blk0 = wn * nb_base + min(wn, nb_rem);

  // staging items, fixed per thread: (step tt of the chunk, group g of four floats).  A: x, then h of the step
  // before, then the group that starts with the constant 1.  B: this half's columns of the gate gradients.
  const int a_groups = (Din + H) / 4 + 1, b_groups = n_cols / 4;
  int a_lds[LWG_ITEMS], a_src[LWG_ITEMS], a_tk[LWG_ITEMS]; // LDS offset (-1: none); source offset from step t0; tt | kind << 8
  int b_lds[LWG_ITEMS], b_src[LWG_ITEMS], b_tt[LWG_ITEMS];
#pragma unroll
  for (int q = 0; q < LWG_ITEMS; ++q) {
    const int it = tid + q * LWG_THREADS;
    {
      const int tt = it / a_groups, g = it - tt * a_groups;
      const int kind = 4 * g < Din ? 1 : (4 * g < Din + H ? 2 : 3);
      a_lds[q] = tt < LWG_BK ? tt * LWG_LD + 4 * g : -1;
      a_src[q] = kind == 1 ? tt * Din + 4 * g : (kind == 2 ? (tt - 1) * H + (4 * g - Din) : 0);
      a_tk[q] = tt | (kind << 8);
    }
    {
      const int tt = b_groups > 0 ? it / b_groups : LWG_BK, g = it - tt * b_groups;
      b_lds[q] = tt < LWG_BK ? tt * LWG_LD + 4 * g : -1;
      b_src[q] = tt * G + n_half0 + 4 * g;
      b_tt[q] = tt;
    }
  }
  float4 ra[LWG_ITEMS], rb[LWG_ITEMS];

  // fetch only issues loads, every one unconditional and from a valid address (a load under a branch would be waited
  // for at the join, one memory latency per item); what an item is worth is decided when it is written to LDS
  auto fetch = [&](int b, int t0) {
    const float *xb = a.x + (long)b * T * Din, *hb = a.hs + (long)b * T * H, *gb = a.dg + (long)b * T * G;
#pragma unroll
    for (int q = 0; q < LWG_ITEMS; ++q) {
      const int tt = a_tk[q] & 255, kind = a_tk[q] >> 8, t = t0 + tt;
      const bool ld = a_lds[q] >= 0 && t < T && (kind == 1 || (kind == 2 && t > 0));
      const float *base = kind == 2 ? hb : xb;
      const long off = ld ? (long)t0 * (kind == 2 ? H : Din) + a_src[q] : 0;
      ra[q] = *reinterpret_cast<const float4 *>(base + off);
    }
#pragma unroll
    for (int q = 0; q < LWG_ITEMS; ++q) {
      const bool ok = b_lds[q] >= 0 && t0 + b_tt[q] < T;
      const long off = ok ? (long)t0 * G + b_src[q] : 0;
      rb[q] = *reinterpret_cast<const float4 *>(gb + off);
    }
  };
  auto stash = [&](float *As, float *Bs, int t0) {
#pragma unroll
    for (int q = 0; q < LWG_ITEMS; ++q) {
      const int tt = a_tk[q] & 255, kind = a_tk[q] >> 8, t = t0 + tt;
      const bool ok = t < T, ld = ok && (kind == 1 || (kind == 2 && t > 0));
      float4 v = ra[q];
      const float one = (ok && kind == 3) ? 1.f : 0.f; // the group that opens with the constant 1 (the bias row)
      v.x = ld ? v.x : one; v.y = ld ? v.y : 0.f; v.z = ld ? v.z : 0.f; v.w = ld ? v.w : 0.f;
      if (a_lds[q] >= 0) *reinterpret_cast<float4 *>(As + a_lds[q]) = v;
      float4 w = rb[q];
      const bool okb = t0 + b_tt[q] < T;
      w.x = okb ? w.x : 0.f; w.y = okb ? w.y : 0.f; w.z = okb ? w.z : 0.f; w.w = okb ? w.w : 0.f;
      if (b_lds[q] >= 0) *reinterpret_cast<float4 *>(Bs + b_lds[q]) = w;
    }
  };

  // rows / columns beyond the operands' width are never staged: zero them once, in both buffers
  {
    const int a0 = 4 * a_groups, b0 = 4 * b_groups; // first unstaged column of an A row, of a B row
    for (int i = tid; i < 2 * LWG_BK * LWG_LD; i += LWG_THREADS) {
      const int row = i / LWG_LD, col = i - row * LWG_LD;       // row: buffer * 32 + step
      float *base = lds + (row >> 5) * (LWG_BK * 2 * LWG_LD) + (row & 31) * LWG_LD;
      if (col >= a0) base[col] = 0.f;
      if (col >= b0) base[LWG_BK * LWG_LD + col] = 0.f;
    }
  }
  __syncthreads();
  const int n_chunks = (T + LWG_BK - 1) / LWG_BK;
  const int b_first = blockIdx.x, b_step = gridDim.x;
  if (b_first >= a.B) return;
  const int n_items = (a.B - b_first + b_step - 1) / b_step;
  fetch(b_first, 0);
  // The multiply loop and the epilogue, compiled for each of the four wave tiles (7 or 6 row blocks x 4 or 3 column
  // blocks): with the block counts as constants the loop body is branch-free, so the LDS reads of one k-step are
  // issued under the multiplies of the one before.  A wave with fewer than three column blocks of real data runs the
  // 3-wide tile: the blocks beyond its data multiply zeros or values of another row, and are masked when stored.
  auto run = [&](auto mc_, auto nc_) {
    constexpr int MC = decltype(mc_)::value, NC = decltype(nc_)::value;
    lwg_f32x4 acc[MC][NC];
#pragma unroll
    for (int i = 0; i < MC; ++i)
#pragma unroll
      for (int j = 0; j < NC; ++j) acc[i][j] = (lwg_f32x4){0.f, 0.f, 0.f, 0.f};
    // the example's gradient (optional) and this wave's share of its squared norm; accumulator register r of a lane
    // is row 4 kq + r, column i16 of its block.  Leaves the accumulators at zero for the next example.
    auto finish = [&](int b) {
      // (lane indices from an opaque copy of the thread index: the compiler would otherwise keep the 112 store
      // addresses alive across the chunk loop and spill)
      int t_ = tid;
      asm volatile("" : "+v"(t_));
      const int i16_ = t_ & 15, kq_ = (t_ >> 4) & 3;
      float *gs = a.gstore ? a.gstore + (long)b * a.gstride : nullptr;
      const int m_lane = m_blk0 * 16 + 4 * kq_, nl_lane = n_blk0 * 16 + i16_;
      float *gl = gs ? gs + (long)m_lane * G + n_half0 + nl_lane : nullptr;
      float q2 = 0.f;
#pragma unroll
      for (int i = 0; i < MC; ++i)
#pragma unroll
        for (int j = 0; j < NC; ++j) {
          const int nl = nl_lane + j * 16;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int m = m_lane + i * 16 + r;
            if (j < n_cnt && m < M && nl < n_cols) {
              const float v = acc[i][j][r];
              q2 = fmaf(v, v, q2);
              if (gl) gl[(long)(i * 16 + r) * G + j * 16] = v;
            }
          }
          acc[i][j] = (lwg_f32x4){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) q2 += __shfl_xor(q2, o, 64);
      if ((t_ & 63) == 0) a.slots[(long)(a.slot0 + half * 8 + wave) * a.slot_stride + b] = q2;
    };
    int b_cur = b_first, c = 0, b_done = -1;
    const int total = n_items * n_chunks;
    for (int g = 0; g < total; ++g) {
      float *As = lds + (g & 1) * LWG_BK * 2 * LWG_LD, *Bs = As + LWG_BK * LWG_LD;
      stash(As, Bs, c * LWG_BK);
      __syncthreads(); // chunk g is staged; every wave has finished chunk g - 1 (it stashed g after its multiplies)
      int b_next = b_cur, c_next = c + 1;
      if (c_next == n_chunks) { c_next = 0; b_next += b_step; }
      if (g + 1 < total) fetch(b_next, c_next * LWG_BK);
      if (b_done >= 0) { finish(b_done); b_done = -1; } // the example completed by the previous chunk
      const float *ap = As + kq * LWG_LD + m_blk0 * 16 + i16, *bp = Bs + kq * LWG_LD + n_blk0 * 16 + i16;
#pragma unroll
      for (int ks = 0; ks < LWG_BK / 4; ++ks) {
        float av[MC], bv[NC];
#pragma unroll
        for (int i = 0; i < MC; ++i) av[i] = ap[ks * 4 * LWG_LD + i * 16];
#pragma unroll
        for (int j = 0; j < NC; ++j) bv[j] = bp[ks * 4 * LWG_LD + j * 16];
#pragma unroll
        for (int i = 0; i < MC; ++i)
#pragma unroll
          for (int j = 0; j < NC; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], bv[j], acc[i][j], 0, 0, 0);
      }
      if (c == n_chunks - 1) b_done = b_cur;
      b_cur = b_next; c = c_next;
    }
    if (b_done >= 0) finish(b_done);
  };
  if (m_cnt == 7) {
    if (n_cnt == 4) run(std::integral_constant<int, 7>{}, std::integral_constant<int, 4>{});
    else run(std::integral_constant<int, 7>{}, std::integral_constant<int, 3>{});
  } else {
    if (n_cnt == 4) run(std::integral_constant<int, 6>{}, std::integral_constant<int, 4>{});
    else run(std::integral_constant<int, 6>{}, std::integral_constant<int, 3>{});
  }
}

// Forward pass of a first convolution layer: 3x3, stride 1, pad 1, at most 3 input channels (an RGB image), at most
// 32 output channels, 32-wide planes (the CIFAR10-shaped networks of Section 3 and Appendix B).  With 27 multiplies
// per output the layer is a memory write: B x 32 x 32 x 32 floats out, a tenth of that in.  A workgroup of the
// generic direct kernel loads, multiplies and stores one tile, one phase after the other, and the workgroups of a
// round march in step, so the stores of the chip never overlap its loads.  Here a PERSISTENT workgroup walks over
// tiles of 8 pixel rows: the next tile's input is requested (buffer loads; positions outside the image read as
// zero) before the current one is multiplied, and nothing waits for the stores, whose number per tile is a constant.
// The weights never move: lane (m, k-half) of a wave keeps W[m][k] for its 14 k-steps of v_mfma_f32_32x32x2_f32
// (K = 27 padded to 28) in registers, read straight from the parameter vector.  Wave w owns pixel rows 2w and 2w+1 of
// the tile (an MFMA block is one row of 32 pixels); B operands are read from the haloed LDS tile at
// [channel][row + kh][column + kw].  Output addresses are a descriptor per image, a scalar offset per accumulator
// register (its output channel) and one lane offset.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_misc.h"

typedef float cf_f32x16 __attribute__((ext_vector_type(16)));

#define CF_W 32
#define CF_TR 8                       // pixel rows per tile
#define CF_LDW (CF_W + 2)
#define CF_PLANE ((CF_TR + 2) * CF_LDW) // 340 staged positions per channel
#define CF_NI 4                       // staged positions per thread: 3 * 340 <= 4 * 256
#define CF_KS 14                      // k-steps of two

struct ConvFirstArgs {
  const float *x;    // [B][Cin][H][32]
  const float *w;    // W[M][Cin][3][3] in the parameter layout
  const float *bias; // [M]
  float *out;        // [B][M][H][32]
  int B, Cin, H, M, act;
  int n_tiles, tiles_per_wg; // tiles = B * H / 8
};

static inline bool conv_first_fits(int Cin, int H, int W, int M, int KH, int KW, int S, int PAD) {
  return Cin >= 1 && Cin <= 3 && W == CF_W && H >= CF_TR && H % CF_TR == 0 && M >= 1 && M <= 32 && KH == 3 && KW == 3 && S == 1 &&
         PAD == 1;
}

// FULL: M = 32, every store unconditional.  ACT: the activation, fixed at compile time -- with a run-time switch
// around every output value the compiler no longer counts the stores between a load and its use and drains all of
// them before the next tile is staged.
template <bool FULL, int ACT>
__global__ __launch_bounds__(256) void conv_first_kernel(const ConvFirstArgs a) {
  __shared__ float Xl[2][CF_NI * 256];
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int H = a.H, HW = H * CF_W, Cin = a.Cin, K = Cin * 9;
  const int t_begin = blockIdx.x * a.tiles_per_wg, t_end = min(a.n_tiles, t_begin + a.tiles_per_wg);
  if (t_begin >= t_end) return;
  const int per = H / CF_TR;
  constexpr unsigned OUTSIDE = 0x80000000u;

  // weights and bias of this lane
  float wr[CF_KS];
#pragma unroll
  for (int ks = 0; ks < CF_KS; ++ks) {
    const int k = 2 * ks + lk;
    const bool ok = li < a.M && k < K;
    const float v = a.w[ok ? li * K + k : 0];
    wr[ks] = ok ? v : 0.f;
  }
  float bias_r[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) bias_r[r] = a.bias[min(8 * (r >> 2) + 4 * lk + (r & 3), a.M - 1)];
  // LDS byte offset of the lane's B operand per k-step: [channel][row + kh][column + kw] for row 2*wave of the tile
  int koff[CF_KS];
#pragma unroll
  for (int ks = 0; ks < CF_KS; ++ks) {
    const int k = min(2 * ks + lk, K - 1), c = k / 9, tap = k - 9 * c, kh = tap / 3, kw = tap - 3 * kh;
    koff[ks] = 4 * (c * CF_PLANE + (2 * wave + kh) * CF_LDW + li + kw);
  }
  // staging items: position p = tid + 256 q of [Cin][10][34]
  unsigned s_off[CF_NI];
  int s_rr[CF_NI];
#pragma unroll
  for (int q = 0; q < CF_NI; ++q) {
    const int p = tid + 256 * q, c = p / CF_PLANE, rem = p - c * CF_PLANE, rr = rem / CF_LDW, col = rem - rr * CF_LDW;
    const bool in = c < Cin && col >= 1 && col <= CF_W;
    s_off[q] = in ? 4u * (unsigned)(c * HW + rr * CF_W + col - 1) : OUTSIDE; // bytes from one pixel row above the tile
    s_rr[q] = rr;
  }
  // output: lane offset inside an image (accumulator register r adds (8 (r / 4) + r % 4) planes through the scalar offset)
  const unsigned o_lane = 4u * (unsigned)(4 * lk * HW + li);

  struct Tile { __amdgpu_buffer_rsrc_t rs; int img, row0; };
  auto setup = [&](int t) {
    Tile q;
    q.img = t / per; q.row0 = (t - q.img * per) * CF_TR;
    const float *base = a.x + (long)q.img * Cin * HW + (q.row0 - 1) * CF_W;
    q.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, 4 * (Cin * HW + CF_W), 0x00020000);
    return q;
  };
  float xr[CF_NI];
  auto fetch = [&](const Tile &q) {
#pragma unroll
    for (int i = 0; i < CF_NI; ++i) {
      const int ih = q.row0 + s_rr[i] - 1;
      const unsigned off = (unsigned)ih < (unsigned)H ? s_off[i] : OUTSIDE;
      xr[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(q.rs, off, 0, 0));
    }
  };

  // The first tile is staged before the loop and every iteration stages the next one AFTER its own stores: the loads
  // it waits for are then always followed by exactly the 32 stores of one tile, on the first pass as on every other,
  // so the wait is for "all but the last 32" and never for the stores themselves.
  Tile cur = setup(t_begin);
  fetch(cur);
#pragma unroll
  for (int i = 0; i < CF_NI; ++i) Xl[0][tid + 256 * i] = xr[i];
  __syncthreads();
  Tile nxt = setup(min(t_begin + 1, t_end - 1)); // (past the run's last tile: it is read again, unused)
  fetch(nxt);
  int buf = 0;
  for (int t = t_begin; t < t_end; ++t) {
    __amdgpu_buffer_rsrc_t ors =
        __builtin_amdgcn_make_buffer_rsrc(a.out + (long)cur.img * a.M * HW, 0, 4 * a.M * HW, 0x00020000);
    const char *xb = reinterpret_cast<const char *>(&Xl[buf][0]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      cf_f32x16 acc;
#pragma unroll
      for (int ks = 0; ks < CF_KS; ++ks) {
        const float bv = *reinterpret_cast<const float *>(xb + koff[ks] + 4 * j * CF_LDW);
        if (ks == 0) {
          const cf_f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[ks], bv, z, 0, 0, 0);
        } else {
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[ks], bv, acc, 0, 0, 0);
        }
      }
      const unsigned o_row = o_lane + 4u * (unsigned)((cur.row0 + 2 * wave + j) * CF_W);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mu = 8 * (r >> 2) + (r & 3); // output channel mu + 4 lk
        const float v = act_apply(ACT, acc[r] + bias_r[r]);
        const unsigned off = (FULL || mu + 4 * lk < a.M) ? o_row : OUTSIDE;
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), ors, off, 4 * mu * HW, 0);
      }
    }
    // the next tile into the other buffer (last read before the previous barrier), then its successor's loads
#pragma unroll
    for (int i = 0; i < CF_NI; ++i) Xl[buf ^ 1][tid + 256 * i] = xr[i];
    __syncthreads();
    cur = nxt;
    nxt = setup(min(t + 2, t_end - 1));
    fetch(nxt);
    buf ^= 1;
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Per-example weight gradient of the same layer (Section 1, item 2a): G_b[d][(c, tap)] = sum over pixels p of
// Delta_b[d][p] x_b[c][p + tap], its squared norm (item 2b: the layer's slot of the example) and, optionally, the
// gradient itself for the weighted sum that forms the clipped sum (item 3), plus the bias gradient sum_p Delta_b[d][p].
// 32 x 27 outputs and 1024 pixels per example: the work is reading Delta (B x 32 x H x 32 floats) once.
// MFMA roles: M = output channel d, N = (channel, tap) index k, K = pixel.  The Delta operand never passes through
// LDS: lane (d, half) loads 16 bytes = four consecutive pixels of row d of the plane straight from memory (lanes of a
// d beyond D are zeroed) and feeds them to four k-steps -- a k-step pairs pixel 8 s + e of the lower
// half-wave with pixel 8 s + 4 + e of the upper, and the x operand, read from the example's zero-haloed image in LDS
// at [c][row + kh][column + kw], follows the same pairing.  A workgroup owns whole examples, one after the other
// (persistent); wave w takes the pixel rows w, w + 4, ... and keeps Delta rows four row-steps ahead in registers (a
// trip to memory is longer than the sixteen multiplies of a row), the next example's image travels meanwhile.  Per
// example the four waves' accumulators meet in LDS and each wave squares, stores and reduces a quarter of them.  The stored row has the
// accumulator order [register][lane] of conv_s1_wgrad_kernel's flattened variant, so either kernel can write it.
#define CFW_LDW 40                          // LDS row length: interior at columns 4 .. 35 (16-byte aligned), halo at 3 and 36
#define CFW_PLANE ((CF_W + 2) * CFW_LDW)    // 34 rows
#define CFW_XI 3                            // float4 items per thread: 3 channels x 32 rows x 8 groups / 256

struct ConvFirstWgArgs {
  const float *x;      // [B][Cin][H][32]
  const float *dy;     // [B][D][H][32]
  float *slots;        // squared norms, one partial per wave: slots[w * slot_stride + b], w = 0 .. 3
  long slot_stride;
  float *gstore;       // [B][gstride] or null
  long gstride, gbias_off;
  int B, Cin, H, D;
  int ex_per_wg;
};

static inline bool conv_first_wgrad_fits(int Cin, int H, int W, int D, int KH, int KW, int S, int PAD) {
  return conv_first_fits(Cin, H, W, D, KH, KW, S, PAD) && H % 16 == 0 && H <= 32;
}

// FULL: D = 32 (no lane of the Delta operand is masked); STORE: the gradients are written out; H_: rows of the plane.
// All three are compile-time so that one example is straight-line code in which every wave issues the same memory
// instructions: the compiler can then wait for "all but the last n" of them, instead of draining the Delta rows in
// flight and the stores whenever it needs the oldest load.
template <bool FULL, bool STORE, int H_>
__global__ __launch_bounds__(256) void conv_first_wgrad_kernel(const ConvFirstWgArgs a) {
  __shared__ __attribute__((aligned(16))) float Xl[2][3 * CFW_PLANE];
  __shared__ float xs[4][16][64];
  __shared__ float bs[4][32];
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int H = H_, HW = H * CF_W, RPW = H / 4; // RPW: pixel rows per wave and example, a multiple of 4
  const int Cin = a.Cin, D = a.D, K = Cin * 9;
  const int b_begin = blockIdx.x * a.ex_per_wg, b_end = min(a.B, b_begin + a.ex_per_wg);
  if (b_begin >= b_end) return;

  for (int i = tid; i < 2 * 3 * CFW_PLANE; i += 256) (&Xl[0][0])[i] = 0.f; // halos stay zero: only interiors are written

  // x operand: byte offset of (c, kh, kw) of this lane's k in the image, plus the upper half-wave's four pixels
  int kbase;
  {
    const int k = min(li, K - 1), c = k / 9, tap = k - 9 * c, kh = tap / 3, kw = tap - 3 * kh;
    kbase = 4 * (c * CFW_PLANE + kh * CFW_LDW + kw + 3 + 4 * lk); // pixel column 0 with kw = 0 is LDS column 3 (the halo)
  }
  // Delta operand: lane byte offset in the example's Delta block (a lane of a d beyond D reads row 0 and is zeroed);
  // every load below is (wave-uniform pointer) + (unsigned lane offset), so its address costs no vector instruction
  const bool d_ok = li < D;
  const unsigned d_lane = 4u * (unsigned)((d_ok ? li : 0) * HW + 4 * lk);
  // x staging: item (c, row, group of four columns)
  unsigned xs_off[CFW_XI];
  int xs_lds[CFW_XI];
#pragma unroll
  for (int q = 0; q < CFW_XI; ++q) {
    const int it = tid + 256 * q, c = it / (H * 8), rem = it - c * (H * 8), row = rem >> 3, g = rem & 7;
    const bool ok = c < Cin;
    xs_off[q] = ok ? 4u * (unsigned)(c * HW + row * CF_W + 4 * g) : 0u;
    xs_lds[q] = ok ? c * CFW_PLANE + (row + 1) * CFW_LDW + 4 + 4 * g : -1;
  }
  static_assert(CFW_XI == 3, "three staged items, held in three named registers (an array of them ended up in scratch memory)");
  float4 xv0, xv1, xv2;
  auto fetch_x = [&](int b) {
    const char *xb = reinterpret_cast<const char *>(a.x + (long)b * Cin * HW);
    xv0 = *reinterpret_cast<const float4 *>(xb + xs_off[0]);
    xv1 = *reinterpret_cast<const float4 *>(xb + xs_off[1]);
    xv2 = *reinterpret_cast<const float4 *>(xb + xs_off[2]);
  };
  // Delta rows in flight: ring of four row-steps, four float4 each (pixels 8 s + 4 lk .. + 3 of the row)
  float4 dr[4][4];
  auto fetch_d = [&](int b, int row, float4 (&dst)[4]) {
    const char *db = reinterpret_cast<const char *>(a.dy + (long)b * D * HW + row * CF_W);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const float4 v = *reinterpret_cast<const float4 *>(db + 32 * s + d_lane);
      dst[s] = FULL ? v : make_float4(d_ok ? v.x : 0.f, d_ok ? v.y : 0.f, d_ok ? v.z : 0.f, d_ok ? v.w : 0.f);
    }
  };
  // row-step t of the run: example b_begin + t / RPW, pixel row wave + 4 (t % RPW); past the run: the last one again
  const int n_steps = (b_end - b_begin) * RPW;
  auto fetch_step = [&](int t, float4 (&dst)[4]) {
    const int tt = min(t, n_steps - 1), e = tt / RPW, j = tt - e * RPW;
    fetch_d(b_begin + e, wave + 4 * j, dst);
  };

  fetch_x(b_begin);
  fetch_step(0, dr[0]); fetch_step(1, dr[1]); fetch_step(2, dr[2]); fetch_step(3, dr[3]);
  __syncthreads(); // the zeros are in place
  int buf = 0, t = 0;
  for (int b = b_begin; b < b_end; ++b) {
    if (xs_lds[0] >= 0) *reinterpret_cast<float4 *>(&Xl[buf][xs_lds[0]]) = xv0;
    if (xs_lds[1] >= 0) *reinterpret_cast<float4 *>(&Xl[buf][xs_lds[1]]) = xv1;
    if (xs_lds[2] >= 0) *reinterpret_cast<float4 *>(&Xl[buf][xs_lds[2]]) = xv2;
    __syncthreads(); // the image is staged (the other buffer was last read before the previous example's second barrier)
    fetch_x(min(b + 1, b_end - 1));
    cf_f32x16 acc;
    float bsum = 0.f;
    const char *xb = reinterpret_cast<const char *>(&Xl[buf][0]) + kbase;
#pragma unroll
    for (int j0 = 0; j0 < RPW; j0 += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const char *xrow = xb + 4 * (wave + 4 * (j0 + u)) * CFW_LDW;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const float dv[4] = {dr[u][s].x, dr[u][s].y, dr[u][s].z, dr[u][s].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float bv = *reinterpret_cast<const float *>(xrow + 4 * (8 * s + e));
            if (j0 == 0 && u == 0 && s == 0 && e == 0) {
              const cf_f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
              acc = __builtin_amdgcn_mfma_f32_32x32x2f32(dv[e], bv, z, 0, 0, 0);
            } else {
              acc = __builtin_amdgcn_mfma_f32_32x32x2f32(dv[e], bv, acc, 0, 0, 0);
            }
            bsum += dv[e];
          }
        }
        fetch_step(t + 4, dr[u]);
        ++t;
      }
    }
    // ---- the example is complete: the four waves' accumulators and bias sums meet in LDS; wave w finishes registers
    // 4 w .. 4 w + 3 (and eight of the bias gradients), with stores that every lane of every wave executes
    bsum += __shfl_xor(bsum, 32, 64);
    if (lk == 0) bs[wave][li] = bsum;
#pragma unroll
    for (int r = 0; r < 16; ++r) xs[wave][r][lane] = acc[r];
    __syncthreads();
    {
      float *gb = STORE ? a.gstore + (long)b * a.gstride : nullptr;
      float part = 0.f;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * wave + rr;
        float v = (xs[0][r][lane] + xs[1][r][lane]) + (xs[2][r][lane] + xs[3][r][lane]);
        v = li < K ? v : 0.f; // lanes past the last (channel, tap) pair multiplied a duplicate of it
        part = fmaf(v, v, part);
        if (STORE) gb[r * 64 + lane] = v;
      }
      {
        // bias gradient d = 8 w + lane % 8 (every lane of the wave takes part: lanes with the same d store the same word)
        const int d = 8 * wave + (lane & 7), dc = min(d, D - 1);
        const float bd = (bs[0][dc] + bs[1][dc]) + (bs[2][dc] + bs[3][dc]);
        part = (lane < 8 && d < D) ? fmaf(bd, bd, part) : part;
        if (STORE) gb[a.gbias_off + dc] = bd;
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
      a.slots[(long)wave * a.slot_stride + b] = part; // one slot per wave; the clip factor adds them in a fixed order
    }
    buf ^= 1;
  }
}

// Stride-1 convolution kernels with the input tile staged once in LDS ("LDS-staged
// im2col"): the MFMA operands are read straight from the staged image tile with a
// per-tap offset, so no im2col matrix exists anywhere and a pixel is fetched from
// HBM/L2 about 1.5 times instead of KH*KW times.
//
//   conv_s1_kernel        forward  (bias + activation epilogue) and backward-data
//                         (the same correlation with transposed, flipped weights and
//                         an activation-derivative epilogue)
//   conv_s1_wgrad_kernel  weight gradient  G[d, c, tap] = sum_p Delta[d, p] x[c, p + tap]
//                         per example with its squares reduced to the per-example norm
//                         (never written), or summed over a range of examples with the
//                         clip factor applied to Delta while staging (split partial of
//                         the clipped sum, DPSGD item 3).
//
// MFMA mapping (v_mfma_f32_32x32x2_f32): forward  M = output channel, N = pixel,
// K = input-channel pair for one tap;  wgrad  M = output channel d, N = input channel c
// for one tap, K = pixel pair.  Lanes of the B operand walk pixels (forward) or
// channels with an odd plane stride (wgrad), lanes of the A operand walk channels:
// all LDS operand reads are conflict-free 4-byte reads with uniform offsets.
#pragma once
#include <type_traits>
#include "gemm_tile.h"
#include "kernels_misc.h"

struct ConvTile {
  int TR, NIMG;       // tile = NIMG images x TR output rows x OW columns
  int row_tiles;      // ceil(OH / TR)            (1 when NIMG > 1)
  int LDW, IMGPL;     // staged row length OW+KW-1; floats per staged image = (TR+KH-1)*LDW
  int XPLANE;         // floats per staged channel (>= NIMG*IMGPL)
  FastDiv dOW, dTROW, dLDW, dIMGPL, dXPLANE, dRT;
};

struct ConvS1Args {
  const float *x;      // input  [B, Cin, H, W]
  const float *wt;     // weights laid out [Cin][KK][Mpad], Mpad = M rounded up to 4, pad columns zero
  const float *bias;   // forward: bias[M]; backward-data: null
  const float *a_prev; // backward-data: output of the activation whose derivative multiplies the result
  float *out;          // [B, M, OH, OW]
  int B, Cin, H, W, M, Mpad, OH, OW, pad;
  int act;
  ConvTile t;
};

// Re-lays a conv weight W[D][C][KK] for the two correlations that use it:
//   wt_f[(c*KK + tap)*Dp + d] = W[d][c][tap]            forward       (M = D, Cin = C)
//   wt_b[(d*KK + tap)*Cp + c] = W[d][c][KK-1-tap]       backward-data (M = C, Cin = D)
// (Dp, Cp = D, C rounded up to 4; the pad columns stay zero from the allocation) so that a
// chunk of input channels is copied into LDS with aligned 16-byte loads in the order the
// MFMA A operand reads it.
// One launch covers every such layer of the model: blockIdx.y = layer, the x grid is sized for the largest one.
#define CONV_LAYOUT_MAX 16
struct ConvLayoutArgs {
  int n;
  struct { long w_off; float *wt_f, *wt_b; int D, C, Dp, Cp; } l[CONV_LAYOUT_MAX];
};
__device__ __forceinline__ void conv_weight_layout_body(const float *__restrict__ params, const ConvLayoutArgs &a, int layer) {
  constexpr int KK = 9;
  const auto &L = a.l[layer];
  const int total = L.D * L.C * KK;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const int d = i / (L.C * KK), r = i - d * L.C * KK;
    const int c = r / KK, tap = r - c * KK;
    const float v = params[L.w_off + i];
    if (L.wt_f) L.wt_f[((long)c * KK + tap) * L.Dp + d] = v; // (null: that correlation runs on another kernel)
    if (L.wt_b) L.wt_b[((long)d * KK + (KK - 1 - tap)) * L.Cp + c] = v;
  }
}
__global__ void conv_weight_layout_kernel(const float *__restrict__ params, const ConvLayoutArgs a) {
  conv_weight_layout_body(params, a, blockIdx.y);
}

#define CONV_XPLANE_MAX 448 // staged floats per channel: a thread stages at most CC*448/256 elements per chunk
#define CONV_CC 8           // input channels staged per chunk

// CC = input channels staged per chunk (8 or 16): a longer chunk amortises the two barriers
// and gives the prefetch of the next chunk more multiply time to hide behind.
// While another wave of the SIMD streams MFMAs, every other instruction of this kernel takes about
// one MFMA slot to issue, so the phases around the K loop are written for instruction count: global
// addresses are a wave-uniform pointer (scalar arithmetic) plus a 32-bit lane offset fixed for the
// tile, validity is folded into that offset (an invalid item reads a valid address and is zeroed when
// staged), the re-laid weights are padded so that no weight load needs a test, and the epilogue uses
// one pointer per output row with a lane offset per pixel.
// (the waves-per-SIMD ceiling keeps the compiler from spilling the prefetched tiles to reach a higher occupancy)
template <int KH, int KW, int DT, int NPW, int CC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((DT * NPW <= 32 * 64 ? 4 : 1), (DT * NPW <= 32 * 64 ? 4 : 2))))
void conv_s1_kernel(const ConvS1Args a) {
  constexpr int KK = KH * KW, DB = DT / 32, PB = NPW / 32;
  constexpr int XP = (CONV_XPLANE_MAX + 255) / 256; // staged positions per thread within a channel plane
  constexpr int WROWS = CC * KK;                     // weight rows per chunk
  constexpr int WV = (WROWS * DT / 4 + 255) / 256;   // float4 weight registers per thread
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float *Wl = smem;                 // [WROWS][DT]
  float *Xl = smem + WROWS * DT;    // [CC][XPLANE]
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = blockIdx.y * DT;
  // tile -> first image and first row
  int b0, r0;
  if (a.t.NIMG > 1) { b0 = blockIdx.x * a.t.NIMG; r0 = 0; }
  else { b0 = (int)a.t.dRT.div(blockIdx.x); r0 = (blockIdx.x - b0 * a.t.row_tiles) * a.t.TR; }
  const int HW = a.H * a.W, OHW = a.OH * a.OW;

  // this lane's pixels (one per 32-pixel block of the wave)
  int xoff[PB];
  unsigned ooff[PB]; // lane byte offset of the pixel in out relative to the tile's first image / row, row 4*lk of a block
  bool pix_ok[PB];
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    const int lp = wave * NPW + pb * 32 + li;
    const int img = (int)a.t.dTROW.div(lp), rem = lp - img * a.t.TR * a.OW;
    const int r = (int)a.t.dOW.div(rem), col = rem - r * a.OW;
    const bool ok = img < a.t.NIMG && (b0 + img) < a.B && (r0 + r) < a.OH;
    pix_ok[pb] = ok;
    xoff[pb] = (ok ? img * a.t.IMGPL + r * a.t.LDW + col : 0) + lk * a.t.XPLANE;
    ooff[pb] = ok ? 4u * (unsigned)((img * a.M + 4 * lk) * OHW + r * a.OW + col) : 0u; // bytes
  }
  // staged input: a thread owns up to XP positions of the channel plane (img, rr, cc) and stages them for every
  // channel of the chunk.  xg = lane offset in x relative to xtile (below); positions that hold no input (halo,
  // outside the batch, past the plane) point at element (0, 0) of the channel and are zeroed when staged.
  unsigned xg[XP];
  bool xv[XP];
#pragma unroll
  for (int j = 0; j < XP; ++j) {
    const int pos = tid + j * 256;
    const int img = (int)a.t.dIMGPL.div(pos), rem2 = pos - img * a.t.IMGPL;
    const int rr = (int)a.t.dLDW.div(rem2), cc = rem2 - rr * a.t.LDW;
    const int ih = r0 + rr - a.pad, iw = cc - a.pad;
    xv[j] = pos < a.t.XPLANE && img < a.t.NIMG && (b0 + img) < a.B && (unsigned)ih < (unsigned)a.H &&
            (unsigned)iw < (unsigned)a.W;
    xg[j] = xv[j] ? 4u * (unsigned)(img * a.Cin * HW + ih * a.W + iw) : 0u; // bytes
  }
  const float *xtile = a.x + (long)b0 * a.Cin * HW; // channel 0 of the tile's first image
  // weight items: float4 q = tid + j*256 covers row q / (DT/4), columns 4*(q % (DT/4)) ..+3 (rows past the
  // chunk and columns past Mpad read the zero padding of the re-laid weights or finite values nobody uses)
  unsigned wg[WV];
#pragma unroll
  for (int j = 0; j < WV; ++j) {
    const int q = tid + j * 256;
    const int row = q / (DT / 4);
    wg[j] = 4u * (unsigned)(row * a.Mpad + 4 * (q - row * (DT / 4))); // bytes
  }

  f32x16 acc[DB][PB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int j = 0; j < PB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float xr[XP][CC];
  float4 wr[WV];
  auto prefetch = [&](int c0) {
#pragma unroll
    for (int c = 0; c < CC; ++c) {
      const float *xc = xtile + (long)min(c0 + c, a.Cin - 1) * HW; // a channel past Cin re-reads the last one
#pragma unroll
      for (int j = 0; j < XP; ++j) xr[j][c] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(xc) + xg[j]);
    }
    const float *wc = a.wt + ((long)c0 * KK * a.Mpad + m0);
#pragma unroll
    for (int j = 0; j < WV; ++j) {
      const float4 v = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(wc) + wg[j]);
      wr[j] = make_float4(v.x, v.y, v.z, v.w);
    }
  };

  prefetch(0);
  for (int c0 = 0; c0 < a.Cin; c0 += CC) {
    __syncthreads(); // the previous chunk has been consumed
#pragma unroll
    for (int j = 0; j < XP; ++j) {
      const int pos = tid + j * 256;
      if (pos < a.t.XPLANE)
#pragma unroll
        for (int c = 0; c < CC; ++c) Xl[c * a.t.XPLANE + pos] = (xv[j] && c0 + c < a.Cin) ? xr[j][c] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < WV; ++j) {
      const int q = tid + j * 256;
      if (q < WROWS * DT / 4) *reinterpret_cast<float4 *>(&Wl[4 * q]) = wr[j];
    }
    __syncthreads();
    if (c0 + CC < a.Cin) prefetch(c0 + CC); // in flight while this chunk is multiplied
    // (channel pair, tap) steps; the LDS operands of step s+1 are read before the MFMAs of step s
    {
      constexpr int NS = (CC / 2) * KK;
      float av[2][DB], bv[2][PB];
      auto ld = [&](int s, float *pa, float *pb) {
        const int cp = s / KK, tap = s - cp * KK, kh = tap / KW, kw = tap - kh * KW;
        const int wrow = ((2 * cp + lk) * KK + tap) * DT;
#pragma unroll
        for (int i = 0; i < DB; ++i) pa[i] = Wl[wrow + i * 32 + li];
        const int xo = 2 * cp * a.t.XPLANE + kh * a.t.LDW + kw;
#pragma unroll
        for (int j = 0; j < PB; ++j) pb[j] = Xl[xoff[j] + xo];
      };
      ld(0, av[0], bv[0]);
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        if (s + 1 < NS) ld(s + 1, av[(s + 1) & 1], bv[(s + 1) & 1]);
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
          for (int j = 0; j < PB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s & 1][i], bv[s & 1][j], acc[i][j], 0, 0, 0);
      }
    }
  }

  // epilogue: bias + activation (forward) or the derivative of the producing activation (backward-data).
  // Output row m = m0 + 32*i + 8*(r/4) + 4*lk + r%4 of pixel j lives at
  //   (uniform pointer of row m0 + 32*i + 8*(r/4) + r%4 of the tile's first image) + ooff[j].
  const bool fwd = a.bias != nullptr;
  const long tile_off = (long)b0 * a.M * OHW + (long)r0 * a.OW;
  const int mrem = a.M - m0 - 4 * lk; // rows i*32 + 8*(r/4) + r%4 below mrem exist for this lane
#pragma unroll
  for (int i = 0; i < DB; ++i) {
    float bias_v[16]; // forward: the bias of the lane's 16 rows (backward-data loads x[0..] here and ignores it)
    {
      const float *bsrc = fwd ? a.bias : a.x;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mu = i * 32 + 8 * (r >> 2) + (r & 3);
        bias_v[r] = bsrc[fwd ? min(m0 + mu + 4 * lk, a.M - 1) : 0];
      }
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {
      if (!pix_ok[j]) continue;
      const float *side = (fwd || !a.act) ? a.x : a.a_prev; // backward-data: the producing activation's output
      float sv[16];
      const bool need_side = !fwd && a.act;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mu = i * 32 + 8 * (r >> 2) + (r & 3);
        // (a row past M is not read: the pointer stays on the last real row and the lane offset is dropped)
        const float *row = need_side ? side + (tile_off + (long)(m0 + min(mu, a.M - 1 - m0)) * OHW) : a.x;
        sv[r] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(row) + ((need_side && mu < mrem) ? ooff[j] : 0u));
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mu = i * 32 + 8 * (r >> 2) + (r & 3);
        float v = acc[i][j][r];
        if (fwd) v = act_apply(a.act, v + bias_v[r]);
        else if (a.act) v *= act_deriv_from_out(a.act, sv[r]);
        float *row = a.out + (tile_off + (long)(m0 + mu) * OHW);
        if (mu < mrem) *reinterpret_cast<float *>(reinterpret_cast<char *>(row) + ooff[j]) = v;
      }
    }
  }
}

// ---------------------------------------------------------------- weight gradient

struct ConvWgArgs {
  const float *x;     // layer input [B, C, H, W]
  const float *delta; // [B, D, OH, OW]
  const float *scale; // clip factors s[b]; always valid (a vector of ones when nothing is clipped)
  float *out;         // norm mode: slots base; clipped mode: partials base
  int B, C, H, W, D, OH, OW, pad; // D: the output channels this launch covers (at most 128, a slice of the layer's)
  int Dstride;        // output channels of the whole layer: Delta's per-example stride is Dstride*OH*OW
  long bias_off;      // clipped mode: the slice's bias gradients go to part[bias_off + d]
  int mode;           // 0: per-example squared norm; 1: sum over the block's examples
  int ex_per_block;   // clipped mode
  int PCH, LDP;       // pixels per K-chunk (= NIMG*TR*OW) and padded (odd) row length of the staged Delta
  int WQ, ROWS;       // W/4 float4 groups per input row; staged rows per image = TR + KH - 1
  FastDiv dWQ, dROWS, dNIMG, dPQ; // item decoding (PQ = PCH/4)
  long slot_stride; int slot0; // norm: slots[(slot0 + cblock)*slot_stride + b]
  long part_stride;   // clipped: part[split*part_stride + (d*C + c)*KK + tap]
  float *gstore;      // norm mode, optional (null: norms only): example b's gradient goes to gstore[b*gstride + ...]
  long gstride;       // in accumulator order, [channel block][wave group][tap slot][16 registers][64 lanes], so
  long gbias_off;     // that every store instruction writes 256 consecutive bytes; the bias follows at gbias_off
  ConvTile t;         // XPLANE odd
};

#define CONV_WG_XV 7  // float4 input items per thread and chunk: 32*NIMG*ROWS*W/4 <= 7*256

// DB = number of 32-row blocks of output channels (D <= 32*DB); the block owns one
// group of 32 input channels; the KH*KW taps are its N blocks.  W and OW must be
// multiples of 4: rows are moved as float4 items.  The items of the next K-chunk
// are fetched into registers while the current chunk is multiplied.
// FLATC (first layers, C*KH*KW <= 32, DB == 1): the single N block holds the flattened
// (channel, tap) pairs, one per lane, and the four waves split the pixel pairs instead;
// their accumulators are summed through LDS at the end.
// CLIP: the clipped-sum mode (a.mode == 1); the norm mode never touches the clip factors.
template <int KH, int KW, int DB, bool FLATC, bool CLIP>
__global__ __launch_bounds__(256, (DB <= 2 ? 2 : 1)) void conv_s1_wgrad_kernel(const ConvWgArgs a) {
  constexpr int KK = KH * KW;
  // the four waves: WD along output-channel blocks, WN along taps, WK interleaved over pixel pairs
  // (waves that share (wd, wn) see disjoint pixel pairs; their accumulators are summed through LDS)
  constexpr int WD = FLATC ? 1 : (DB >= 4 ? 4 : DB);
  constexpr int WN = FLATC ? 1 : (DB >= 4 ? 1 : 2);
  constexpr int WK = 4 / (WD * WN);
  constexpr int DBW = DB / WD, NBW = FLATC ? 1 : (KK + WN - 1) / WN;
  static_assert(WD * WN * WK == 4 && DBW == 1, "wave decomposition");
  constexpr int DT = 32 * DB;
  constexpr int XV = CONV_WG_XV;
  constexpr int DV = (DB == 1 && !FLATC) ? 4 : 8;   // float4 Delta items per thread: DT*PCH/4 <= DV*256
  constexpr int NSL = 256 / DT;                     // row-sum slices
  static_assert(!FLATC || DB == 1, "flattened (channel, tap) block needs D <= 32");
  extern __shared__ float smem[];
  const int xch = FLATC ? a.C : 32;     // staged input channels
  float *Xl = smem;                     // [xch][XPLANE]
  float *Dl = smem + xch * a.t.XPLANE;  // [DT][LDP]
  __shared__ float red[4];
  __shared__ float rsum[256];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), li = lane & 31, lk = lane >> 5;
  const int wd = wave / (WN * WK), wn = (wave / WK) % WN, wk = wave % WK;
  const int cb = blockIdx.x, c0 = cb * 32;
  const int HW = a.H * a.W, OHW = a.OH * a.OW;
  // examples bbeg .. bend-1 belong to this block: summed into one partial (CLIP), or one after the
  // other with a squared-norm epilogue each, the next example's data in flight meanwhile (norm mode)
  const int bbeg = blockIdx.y * a.ex_per_block, bend = min(a.B, bbeg + a.ex_per_block);
  const int nimg_max = !CLIP ? 1 : a.t.NIMG;

  // zero the staged input once: the left / right halo columns are never written again
  for (int e = tid; e < xch * a.t.XPLANE; e += 256) Xl[e] = 0.f;

  // static item descriptors.  Input item it = ((c*NIMG + img)*ROWS + rr)*WQ + q
  int x_lds[XV], x_goff[XV], x_ir[XV];
#pragma unroll
  for (int j = 0; j < XV; ++j) {
    const int it = tid + j * 256;
    const int t1 = (int)a.dWQ.div(it), q = it - t1 * a.WQ;
    const int t2 = (int)a.dROWS.div(t1), rr = t1 - t2 * a.ROWS;
    const int c = (int)a.dNIMG.div(t2), img = t2 - c * a.t.NIMG;
    const bool ok = c < xch && c0 + c < a.C;
    x_lds[j] = ok ? c * a.t.XPLANE + img * a.t.IMGPL + rr * a.t.LDW + a.pad + 4 * q : -1;
    x_goff[j] = (img * a.C + c) * HW + (rr - a.pad) * a.W + 4 * q;
    x_ir[j] = (img << 16) | rr;
  }
  // Delta item it = d*PQ + p4: pixels 4*p4..4*p4+3 of the chunk (same output row)
  const int PQ = a.PCH >> 2;
  int d_lds[DV], d_goff[DV], d_ir[DV];
#pragma unroll
  for (int j = 0; j < DV; ++j) {
    const int it = tid + j * 256;
    const int d = (int)a.dPQ.div(it), p = 4 * (it - d * PQ);
    const int img = (int)a.t.dTROW.div(p), rem = p - img * a.t.TR * a.OW;
    const int r = (int)a.t.dOW.div(rem);
    const bool ok = d < DT;
    d_lds[j] = ok ? d * a.LDP + p : -1;
    d_goff[j] = (d < a.D) ? (img * a.Dstride + d) * OHW + rem : -1;
    d_ir[j] = (img << 16) | r;
  }

  f32x16 acc[DBW][NBW];
#pragma unroll
  for (int i = 0; i < DBW; ++i)
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  float rowsum = 0.f; // partial sum_p Delta[d, p] of row tid % DT over this thread's slice (bias gradient)

  int xlane = li * a.t.XPLANE + lk;
  const int dlane = li * a.LDP + lk;
  int tapoff[NBW];
  bool tapok[NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    const int tap = wn * NBW + j;
    const int kh = tap / KW, kw = tap - kh * KW;
    tapok[j] = tap < KK;
    tapoff[j] = tapok[j] ? kh * a.t.LDW + kw : 0;
  }
  if (FLATC) { // lane = (channel, tap)
    const int ch = li / KK, tap = li - ch * KK, kh = tap / KW, kw = tap - kh * KW;
    tapok[0] = li < a.C * KK;
    tapoff[0] = 0;
    xlane = (tapok[0] ? ch * a.t.XPLANE + kh * a.t.LDW + kw : 0) + lk;
  }
  const int col0 = 2 * wk;
  constexpr int colstep = 2 * WK;

  float4 xr[XV], dr[DV];
  float dsv[DV];        // clip factor of each Delta item (CLIP), applied when the item is written to LDS
  unsigned xok = 0, dok = 0; // validity bits of the fetched items: nothing touches a loaded register before the stash
  auto prefetch = [&](int b, int nimg, int r0, int rows) {
    const long xb = ((long)b * a.C + c0) * HW + (long)r0 * a.W;
    // unconditional loads with a safe address for invalid items (see conv_s1_kernel)
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      const int img = x_ir[j] >> 16, rr = x_ir[j] & 0xffff;
      const int ih = r0 + rr - a.pad;
      const bool ok = x_lds[j] >= 0 && img < nimg && rr < rows + KH - 1 && (unsigned)ih < (unsigned)a.H;
      xr[j] = *reinterpret_cast<const float4 *>(a.x + (ok ? xb + x_goff[j] : 0));
      xok = ok ? (xok | (1u << j)) : (xok & ~(1u << j));
    }
    const long db_ = (long)b * a.Dstride * OHW + (long)r0 * a.OW;
#pragma unroll
    for (int j = 0; j < DV; ++j) {
      const int img = d_ir[j] >> 16, r = d_ir[j] & 0xffff;
      const bool ok = d_goff[j] >= 0 && img < nimg && r < rows;
      dr[j] = *reinterpret_cast<const float4 *>(a.delta + (ok ? db_ + d_goff[j] : 0));
      if (CLIP) dsv[j] = a.scale[ok ? b + img : 0];
      dok = ok ? (dok | (1u << j)) : (dok & ~(1u << j));
    }
  };

  // bias gradient of the examples summed so far: combine the slices
  auto bias_total = [&]() {
    float bias_d = 0.f;
    if (cb == 0) {
      rsum[tid] = rowsum;
      __syncthreads();
      if (tid < DT) {
#pragma unroll
        for (int s = 0; s < NSL; ++s) bias_d += rsum[s * DT + tid];
      }
    }
    return bias_d;
  };
  // sum the accumulators of the waves that split the pixel pairs into the wk == 0 wave (the others end at zero)
  auto wave_total = [&]() {
    if (WK > 1) {
      __syncthreads(); // staging area no longer read
      float *xs = smem; // [(WD*WN) groups][WK-1][NBW*16][64], reusing the staging area
      const int grp = wave / WK;
      if (wk > 0)
#pragma unroll
        for (int j = 0; j < NBW; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            xs[(((grp * (WK - 1) + wk - 1) * NBW + j) * 16 + r) * 64 + lane] = acc[0][j][r];
      __syncthreads();
#pragma unroll
      for (int j = 0; j < NBW; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (wk == 0) {
#pragma unroll
            for (int q = 0; q < WK - 1; ++q) acc[0][j][r] += xs[(((grp * (WK - 1) + q) * NBW + j) * 16 + r) * 64 + lane];
          } else acc[0][j][r] = 0.f;
        }
        __builtin_amdgcn_sched_barrier(0); // one block of 16 loads in flight at a time (register pressure)
      }
    }
  };
  // accumulator: lane column = input channel c0 + li (FLATC: flattened channel*KK + tap); rows = output channels
  const int c = c0 + li;
  // norm mode, end of example b: squared norm of this block's share into its slot, accumulators back to zero.
  // Waves that split the pixel pairs (WK > 1) hand their accumulators to the wk == 0 wave through the
  // staging area; that wave squares the sums as it reads them.
  auto norm_epilogue = [&](int b) {
    const float bias_d = bias_total();
    const float *xs = smem; // [(WD*WN) groups][WK-1][NBW*16][64]
    const int grp = wave / WK;
    if (WK > 1) {
      __syncthreads(); // staging area no longer read
      if (wk > 0) {
        float *dst = smem + ((grp * (WK - 1) + wk - 1) * NBW * 16) * 64 + lane;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[(j * 16 + r) * 64] = acc[0][j][r];
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __syncthreads();
    }
    float part = 0.f;
    if (wk == 0 && a.gstore != nullptr) {
      // the same sums, also written out as example b's gradient.  Taps innermost: the words one lane stores are
      // consecutive, so whole cache lines fill within a few instructions.
      float *gb = a.gstore + (long)b * a.gstride;
      if (cb == 0 && tid < a.D) gb[a.gbias_off + tid] = bias_d;
      // accumulator order: no range tests (slots outside the real ranges hold exact zeros) and no address that
      // depends on more than the lane
      float *gw = gb + ((long)(cb * (WD * WN) + grp) * NBW * 16) * 64 + lane;
#pragma unroll
      for (int j = 0; j < NBW; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = acc[0][j][r];
#pragma unroll
          for (int q = 0; q < WK - 1; ++q) v += xs[(((grp * (WK - 1) + q) * NBW + j) * 16 + r) * 64 + lane];
          part += v * v;
          gw[(j * 16 + r) * 64] = v;
        }
        if (WK > 1) __builtin_amdgcn_sched_barrier(0); // one block of 16 loads in flight at a time (register pressure)
      }
    } else if (wk == 0) {
      const int CKK = a.C * KK;
#pragma unroll
      for (int i = 0; i < DBW; ++i)
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
          const int tap = wn * NBW + j;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int d = (wd * DBW + i) * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
            float v = acc[i][j][r];
#pragma unroll
            for (int q = 0; q < WK - 1; ++q) v += xs[(((grp * (WK - 1) + q) * NBW + j) * 16 + r) * 64 + lane];
            // entries outside the real (d, c, tap) range are exact zeros (zero-filled operands, skipped
            // tap slots), so every accumulator is squared without a range test
            part += v * v;
          }
          if (WK > 1) __builtin_amdgcn_sched_barrier(0); // one block of 16 loads in flight at a time (register pressure)
        }
    }
    if (cb == 0 && tid < a.D) part += bias_d * bias_d;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
    if (lane == 0) red[wave] = part;
    __syncthreads();
    // red[] is next written after two more barriers (top of the chunk loop), so this read cannot race
    if (tid == 0) a.out[(long)(a.slot0 + cb) * a.slot_stride + b] = red[0] + red[1] + red[2] + red[3];
#pragma unroll
    for (int i = 0; i < DBW; ++i)
#pragma unroll
      for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    rowsum = 0.f;
    if (WK > 1) {
      // the cross-wave area lies over the staged input: put the zeros back into the halo columns, which the
      // staging of the next example does not write (every read of the area is behind the barrier above, and
      // the next reads of the input are two barriers away)
      const int halo = a.t.LDW - a.W, rows_l = xch * a.t.NIMG * a.ROWS; // halo = 2*pad cells per staged row
      for (int e = tid; e < rows_l * halo; e += 256) {
        const int rowi = e / halo, h = e - rowi * halo;
        const int cimg = rowi / a.ROWS, rr = rowi - cimg * a.ROWS;
        const int ch = cimg / a.t.NIMG, img = cimg - ch * a.t.NIMG;
        Xl[ch * a.t.XPLANE + img * a.t.IMGPL + rr * a.t.LDW + (h < a.pad ? h : a.W + h)] = 0.f;
      }
    }
  };

  const int n_chunks = ((bend - bbeg + nimg_max - 1) / nimg_max) * a.t.row_tiles;
  int cb_b = bbeg, cb_rt = 0; // chunk being fetched
  if (n_chunks > 0) prefetch(cb_b, min(nimg_max, bend - cb_b), 0, min(a.t.TR, a.OH));
  for (int ci = 0; ci < n_chunks; ++ci) {
    const int b = cb_b, r0 = cb_rt * a.t.TR;
    const int nimg = min(nimg_max, bend - b), rows = min(a.t.TR, a.OH - r0);
    __syncthreads(); // previous chunk consumed
#pragma unroll
    for (int j = 0; j < XV; ++j)
      if (x_lds[j] >= 0) {
        const float4 v = ((xok >> j) & 1u) ? xr[j] : f4zero();
        float *d = Xl + x_lds[j];
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
      }
#pragma unroll
    for (int j = 0; j < DV; ++j)
      if (d_lds[j] >= 0) {
        const float sv = ((dok >> j) & 1u) ? (CLIP ? dsv[j] : 1.f) : 0.f;
        const float4 v = ((dok >> j) & 1u) ? dr[j] : f4zero();
        float *d = Dl + d_lds[j];
        d[0] = v.x * sv; d[1] = v.y * sv; d[2] = v.z * sv; d[3] = v.w * sv;
      }
    __syncthreads();
    // advance to the next chunk and start fetching it
    if (++cb_rt == a.t.row_tiles) { cb_rt = 0; cb_b += nimg_max; }
    if (ci + 1 < n_chunks) {
      const int r0n = cb_rt * a.t.TR;
      prefetch(cb_b, min(nimg_max, bend - cb_b), r0n, min(a.t.TR, a.OH - r0n));
    }
    if (cb == 0) { // bias gradient: row sums of the staged Delta, NSL slices per row
      const int d = tid % DT, sl = tid / DT;
      const int per = (a.PCH + NSL - 1) / NSL;
      const int p1 = min(a.PCH, (sl + 1) * per);
      // four independent partial sums: the LDS reads of a slice are issued together, not one per add
      const float *row = Dl + d * a.LDP;
      float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
      int p = sl * per;
      for (; p + 4 <= p1; p += 4) { s0 += row[p]; s1 += row[p + 1]; s2 += row[p + 2]; s3 += row[p + 3]; }
      for (; p < p1; ++p) s0 += row[p];
      rowsum += (s0 + s1) + (s2 + s3);
    }
    // K loop: one step = one pixel pair of the chunk (OW is even: a pair never straddles a row); this wave
    // takes the pairs at columns col0, col0 + colstep, ... of every row, in groups of four steps.  Inside a
    // group the operand addresses are immediate offsets from one pointer per operand (six address adds per
    // group instead of per step), the LDS reads of step s+1 are issued before the MFMAs of step s, and the
    // only branches are the wave-uniform skips of steps past the row's end and of an empty last tap slot.
    // All loop state is wave-uniform (scalar).
    {
      const int d_skip = (a.t.TR - rows) * a.OW, x_skip = a.t.IMGPL - rows * a.t.LDW; // to the next image
      const int spr = (a.OW - col0 + colstep - 1) / colstep; // steps per row
      const int gpr = (spr + 3) >> 2;                        // groups per row
      const int ngroups = nimg * rows * gpr;
      const int back = 4 * colstep * (gpr - 1);              // from a row's last group back to its first column
      const bool last_ok = FLATC || tapok[NBW - 1];
      const float *dp = Dl + dlane + (wd * 32) * a.LDP + col0;
      const float *xp[NBW];
#pragma unroll
      for (int j = 0; j < NBW; ++j) xp[j] = Xl + xlane + col0 + tapoff[j];
      float av[2], bv[2][NBW];
      av[0] = dp[0];
#pragma unroll
      for (int j = 0; j < NBW; ++j) bv[0][j] = xp[j][0];
      int gi = 0, r = 0;
      for (int g = 0; g < ngroups; ++g) {
        const int nv = spr - 4 * gi; // steps of this group inside the row (>= 4: all)
        // pointers of the next group (the last group re-reads its own first step: in bounds, unused)
        int dd = 4 * colstep, dx = 4 * colstep;
        if (++gi == gpr) {
          gi = 0; dd = a.OW - back; dx = a.t.LDW - back;
          if (++r == rows) { r = 0; dd += d_skip; dx += x_skip; }
        }
        if (g + 1 == ngroups) { dd = 0; dx = 0; }
        const float *dpn = dp + dd;
        const float *xpn[NBW];
#pragma unroll
        for (int j = 0; j < NBW; ++j) xpn[j] = xp[j] + dx;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int cur = u & 1, nxt = cur ^ 1;
          if (u < 3) {
            av[nxt] = dp[(u + 1) * colstep];
#pragma unroll
            for (int j = 0; j < NBW; ++j) bv[nxt][j] = xp[j][(u + 1) * colstep];
          } else {
            av[nxt] = dpn[0];
#pragma unroll
            for (int j = 0; j < NBW; ++j) bv[nxt][j] = xpn[j][0];
          }
          if (u < nv) {
            if (FLATC && !tapok[0]) bv[cur][0] = 0.f; // lanes beyond the C*KK flattened columns
#pragma unroll
            for (int j = 0; j + 1 < NBW; ++j)
              acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur], bv[cur][j], acc[0][j], 0, 0, 0);
            if (last_ok) // the last tap slot of the last wave may be empty
              acc[0][NBW - 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur], bv[cur][NBW - 1], acc[0][NBW - 1], 0, 0, 0);
          }
        }
        dp = dpn;
#pragma unroll
        for (int j = 0; j < NBW; ++j) xp[j] = xpn[j];
      }
    }
    if (!CLIP && r0 + rows >= a.OH) norm_epilogue(b); // last row tile of example b (one image per chunk)
  }

  if (!CLIP) return; // every example already went through norm_epilogue
  const float bias_d = bias_total();
  wave_total();
  float *part = a.out + (long)blockIdx.y * a.part_stride;
  if (FLATC) {
    const int CKK = a.C * KK;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int d = 8 * (r >> 2) + 4 * lk + (r & 3);
      if (wk == 0 && li < CKK && d < a.D) part[(long)d * CKK + li] = acc[0][0][r];
    }
    if (tid < a.D) part[a.bias_off + tid] = bias_d;
    return;
  }
  // taps innermost: the stores of one (row, lane) are consecutive words, so the 32 lanes fill whole
  // cache lines within a few instructions and the L2 merges them before it writes them back
#pragma unroll
  for (int i = 0; i < DBW; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int d = (wd * DBW + i) * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
      float *row = part + ((long)d * a.C + c) * KK + wn * NBW;
#pragma unroll
      for (int j = 0; j < NBW; ++j)
        if (wk == 0 && wn * NBW + j < KK && c < a.C && d < a.D) row[j] = acc[i][j][r];
    }
  if (cb == 0 && tid < a.D) part[a.bias_off + tid] = bias_d;
}

// ---------------------------------------------------------------- weight gradient, specialised waves
//
// Same contraction as conv_s1_wgrad_kernel, with the work of a workgroup split by role:
// waves 0-3 only multiply (K loop, epilogues), waves 4-7 only stage (global -> registers -> LDS),
// one chunk ahead, into the other of two LDS buffers.  In the kernel above a wave alternates both
// roles, and while the other wave of its SIMD streams MFMAs every staging instruction waits about
// one MFMA slot, so the staging phase costs tens of percent of the wave's time; here the staging
// waves are off the multiplying waves' critical path as long as they finish a chunk within one K
// loop.  The two roles are two separate code paths (so each gets the register file to itself:
// accumulators on one side, in-flight tiles and item descriptors on the other) that walk the same
// chunk schedule and execute the same sequence of workgroup barriers:
//   Z (buffers zeroed), F (buffer 0 staged), then per chunk [E1 (WK > 1), E2 at the end of an
//   example in norm mode], I (chunk consumed / next chunk staged), and after the last chunk in
//   clipped mode [E1 (WK > 1)], S (bias sums complete).
// LDS: [buffer 0][buffer 1][cross-wave area (WK > 1)], each buffer = [xch][XPLANE] input + [DT][LDP] Delta.
template <int KH, int KW, int DB, bool FLATC, bool CLIP>
__global__ __launch_bounds__(512, 1) void conv_s1_wgrad_ws_kernel(const ConvWgArgs a) {
  constexpr int KK = KH * KW;
  constexpr int WD = FLATC ? 1 : (DB >= 4 ? 4 : DB);
  constexpr int WN = FLATC ? 1 : (DB >= 4 ? 1 : 2);
  constexpr int WK = 4 / (WD * WN);
  constexpr int NBW = FLATC ? 1 : (KK + WN - 1) / WN;
  static_assert(WD * WN * WK == 4, "wave decomposition");
  constexpr int DT = 32 * DB;
  constexpr int XV = CONV_WG_XV;
  constexpr int DV = (DB == 1 && !FLATC) ? 4 : 8;
  extern __shared__ float smem[];
  const int xch = FLATC ? a.C : 32;
  const int XS = xch * a.t.XPLANE, BUF = XS + DT * a.LDP;  // a buffer: input planes, then Delta rows
  float *xs = smem + 2 * BUF;                               // [(WD*WN) groups][WK-1][NBW*16][64]
  __shared__ float red[4];
  __shared__ float rsum[2][128]; // bias gradient of the example being staged / being reduced (norm mode: by parity)
  const int tid = threadIdx.x;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cb = blockIdx.x, c0 = cb * 32;
  const int HW = a.H * a.W, OHW = a.OH * a.OW;
  const int bbeg = blockIdx.y * a.ex_per_block, bend = min(a.B, bbeg + a.ex_per_block);
  const int nimg_max = !CLIP ? 1 : a.t.NIMG;
  const int n_chunks = ((bend - bbeg + nimg_max - 1) / nimg_max) * a.t.row_tiles;

  // zero both buffers once: the halo columns of the input planes are never written again
  for (int e = tid; e < 2 * BUF; e += 512) smem[e] = 0.f;
  if (tid < 256) rsum[tid >> 7][tid & 127] = 0.f;
  __syncthreads(); // Z

  if (wave8 >= 4) {
    // ================================================================ staging waves
    const int ptid = tid & 255;
    // static item descriptors (same item order as conv_s1_wgrad_kernel, 256 staging threads)
    int x_lds[XV], x_goff[XV], x_ir[XV];
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      const int it = ptid + j * 256;
      const int t1 = (int)a.dWQ.div(it), q = it - t1 * a.WQ;
      const int t2 = (int)a.dROWS.div(t1), rr = t1 - t2 * a.ROWS;
      const int c = (int)a.dNIMG.div(t2), img = t2 - c * a.t.NIMG;
      const bool ok = c < xch && c0 + c < a.C;
      x_lds[j] = ok ? c * a.t.XPLANE + img * a.t.IMGPL + rr * a.t.LDW + a.pad + 4 * q : -1;
      x_goff[j] = (img * a.C + c) * HW + (rr - a.pad) * a.W + 4 * q;
      x_ir[j] = (img << 16) | rr;
    }
    const int PQ = a.PCH >> 2;
    int d_lds[DV], d_goff[DV], d_ir[DV];
#pragma unroll
    for (int j = 0; j < DV; ++j) {
      const int it = ptid + j * 256;
      const int d = (int)a.dPQ.div(it), p = 4 * (it - d * PQ);
      const int img = (int)a.t.dTROW.div(p), rem = p - img * a.t.TR * a.OW;
      const int r = (int)a.t.dOW.div(rem);
      const bool ok = d < DT;
      d_lds[j] = ok ? d * a.LDP + p : -1;
      d_goff[j] = (d < a.D) ? (img * a.Dstride + d) * OHW + rem : -1;
      d_ir[j] = (img << 16) | r;
    }
    float rowsum[DV]; // bias gradient: sum of the staged (scaled) Delta of item j's row, this thread's pixels
#pragma unroll
    for (int j = 0; j < DV; ++j) rowsum[j] = 0.f;
    float4 xr[XV], dr[DV];
    float dsv[DV];
    unsigned xok = 0, dok = 0;
    auto prefetch = [&](int b, int nimg, int r0, int rows) {
      const long xb = ((long)b * a.C + c0) * HW + (long)r0 * a.W;
#pragma unroll
      for (int j = 0; j < XV; ++j) {
        const int img = x_ir[j] >> 16, rr = x_ir[j] & 0xffff;
        const int ih = r0 + rr - a.pad;
        const bool ok = x_lds[j] >= 0 && img < nimg && rr < rows + KH - 1 && (unsigned)ih < (unsigned)a.H;
        xr[j] = *reinterpret_cast<const float4 *>(a.x + (ok ? xb + x_goff[j] : 0));
        xok = ok ? (xok | (1u << j)) : (xok & ~(1u << j));
      }
      const long db_ = (long)b * a.Dstride * OHW + (long)r0 * a.OW;
#pragma unroll
      for (int j = 0; j < DV; ++j) {
        const int img = d_ir[j] >> 16, r = d_ir[j] & 0xffff;
        const bool ok = d_goff[j] >= 0 && img < nimg && r < rows;
        dr[j] = *reinterpret_cast<const float4 *>(a.delta + (ok ? db_ + d_goff[j] : 0));
        if (CLIP) dsv[j] = a.scale[ok ? b + img : 0];
        dok = ok ? (dok | (1u << j)) : (dok & ~(1u << j));
      }
    };
    // The row sums into rsum[par], in a fixed order: the PQ threads that hold the pixels of one row are consecutive
    // lanes of one wave (PQ is a power of two of at most 64: the host selects this kernel only then), so they are
    // summed with exchanges inside the wave and the row's first lane is the only writer of its entry.
    auto flush_rows = [&](int par) {
#pragma unroll
      for (int j = 0; j < DV; ++j) {
        const int d = (int)a.dPQ.div(ptid + j * 256);
        float v = rowsum[j];
        for (int o = PQ >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        if (d_lds[j] >= 0 && (ptid & (PQ - 1)) == 0) rsum[par][d] += v;
        rowsum[j] = 0.f;
      }
    };
    // registers -> LDS buffer; `last`: the chunk ends its example (norm mode), whose bias sums go to rsum[par]
    auto stash = [&](float *buf, bool last, int par) {
      float *Xl = buf, *Dl = buf + XS;
#pragma unroll
      for (int j = 0; j < XV; ++j)
        if (x_lds[j] >= 0) {
          const float4 v = ((xok >> j) & 1u) ? xr[j] : f4zero();
          float *d = Xl + x_lds[j];
          d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
#pragma unroll
      for (int j = 0; j < DV; ++j)
        if (d_lds[j] >= 0) {
          const float sv = ((dok >> j) & 1u) ? (CLIP ? dsv[j] : 1.f) : 0.f;
          const float4 v = ((dok >> j) & 1u) ? dr[j] : f4zero();
          float *d = Dl + d_lds[j];
          const float w0 = v.x * sv, w1 = v.y * sv, w2 = v.z * sv, w3 = v.w * sv;
          d[0] = w0; d[1] = w1; d[2] = w2; d[3] = w3;
          if (cb == 0) rowsum[j] += (w0 + w1) + (w2 + w3);
        }
      if (cb == 0 && last) flush_rows(par);
    };
    int f_b = bbeg, f_rt = 0, f_ex = 0; // chunk held in registers (example ordinal f_ex)
    auto f_prefetch = [&]() {
      const int r0 = f_rt * a.t.TR;
      prefetch(f_b, min(nimg_max, bend - f_b), r0, min(a.t.TR, a.OH - r0));
    };
    auto f_stash = [&](float *buf) {
      stash(buf, !CLIP && f_rt == a.t.row_tiles - 1, f_ex & 1);
      if (++f_rt == a.t.row_tiles) { f_rt = 0; f_b += nimg_max; ++f_ex; }
    };
    if (n_chunks > 0) {
      f_prefetch();
      f_stash(smem);
      if (n_chunks > 1) f_prefetch();
    }
    __syncthreads(); // F
    int m_rt = 0; // row tile of the chunk being multiplied by the other waves
    for (int ci = 0; ci < n_chunks; ++ci) {
      if (ci + 1 < n_chunks) { // registers hold chunk ci+1
        f_stash(smem + ((ci + 1) & 1) * BUF);
        if (ci + 2 < n_chunks) f_prefetch();
      }
      if (!CLIP && m_rt == a.t.row_tiles - 1) {
        if (WK > 1) __syncthreads(); // E1
        __syncthreads();             // E2
      }
      if (++m_rt == a.t.row_tiles) m_rt = 0;
      __syncthreads(); // I
    }
    if (!CLIP) return;
    if (cb == 0) flush_rows(0);
    if (WK > 1) __syncthreads(); // E1
    __syncthreads();             // S
    return;
  }

  // ================================================================ multiplying waves
  const int lane = tid & 63, li = lane & 31, lk = lane >> 5, wave = wave8;
  const int wd = wave / (WN * WK), wn = (wave / WK) % WN, wk = wave % WK;
  f32x16 acc[NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  int xlane = li * a.t.XPLANE + lk;
  const int dlane = li * a.LDP + lk;
  int tapoff[NBW];
  bool tapok[NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    const int tap = wn * NBW + j;
    const int kh = tap / KW, kw = tap - kh * KW;
    tapok[j] = tap < KK;
    tapoff[j] = tapok[j] ? kh * a.t.LDW + kw : 0;
  }
  if (FLATC) { // lane = (channel, tap)
    const int ch = li / KK, tap = li - ch * KK, kh = tap / KW, kw = tap - kh * KW;
    tapok[0] = li < a.C * KK;
    tapoff[0] = 0;
    xlane = (tapok[0] ? ch * a.t.XPLANE + kh * a.t.LDW + kw : 0) + lk;
  }
  const int col0 = 2 * wk;
  constexpr int colstep = 2 * WK;
  const int c = c0 + li;
  const int grp = wave / WK;

  // hand the accumulators of the waves that split the pixel pairs to the wk == 0 wave (barrier E1)
  auto publish = [&]() {
    if (WK > 1) {
      if (wk > 0) {
        float *dst = xs + ((grp * (WK - 1) + wk - 1) * NBW * 16) * 64 + lane;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[(j * 16 + r) * 64] = acc[j][r];
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __syncthreads(); // E1
    }
  };
  auto gathered = [&](int j, int r) { // on wk == 0 waves after publish()
    float v = acc[j][r];
#pragma unroll
    for (int q = 0; q < WK - 1; ++q) v += xs[(((grp * (WK - 1) + q) * NBW + j) * 16 + r) * 64 + lane];
    return v;
  };
  const int spr = (a.OW - col0 + colstep - 1) / colstep; // steps per row
  const int gpr = (spr + 3) >> 2;                        // groups of four steps per row
  const int back = 4 * colstep * (gpr - 1);              // from a row's last group back to its first column

  // The whole chunk loop, compiled once per (ALL4: every group has four steps in the row, LAST: the wave's last
  // tap slot holds a tap), so that the K loop has no branch between its MFMAs.
  auto consume = [&](auto all4_c, auto last_c) {
    constexpr bool ALL4 = decltype(all4_c)::value;
    constexpr int NT = (FLATC || decltype(last_c)::value) ? NBW : NBW - 1;
    int m_b = bbeg, m_rt = 0, m_ex = 0; // chunk being multiplied
    for (int ci = 0; ci < n_chunks; ++ci) {
      const int r0 = m_rt * a.t.TR;
      const int nimg = min(nimg_max, bend - m_b), rows = min(a.t.TR, a.OH - r0);
      {
        // K loop: groups of four pixel-pair steps; operand addresses are immediate offsets from one pointer
        // per operand, the LDS reads of step s+1 are issued before the MFMAs of step s
        const float *buf = smem + (ci & 1) * BUF;
        const int d_skip = (a.t.TR - rows) * a.OW, x_skip = a.t.IMGPL - rows * a.t.LDW; // to the next image
        const int ngroups = nimg * rows * gpr;
        const float *dp = buf + XS + dlane + (wd * 32) * a.LDP + col0;
        const float *xp[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) xp[j] = buf + xlane + col0 + tapoff[j];
        float av[2], bv[2][NT];
        av[0] = dp[0];
#pragma unroll
        for (int j = 0; j < NT; ++j) bv[0][j] = xp[j][0];
        int gi = 0, r = 0;
        for (int g = 0; g < ngroups; ++g) {
          const int nv = spr - 4 * gi; // steps of this group inside the row
          int dd = 4 * colstep, dx = 4 * colstep;
          if (++gi == gpr) {
            gi = 0; dd = a.OW - back; dx = a.t.LDW - back;
            if (++r == rows) { r = 0; dd += d_skip; dx += x_skip; }
          }
          if (g + 1 == ngroups) { dd = 0; dx = 0; } // the last group re-reads its own first step: in bounds, unused
          const float *dpn = dp + dd;
          const float *xpn[NT];
#pragma unroll
          for (int j = 0; j < NT; ++j) xpn[j] = xp[j] + dx;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int cur = u & 1, nxt = cur ^ 1;
            if (u < 3) {
              av[nxt] = dp[(u + 1) * colstep];
#pragma unroll
              for (int j = 0; j < NT; ++j) bv[nxt][j] = xp[j][(u + 1) * colstep];
            } else {
              av[nxt] = dpn[0];
#pragma unroll
              for (int j = 0; j < NT; ++j) bv[nxt][j] = xpn[j][0];
            }
            if (ALL4 || u < nv) {
              if (FLATC && !tapok[0]) bv[cur][0] = 0.f; // lanes beyond the C*KK flattened columns
#pragma unroll
              for (int j = 0; j < NT; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur], bv[cur][j], acc[j], 0, 0, 0);
            }
          }
          dp = dpn;
#pragma unroll
          for (int j = 0; j < NT; ++j) xp[j] = xpn[j];
        }
      }
      if (!CLIP && m_rt == a.t.row_tiles - 1) {
        // end of example m_b: squared norm of this block's share into its slot, accumulators back to zero
        publish();
        float part = 0.f;
        if (wk == 0) {
          const int CKK = a.C * KK;
#pragma unroll
          for (int j = 0; j < NBW; ++j) {
            const int tap = wn * NBW + j;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int d = wd * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
              const float v = gathered(j, r);
              part += v * v; // entries outside the real (d, c, tap) range are exact zeros
            }
            if (WK > 1) __builtin_amdgcn_sched_barrier(0);
          }
        }
        if (cb == 0 && tid < DT) { // staged one chunk ahead: this example's sums were complete a barrier ago
          const float bias_d = rsum[m_ex & 1][tid];
          rsum[m_ex & 1][tid] = 0.f;
          if (tid < a.D) part += bias_d * bias_d;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
        if (lane == 0) red[wave] = part;
#pragma unroll
        for (int j = 0; j < NBW; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
        __syncthreads(); // E2
        if (tid == 0) a.out[(long)(a.slot0 + cb) * a.slot_stride + m_b] = red[0] + red[1] + red[2] + red[3];
      }
      if (++m_rt == a.t.row_tiles) { m_rt = 0; m_b += nimg_max; ++m_ex; }
      __syncthreads(); // I
    }
  };

  __syncthreads(); // F
  {
    const bool all4 = (spr & 3) == 0, last_ok = FLATC || tapok[NBW - 1];
    if (all4 && last_ok) consume(std::true_type{}, std::true_type{});
    else if (all4) consume(std::true_type{}, std::false_type{});
    else if (last_ok) consume(std::false_type{}, std::true_type{});
    else consume(std::false_type{}, std::false_type{});
  }
  if (!CLIP) return;

  // clipped mode: one partial for the block's examples
  publish();       // E1 (WK > 1)
  __syncthreads(); // S
  float *part = a.out + (long)blockIdx.y * a.part_stride;
  if (FLATC) {
    const int CKK = a.C * KK;
    if (wk == 0)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int d = 8 * (r >> 2) + 4 * lk + (r & 3);
        if (li < CKK && d < a.D) part[(long)d * CKK + li] = gathered(0, r);
      }
    if (tid < a.D) part[a.bias_off + tid] = rsum[0][tid];
    return;
  }
  if (wk == 0)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int d = wd * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
      float *row = part + ((long)d * a.C + c) * KK + wn * NBW;
#pragma unroll
      for (int j = 0; j < NBW; ++j)
        if (wn * NBW + j < KK && c < a.C && d < a.D) row[j] = gathered(j, r);
    }
  if (cb == 0 && tid < a.D) part[a.bias_off + tid] = rsum[0][tid];
}

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

// FULL: M = 32, every store unconditional
template <bool FULL>
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

  Tile cur = setup(t_begin);
  fetch(cur);
  int buf = 0;
  for (int t = t_begin; t < t_end; ++t) {
#pragma unroll
    for (int i = 0; i < CF_NI; ++i) Xl[buf][tid + 256 * i] = xr[i];
    __syncthreads(); // the tile is staged; the buffer written next was last read before the previous barrier
    const Tile nxt = setup(min(t + 1, t_end - 1)); // (past the run's last tile: it is read again, unused)
    fetch(nxt);
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
        const float v = act_apply(a.act, acc[r] + bias_r[r]);
        const unsigned off = (FULL || mu + 4 * lk < a.M) ? o_row : OUTSIDE;
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), ors, off, 4 * mu * HW, 0);
      }
    }
    cur = nxt;
    buf ^= 1;
  }
}

// Per-example squared gradient norm of a 3x3 / stride-1 / pad-1 convolution on small planes, from Gram matrices.
//
// The per-example weight gradient is G = sum_p delta_p (x) patch_p (Section 1, item 2a: one gradient per example),
// so  ||G||_F^2 = sum_{p,q} (delta_p . delta_q) (patch_p . patch_q),  and the bias gradient sum_p delta_p has
// squared norm sum_{p,q} delta_p . delta_q.  With the P x P Gram matrices  Gx = X X^T  (X: the P x 9C patch
// matrix) and  Gd = Delta Delta^T  the layer's share of the squared norm is  sum_{p,q} Gd[p][q] (Gx[p][q] + 1).
// That is  P^2 (9C + D)  multiply-adds instead of the  9 C D P  of forming G, and the reduction runs over P^2
// numbers instead of 9 C D: the cheaper route whenever the plane is small (8x8 and 4x4 here).  The result is
// the same number up to rounding order; nothing of the clipped sum changes.
//
// One workgroup per tile of 64 Gram rows: one example with P <= 64 pixels, or four examples with P <= 16 (then
// only the four diagonal 16 x 16 blocks are used).  Each of the four waves owns one 32 x 32 block of the tile
// and runs v_mfma_f32_32x32x2_f32 over k = (plane pair, tap); both operands come from the same LDS image of 32
// haloed planes, at compile-time offsets.  Input planes and Delta planes are staged by the same code (both are
// [planes][OH][OW] in memory); Delta uses the centre tap only.  Several workgroups share a CU and overlap one
// another's staging.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "gemm_tile.h"

struct ConvGramArgs {
  const float *x;     // layer input [B, C, OH, OW] (pad 1, stride 1: the input plane equals the output plane)
  const float *delta; // [B, D, OH, OW]
  float *slot;        // [B]: receives the layer's share of every example's squared norm
  int B, C, D;
};

template <int OH, int OW>
struct ConvGramGeom {
  static constexpr int P = OH * OW;
  static constexpr int SP = P <= 16 ? 16 : 64; // Gram rows reserved per example
  static constexpr int NIMG = 64 / SP;
  // Row and image strides chosen so that the 32 Gram rows a half-wave reads in one instruction fall into 32
  // different LDS banks: 8-wide planes, four rows of 8 at stride 24 -> banks 0-7, 24-31, 16-23, 8-15; 4-wide
  // planes, two images of four rows of 4 at row stride 8 and image stride 52 (= 20 mod 32).  Tap offsets shift
  // all lanes alike.  (With the natural row stride OW + 2 the kernel measured more bank-conflict cycles than
  // LDS instructions.)
  static constexpr int LDW = OW == 8 ? 24 : (OW == 4 ? 8 : OW + 2);
  static constexpr int IMGPL = (OH + 2) * LDW + (OW == 4 ? 4 : 0);
  static constexpr int XPL = (NIMG * IMGPL) | 1; // odd plane stride (the two k-halves of a wave are separate passes)
  static constexpr int CH = 32;                  // planes per staged chunk
  static constexpr int WQ = OW / 4;
  static constexpr int ITEMS = CH * NIMG * OH * WQ; // float4 items per chunk
  static constexpr int IV = (ITEMS + 255) / 256;
  static_assert(P <= 64 && OW % 4 == 0, "plane must fit one 64-row tile and rows must be whole float4 groups");
};

template <int OH, int OW>
__global__ __launch_bounds__(256) void conv_gram_norm_kernel(ConvGramArgs a) {
  typedef ConvGramGeom<OH, OW> Gm;
  constexpr int P = Gm::P, SP = Gm::SP, NIMG = Gm::NIMG, LDW = Gm::LDW, IMGPL = Gm::IMGPL, XPL = Gm::XPL, CH = Gm::CH;
  constexpr int WQ = Gm::WQ, IV = Gm::IV;
  __shared__ float buf[CH * XPL];
  __shared__ float red[4][2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b0 = blockIdx.x * NIMG;

  for (int i = tid; i < CH * XPL; i += 256) buf[i] = 0.f; // the halo cells are never written again

  // staging items: (plane, image, row, float4 group) -> LDS word and offset inside the chunk's global planes
  int s_lds[IV], s_goff[IV], s_img[IV], s_pl[IV];
#pragma unroll
  for (int j = 0; j < IV; ++j) {
    const int it = tid + j * 256;
    const int q = it % WQ, t1 = it / WQ;
    const int row = t1 % OH, t2 = t1 / OH;
    const int img = t2 % NIMG, pl = t2 / NIMG;
    const bool ok = it < Gm::ITEMS;
    s_lds[j] = ok ? pl * XPL + img * IMGPL + (row + 1) * LDW + 1 + 4 * q : -1;
    s_goff[j] = pl * P + row * OW + 4 * q;
    s_img[j] = img;
    s_pl[j] = pl;
  }

  // the wave's block (bi, bj) of the 64 x 64 tile; a lane supplies Gram row 32*bi + lane%32 to the A operand and
  // Gram row 32*bj + lane%32 to the B operand, for plane (lane / 32) of the current plane pair
  const int bi = wave >> 1, bj = wave & 1;
  auto window = [&](int grow) { // top-left word of the 3x3 window of that Gram row's pixel, in the haloed image
    const int slot = grow / SP, pix = grow % SP;
    const int pc = pix < P ? pix : 0; // rows past the plane are masked in the reduction; keep their reads in range
    return slot * IMGPL + (pc / OW) * LDW + (pc % OW) + (lane >> 5) * XPL;
  };
  const float *pa = buf + window(32 * bi + (lane & 31));
  const float *pb = buf + window(32 * bj + (lane & 31));

  f32x16 accx, accd;
#pragma unroll
  for (int r = 0; r < 16; ++r) { accx[r] = 0.f; accd[r] = 0.f; }
  __syncthreads();

  // One pass over the NPL planes of src ([B, NPL, OH, OW]) in chunks of CH; TAPS = 9 (input) or 1 (Delta, centre).
  auto pass = [&](const float *src, const int NPL, auto taps_tag, f32x16 &acc) {
    constexpr int TAPS = decltype(taps_tag)::value;
    for (int c0 = 0; c0 < NPL; c0 += CH) {
      float4 v[IV];
#pragma unroll
      for (int j = 0; j < IV; ++j) {
        const bool ok = s_lds[j] >= 0 && c0 + s_pl[j] < NPL && b0 + s_img[j] < a.B;
        const long off = ok ? ((long)(b0 + s_img[j]) * NPL + c0) * P + s_goff[j] : 0; // word 0 is always there
        const float4 g = *reinterpret_cast<const float4 *>(src + off);
        v[j] = ok ? g : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      __syncthreads(); // every wave has finished reading the previous chunk
#pragma unroll
      for (int j = 0; j < IV; ++j)
        if (s_lds[j] >= 0) {
          float *d = buf + s_lds[j];
          d[0] = v[j].x; d[1] = v[j].y; d[2] = v[j].z; d[3] = v[j].w;
        }
      __syncthreads();
      const int nv = min(CH, NPL - c0); // planes past nv hold zeros (zero-filled above): whole pairs are skipped
#pragma unroll
      for (int cp = 0; cp < CH / 2; ++cp) {
        if (2 * cp < nv) { // (a guard, not a break: the loop unrolls and every offset is a compile-time constant)
#pragma unroll
          for (int t = 0; t < TAPS; ++t) {
            const int off = cp * 2 * XPL + (TAPS == 9 ? (t / 3) * LDW + (t % 3) : LDW + 1);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[off], pb[off], acc, 0, 0, 0);
          }
        }
      }
    }
  };
  pass(a.x, a.C, std::integral_constant<int, 9>{}, accx);
  pass(a.delta, a.D, std::integral_constant<int, 1>{}, accd);

  // sum of Gd (Gx + 1) over the entries whose row and column belong to the same example and lie inside the plane
  const int gcol = 32 * bj + (lane & 31);
  const int ec = gcol / SP;
  const bool col_ok = (gcol % SP) < P;
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int grow = 32 * bi + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    const bool ok = col_ok && grow / SP == ec && (grow % SP) < P;
    s += ok ? accd[r] * (accx[r] + 1.f) : 0.f;
  }
  // fixed-order reduction: 16-column groups (one example each when SP = 16), then the two k-halves
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
  s += __shfl_xor(s, 32, 64);
  if ((lane & 47) == 0) red[wave][lane >> 4] = s; // lanes 0 and 16: column groups 0 and 1 of the wave's block
  __syncthreads();
  if (tid < NIMG && b0 + tid < a.B) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
      for (int cg = 0; cg < 2; ++cg)
        if ((32 * (w & 1) + 16 * cg) / SP == tid) tot += red[w][cg];
    a.slot[b0 + tid] = tot;
  }
}

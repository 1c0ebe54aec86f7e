// 3x3 / stride-1 / pad-1 convolution (forward and backward-data) by the minimal-filtering form F(2x2, 3x3):
// every 2x2 block of outputs ("tile") is  Y = A^T [ sum_c U_c (.) V_c ] A  with  V_c = B^T d_c B  the transform of
// the tile's 4x4 input patch and  U_c = G g_c G^T  the transform of the 3x3 filter.  The sum over input channels
// is 16 independent contractions (one per transform component) of 16 multiplies per tile and channel instead of
// the 36 of the direct form: the same convolution up to rounding (fp32, a few ulp more than the direct sum).
//
//   B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]   G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]   A^T = [1 1 1 0; 0 1 -1 -1]
//
// One workgroup = 32 tiles (128 output pixels: whole rows of one image, or whole images) x 32*DB output channels.
// The tiles' patches are windows of one haloed region of RS floats per channel.  Per chunk of 8 input channels the
// 8 x RS floats are loaded once (about 1.3 fetches per input element), held in registers one chunk ahead, written to
// a double-buffered LDS array, and every thread transforms one (channel, tile) patch from there into its 16
// components ([component][channel][tile] in LDS, double-buffered as well).  One barrier per chunk:
//   iteration n:  raw(n+1) registers -> Xr[(n+1)%2];  transform Xr[n%2] -> V[n%2];  barrier;  issue the loads of
//                 raw(n+2);  multiply V[n%2], reloading every weight register for chunk n+1 right after its use
// Wave w owns transform row w (components 4w .. 4w+3): v_mfma_f32_32x32x2_f32 with M = output channel, N = tile,
// K = channel pair; the A operand (transformed weights, [component][channel][Mpad] in global memory, zero rows /
// columns as padding) comes straight from global memory into registers.  A wave holds 4*DB accumulator tiles, so
// two or three workgroups share a CU and fill one another's load and transform phases.  (Measured alternatives that
// were no faster: patches loaded straight from global memory, two to four chunks of look-ahead, 16-byte weight
// loads into a second register set.)
// Epilogue: each wave folds its row with A (4 components -> 2 numbers), the four rows meet in LDS, and each wave
// finishes a quarter of the output channels: bias + activation (forward) or the derivative of the producing
// activation (backward-data), 8-byte stores.
#pragma once
#include <type_traits>

#include "gemm_tile.h"
#include "kernels_misc.h"

#define WINO_CC 8 // input channels per chunk

struct ConvWinoArgs {
  const float *x;      // input [B, Cin, H, W]
  const float *u;      // transformed weights [16][Cpad][Mpad]; rows c >= Cin and columns m >= M are zero
  const float *bias;   // forward: bias[M]; backward-data: null
  const float *a_prev; // backward-data with act != 0: output of the activation whose derivative multiplies the result
  float *out;          // [B, M, H, W]
  // forward, optional: the 2x2 / stride-2 pool that follows the layer, taken in the epilogue (a tile is one pool
  // window): pool = 1 maximum (first maximum in row-major order wins, its index 0..3 goes to pool_arg), 2 average
  float *pool_out;     // [B, M, H/2, W/2]
  uint8_t *pool_arg;   // [B, M, H/2, W/2] (maximum only)
  int pool;
  int B, Cin, Cpad, H, W, M, Mpad; // Cpad: multiple of WINO_CC; Mpad: multiple of 32*DB times gridDim.y
  int act;
  int tw_shift, tpi_shift; // log2(W/2), log2((H/2)*(W/2)): tiles per row / per image are powers of two
};

// Weight transforms for one layer W[D][C][3][3]:
//   uf[(comp*Cfp + c)*Dfp + d] = (G W[d][c] G^T)[comp]                 forward       (Cin = C, M = D)
//   ub[(comp*Dbp + d)*Cbp + c] = (G flip(W[d][c]) G^T)[comp]           backward-data (Cin = D, M = C)
// The padding rows / columns stay zero from the allocation.
struct WinoLayoutArgs {
  int n;
  struct { long w_off; float *uf, *ub; int D, C, Cfp, Dfp, Dbp, Cbp; } l[16];
};
DEVI void wino_weight_body(const float *__restrict__ params, const WinoLayoutArgs &a, int layer) {
  const auto &L = a.l[layer];
  const int total = L.D * L.C;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const int d = i / L.C, c = i - d * L.C;
    float g[3][3];
#pragma unroll
    for (int k = 0; k < 9; ++k) g[k / 3][k % 3] = params[L.w_off + (long)i * 9 + k];
#pragma unroll
    for (int flip = 0; flip < 2; ++flip) {
      float *dst = flip ? L.ub : L.uf;
      if (dst == nullptr) continue;
      float t[4][3]; // G g
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const float g0 = flip ? g[2][2 - j] : g[0][j], g1 = flip ? g[1][2 - j] : g[1][j], g2 = flip ? g[0][2 - j] : g[2][j];
        t[0][j] = g0;
        t[1][j] = 0.5f * (g0 + g1 + g2);
        t[2][j] = 0.5f * (g0 - g1 + g2);
        t[3][j] = g2;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float u0 = t[r][0], u1 = 0.5f * (t[r][0] + t[r][1] + t[r][2]), u2 = 0.5f * (t[r][0] - t[r][1] + t[r][2]),
                    u3 = t[r][2];
        const float uu[4] = {u0, u1, u2, u3};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const int comp = r * 4 + s;
          if (flip) dst[((long)comp * L.Dbp + d) * L.Cbp + c] = uu[s];
          else dst[((long)comp * L.Cfp + c) * L.Dfp + d] = uu[s];
        }
      }
    }
  }
}
__global__ void wino_weight_kernel(const float *__restrict__ params, const WinoLayoutArgs a) {
  wino_weight_body(params, a, blockIdx.y);
}
// Both weight preparations of a step in one launch: blockIdx.y walks the direct kernels' layouts, then the transforms.
__global__ void conv_weights_kernel(const float *__restrict__ params, const ConvLayoutArgs ca, const WinoLayoutArgs wa) {
  if ((int)blockIdx.y < ca.n) conv_weight_layout_body(params, ca, blockIdx.y);
  else wino_weight_body(params, wa, blockIdx.y - ca.n);
}

// Output stage shared by the forward / backward-data kernels.  Row w of  M A:  t0 = m0 + m1 + m2,  t1 = m1 - m2 - m3
// (each wave folds its own transform row); the four rows meet in LDS (Tl, [wave][k][r][lane], 32 KB) and
// Y[0][k] = T0 + T1 + T2,  Y[1][k] = T1 - T2 - T3; wave w finishes accumulator rows 4w .. 4w+3 of every block of 32
// output channels: bias + activation (and the 2x2 pool that follows, if any) or the derivative of the producing
// activation, 8-byte stores.  (img, ty, tx): the lane's tile; lanes past the batch only take part in the barriers.
template <int DB>
DEVI void wino_store_tiles(const ConvWinoArgs &a, float *Tl, const f32x16 (&acc)[4][DB], int wave, int lane, int m0,
                           int img, bool img_ok, int ty, int tx, int W) {
  const int lk = lane >> 5;
  const int HW = a.H * W;
  const bool fwd = a.bias != nullptr;
  const bool need_side = !fwd && a.act;
  // (The plane before a fused max-pool is never read again: the next layer and the pool's backward pass, which takes
  // the activation's derivative at the window's maximum, the pooled value, read the pooled plane.)
#pragma unroll
  for (int i = 0; i < DB; ++i) {
    __syncthreads(); // every wave is done with the LDS contents of the previous phase
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      Tl[((wave * 2 + 0) * 16 + r) * 64 + lane] = acc[0][i][r] + acc[1][i][r] + acc[2][i][r];
      Tl[((wave * 2 + 1) * 16 + r) * 64 + lane] = acc[1][i][r] - acc[2][i][r] - acc[3][i][r];
    }
    __syncthreads();
    if (!img_ok) continue;
    // (activation, direction and pool are fixed for the launch: the body is compiled per combination and chosen once
    // here, instead of uniform branches around every value.  MODE: 0 forward, 1 forward + max-pool, 2 forward +
    // average pool, 3 backward-data through an activation, 4 backward-data)
    auto finish = [&](auto act_c, auto mode_c) {
      constexpr int ACT = decltype(act_c)::value, MODE = decltype(mode_c)::value;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * wave + rr;
        const int m = m0 + 32 * i + 8 * wave + 4 * lk + rr; // accumulator row r of a lane: 8*(r/4) + 4*lk + r%4
        if (m >= a.M) continue;
        float T[4][2];
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int k = 0; k < 2; ++k) T[w][k] = Tl[((w * 2 + k) * 16 + r) * 64 + lane];
        float2 y0, y1;
        y0.x = T[0][0] + T[1][0] + T[2][0];
        y0.y = T[0][1] + T[1][1] + T[2][1];
        y1.x = T[1][0] - T[2][0] - T[3][0];
        y1.y = T[1][1] - T[2][1] - T[3][1];
        const long o = ((long)img * a.M + m) * HW + (2 * ty) * W + 2 * tx;
        if (MODE <= 2) {
          const float bv = a.bias[m];
          y0.x = act_apply(ACT, y0.x + bv); y0.y = act_apply(ACT, y0.y + bv);
          y1.x = act_apply(ACT, y1.x + bv); y1.y = act_apply(ACT, y1.y + bv);
          if (MODE == 1 || MODE == 2) {
            const long po = ((long)img * a.M + m) * (HW >> 2) + ty * (W >> 1) + tx;
            if (MODE == 1) {
              float best = y0.x; int bi = 0;
              if (y0.y > best) { best = y0.y; bi = 1; }
              if (y1.x > best) { best = y1.x; bi = 2; }
              if (y1.y > best) { best = y1.y; bi = 3; }
              a.pool_out[po] = best;
              a.pool_arg[po] = (uint8_t)bi;
            } else {
              a.pool_out[po] = ((y0.x + y0.y) + (y1.x + y1.y)) * 0.25f;
            }
          }
        } else if (MODE == 3) {
          const float2 s0 = *reinterpret_cast<const float2 *>(a.a_prev + o);
          const float2 s1 = *reinterpret_cast<const float2 *>(a.a_prev + o + W);
          y0.x *= act_deriv_from_out(ACT, s0.x); y0.y *= act_deriv_from_out(ACT, s0.y);
          y1.x *= act_deriv_from_out(ACT, s1.x); y1.y *= act_deriv_from_out(ACT, s1.y);
        }
        if (MODE != 1) { // (the plane before a fused max-pool is never read again)
          *reinterpret_cast<float2 *>(a.out + o) = y0;
          *reinterpret_cast<float2 *>(a.out + o + W) = y1;
        }
      }
    };
    auto with_mode = [&](auto act_c) {
      if (fwd) {
        if (a.pool == 1) finish(act_c, std::integral_constant<int, 1>{});
        else if (a.pool) finish(act_c, std::integral_constant<int, 2>{});
        else finish(act_c, std::integral_constant<int, 0>{});
      } else if (need_side) {
        finish(act_c, std::integral_constant<int, 3>{});
      } else {
        finish(act_c, std::integral_constant<int, 4>{});
      }
    };
    if (a.act == DP_ACT_TANH_) with_mode(std::integral_constant<int, DP_ACT_TANH_>{});
    else if (a.act == DP_ACT_RELU_) with_mode(std::integral_constant<int, DP_ACT_RELU_>{});
    else with_mode(std::integral_constant<int, DP_ACT_NONE_>{});
  }
}

struct ConvWinoRegion {
  int NIMG, ROWS;     // images per workgroup (tiles per image < 32) or 1; pixel rows per workgroup
  int LDW, IMGPL, RS; // W + 2; (ROWS + 2) * LDW; NIMG * IMGPL (all even)
  FastDiv dRS, dIMGPL, dLDW;
};

template <int DB, int XI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(DB == 1 ? 3 : 2, DB == 1 ? 3 : 2)))
void conv_wino_kernel(const ConvWinoArgs a, const ConvWinoRegion rg) {
  constexpr int CC = WINO_CC;
  constexpr int VSZ = 16 * CC * 32;
  extern __shared__ __attribute__((aligned(16))) float wino_smem[];
  float *Vl = wino_smem;          // [2][comp][c][tile]; the epilogue reuses it
  float *Xr = wino_smem + 2 * VSZ; // [2][CC * RS]
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = blockIdx.y * 32 * DB;
  const int HW = a.H * a.W;
  const int TW = 1 << a.tw_shift, TPI = 1 << a.tpi_shift;
  const int XSZ = CC * rg.RS;

  // the workgroup's region and this lane's tile in it
  const int g0 = blockIdx.x * 32;
  const int img0 = g0 >> a.tpi_shift;
  const int ty0 = (g0 & (TPI - 1)) >> a.tw_shift; // first tile row (0 when the workgroup holds whole images)
  const int gt = g0 + li;
  const int img = gt >> a.tpi_shift, trem = gt & (TPI - 1);
  const int ty = trem >> a.tw_shift, tx = trem & (TW - 1);
  const bool img_ok = img < a.B;
  // patch of (channel 2*wave + lk of the chunk, tile li): top-left word in a raw buffer
  const int cc = 2 * wave + lk;
  const int pbase = cc * rg.RS + (img - img0) * rg.IMGPL + 2 * (ty - ty0) * rg.LDW + 2 * tx;

  // staging items: flat index it = tid + j*256 = c * RS + pos  ->  byte offset from the chunk's first channel of the
  // first image; items that hold no input (halo, past the batch) read word 0 and are zeroed
  unsigned xg[XI];
  int xc[XI];
#pragma unroll
  for (int j = 0; j < XI; ++j) {
    const int it = tid + j * 256;
    const int c = (int)rg.dRS.div(it), pos = it - c * rg.RS;
    const int im = (int)rg.dIMGPL.div(pos), rem = pos - im * rg.IMGPL;
    const int rr = (int)rg.dLDW.div(rem), col = rem - rr * rg.LDW;
    const int ih = 2 * ty0 + rr - 1, iw = col - 1;
    const bool ok = it < XSZ && (img0 + im) < a.B && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
    xg[j] = ok ? 4u * (unsigned)((im * a.Cin + c) * HW + ih * a.W + iw) : 0u;
    xc[j] = ok ? c : (1 << 30); // (an item that never holds input fails the channel test below)
  }
  const float *xblk = a.x + (long)img0 * a.Cin * HW;

  // weights: lane (li, lk) of MFMA step (component 4*wave + jj, channel pair cp, block i) reads
  //   u[((4*wave + jj)*Cpad + c0 + 2*cp + lk)*Mpad + m0 + 32*i + li]  =  (uniform pointer) + the lane's byte offset
  const unsigned wlane = 4u * (unsigned)(lk * a.Mpad + li);
  const float *ubase = a.u + ((long)(4 * wave) * a.Cpad) * a.Mpad + m0;
  auto w_ptr = [&](const float *uc, unsigned wl, int jj, int cp, int i) {
    return reinterpret_cast<const float *>(
        reinterpret_cast<const char *>(uc + ((long)jj * a.Cpad + 2 * cp) * a.Mpad + 32 * i) + wl);
  };

  f32x16 acc[4][DB];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[jj][i][r] = 0.f;

  float xr[XI];
  float wr[4][CC / 2][DB];
  // raw loads of the chunk that starts at channel c0 (any c0: channels past Cin read word 0 and are zeroed)
  auto fetch_raw = [&](int c0, float *dst) {
    const float *xc0 = xblk + (long)min(c0, a.Cin - 1) * HW;
    const int left = a.Cin - c0;
#pragma unroll
    for (int j = 0; j < XI; ++j) {
      const unsigned off = xc[j] < left ? xg[j] : 0u;
      dst[j] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(xc0) + off);
    }
  };
  auto store_raw = [&](int c0, const float *src, float *xbuf) {
    const int left = a.Cin - c0;
#pragma unroll
    for (int j = 0; j < XI; ++j)
      if (tid + j * 256 < XSZ) xbuf[tid + j * 256] = xc[j] < left ? src[j] : 0.f;
  };

  fetch_raw(0, xr);
  store_raw(0, xr, Xr);
  __syncthreads();
  fetch_raw(CC, xr);
  __builtin_amdgcn_sched_barrier(0);
  // (weights after the second chunk's raw loads, as in every later chunk: see conv_wino_reg_kernel)
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int cp = 0; cp < CC / 2; ++cp)
#pragma unroll
      for (int i = 0; i < DB; ++i) wr[jj][cp][i] = *w_ptr(ubase, wlane, jj, cp, i);

  int buf = 0;
  for (int c0 = 0; c0 < a.Cin; c0 += CC) {
    store_raw(c0 + CC, xr, Xr + (buf ^ 1) * XSZ);
    { // transform the patch: t = B^T d (rows), v = t B (columns)
      const float *src = Xr + buf * XSZ + pbase;
      float d[16];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float2 p0 = *reinterpret_cast<const float2 *>(src + i * rg.LDW);
        const float2 p1 = *reinterpret_cast<const float2 *>(src + i * rg.LDW + 2);
        d[4 * i + 0] = p0.x; d[4 * i + 1] = p0.y; d[4 * i + 2] = p1.x; d[4 * i + 3] = p1.y;
      }
      float t[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        t[0 + j] = d[0 + j] - d[8 + j];
        t[4 + j] = d[4 + j] + d[8 + j];
        t[8 + j] = d[8 + j] - d[4 + j];
        t[12 + j] = d[4 + j] - d[12 + j];
      }
      float *dst = Vl + buf * VSZ + cc * 32 + li;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        dst[(4 * i + 0) * CC * 32] = t[4 * i + 0] - t[4 * i + 2];
        dst[(4 * i + 1) * CC * 32] = t[4 * i + 1] + t[4 * i + 2];
        dst[(4 * i + 2) * CC * 32] = t[4 * i + 2] - t[4 * i + 1];
        dst[(4 * i + 3) * CC * 32] = t[4 * i + 1] - t[4 * i + 3];
      }
    }
    __syncthreads(); // V[buf] and the next raw chunk are in place (slower waves may still read the other buffers)
    fetch_raw(c0 + 2 * CC, xr);
    // A weight register is reloaded for the next chunk right after the multiply that consumed it (the last chunk
    // re-reads itself: no branch around loads).
    const int cn = min(c0 + CC, a.Cpad - CC);
    const float *un = ubase + (long)cn * a.Mpad;
    unsigned wl = wlane;
    asm volatile("" : "+v"(wl)); // keeps the weight addresses in the form uniform pointer + lane offset
    const float *vb = Vl + buf * VSZ + (4 * wave) * CC * 32 + lk * 32 + li;
#pragma unroll
    for (int cp = 0; cp < CC / 2; ++cp)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const float bv = vb[(jj * CC + 2 * cp) * 32];
#pragma unroll
        for (int i = 0; i < DB; ++i) {
          acc[jj][i] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[jj][cp][i], bv, acc[jj][i], 0, 0, 0);
          wr[jj][cp][i] = *w_ptr(un, wl, jj, cp, i);
        }
      }
    // instruction order: the raw loads first, then multiplies and weight reloads alternating
    __builtin_amdgcn_sched_group_barrier(0x020, XI, 0);
#pragma unroll
    for (int k = 0; k < 4 * (CC / 2); ++k) {
      __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, DB, 0);
    }
    buf ^= 1;
  }

  wino_store_tiles<DB>(a, Vl, acc, wave, lane, m0, img, img_ok, ty, tx, a.W);
}

// ---------------------------------------------------------------------------------------------------------------
// Variant without the component array, for whole chunks of input channels (Cin a multiple of 8): every lane
// transforms, for its own tile, the four channels whose products it feeds to the matrix unit (channel 2*cp + lk for
// channel pair cp), and only the transform row of its wave -- the results are the B operands themselves.  LDS holds
// the raw region only; the transform of chunk n+1 (16 reads and 32 vector operations per lane) is independent of
// the multiplies of chunk n and is issued between them.
//   iteration n:  raw(n+1) registers -> Xr[(n+1)%2];  barrier;  issue loads of raw(n+2);
//                 { transform Xr[(n+1)%2] -> operands of chunk n+1 }  interleaved with  { multiply chunk n }
// Plane geometries are compile-time (W_ columns, ROWS_ pixel rows and NIMG_ images per workgroup, LDS row length
// LDW_ chosen so that the 16 lanes served together read 32 different banks).  Two operand sets and the accumulators
// of 64 output channels fill the registers of a wave at two waves per SIMD; with 32 output channels per workgroup
// the kernel above (three waves per SIMD) measured faster.
template <int W_, int ROWS_, int NIMG_, int LDW_>
struct WinoGeom {
  static constexpr int W = W_, ROWS = ROWS_, NIMG = NIMG_, LDW = LDW_;
  static constexpr int IMGPL = (ROWS + 2) * LDW, RS = NIMG * IMGPL;           // LDS floats per image / per channel
  static constexpr int REAL_IMG = (ROWS + 2) * (W + 2), REAL = NIMG * REAL_IMG; // positions that are staged
  static constexpr int TW = W / 2, TPG = (ROWS / 2) * TW; // tiles per row; tiles per image inside a workgroup
  static_assert(NIMG * TPG == 32 && LDW >= W + 2 && LDW % 2 == 0, "a workgroup covers 32 tiles");
};

template <int DB, class G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv_wino_reg_kernel(const ConvWinoArgs a) {
  constexpr int CC = WINO_CC, RS = G::RS, LDW = G::LDW, XSZ = CC * RS;
  __shared__ __attribute__((aligned(16))) float smem[8192]; // raw buffers [2][CC * RS]; the epilogue uses all of it
  static_assert(2 * XSZ <= 8192, "raw buffers fit");
  float *Xr = smem;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = blockIdx.y * 32 * DB;
  const int HW = a.H * G::W;

  // the workgroup's region: NIMG whole images, or ROWS pixel rows of one image
  int img0, row0;
  if (G::NIMG > 1) { img0 = blockIdx.x * G::NIMG; row0 = 0; }
  else { const int per = a.H / G::ROWS; img0 = blockIdx.x / per; row0 = (blockIdx.x - img0 * per) * G::ROWS; }
  // this lane's tile
  const int iml = li / G::TPG, trem = li % G::TPG, tyl = trem / G::TW, tx = trem % G::TW;
  const int img = img0 + iml;
  const bool img_ok = img < a.B;
  const int ty = row0 / 2 + tyl;
  // first word of the tile's patch for channel lk of a buffer; channel pair cp adds 2*cp*RS, patch row r adds r*LDW
  const float *pat = Xr + lk * RS + iml * G::IMGPL + 2 * tyl * LDW + 2 * tx;
  // the wave's transform row:  t = d[r1] + s2 * d[r2]  (rows of B^T: d0 - d2, d1 + d2, d2 - d1, d1 - d3)
  const int r1 = wave == 0 ? 0 : (wave == 2 ? 2 : 1);
  const int r2 = wave == 0 ? 2 : (wave == 1 ? 2 : (wave == 2 ? 1 : 3));
  const float s2 = wave == 1 ? 1.f : -1.f;

  // staging: thread tid owns position tid of the region (image, row, column of the haloed plane) for all 8 channels
  // of a chunk.  Buffer loads: one resource descriptor for the workgroup's images (it starts one pixel row above the
  // region, so lane offsets are never negative; only addresses of real pixels are formed from it), the channel in the
  // scalar offset, and a lane offset beyond the descriptor's range for positions that hold no input -- those read as
  // zero without touching memory, so nothing is masked on the way to LDS.
  static_assert(G::REAL <= 256, "one position per thread");
  unsigned xg;
  int xl;
  {
    const int im = tid / G::REAL_IMG, rem = tid % G::REAL_IMG;
    const int rr = rem / (G::W + 2), col = rem % (G::W + 2);
    const int ih = row0 + rr - 1, iw = col - 1;
    const bool xok = tid < G::REAL && (img0 + im) < a.B && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)G::W;
    xg = xok ? 4u * (unsigned)(im * a.Cin * HW + rr * G::W + iw) : 0x80000000u;
    xl = tid < G::REAL ? im * G::IMGPL + rr * LDW + col : -1;
  }
  const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float *>(a.x + (long)img0 * a.Cin * HW + (row0 - 1) * G::W), 0, 4 * (G::NIMG * a.Cin * HW + G::W), 0x00020000);

  const unsigned wlane = 4u * (unsigned)(lk * a.Mpad + li);
  const float *ubase = a.u + ((long)(4 * wave) * a.Cpad) * a.Mpad + m0;
  auto w_ptr = [&](const float *uc, unsigned wl, int jj, int cp, int i) {
    return reinterpret_cast<const float *>(
        reinterpret_cast<const char *>(uc + ((long)jj * a.Cpad + 2 * cp) * a.Mpad + 32 * i) + wl);
  };

  f32x16 acc[4][DB];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[jj][i][r] = 0.f;

  float xr[CC];
  float wr[4][CC / 2][DB];
  auto fetch_raw = [&](int c0) {
    const int cc0 = min(c0, a.Cin - CC); // (past the last chunk: re-reads it, unused)
#pragma unroll
    for (int c = 0; c < CC; ++c)
      xr[c] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xrs, xg, 4 * (cc0 + c) * HW, 0));
  };
  auto store_raw = [&](float *xbuf) {
    if (xl >= 0) {
#pragma unroll
      for (int c = 0; c < CC; ++c) xbuf[xl + c * RS] = xr[c];
    }
  };
  // B operands of one chunk from a raw buffer: bv[cp][jj] = component (wave, jj) of channel 2*cp + lk
  auto transform = [&](const float *xbuf, float (*bv)[4]) {
    const float *p = pat + (xbuf - Xr);
#pragma unroll
    for (int cp = 0; cp < CC / 2; ++cp) {
      const float *q = p + 2 * cp * RS;
      const float2 a0 = *reinterpret_cast<const float2 *>(q + r1 * LDW);
      const float2 a1 = *reinterpret_cast<const float2 *>(q + r1 * LDW + 2);
      const float2 b0 = *reinterpret_cast<const float2 *>(q + r2 * LDW);
      const float2 b1 = *reinterpret_cast<const float2 *>(q + r2 * LDW + 2);
      const float t0 = fmaf(s2, b0.x, a0.x), t1 = fmaf(s2, b0.y, a0.y), t2 = fmaf(s2, b1.x, a1.x), t3 = fmaf(s2, b1.y, a1.y);
      bv[cp][0] = t0 - t2;
      bv[cp][1] = t1 + t2;
      bv[cp][2] = t2 - t1;
      bv[cp][3] = t1 - t3;
    }
  };

  // (the first weight loads are issued AFTER the second chunk's raw loads, as in every later chunk: the wait for a raw
  // chunk is then "all but the 32 weight loads behind it" on every path into the loop, not a drain of everything)
  fetch_raw(0);
  // (padding words of the rows are never read; halo words are rewritten as zeros with every chunk)
  store_raw(Xr);
  __syncthreads();
  fetch_raw(CC);
  __builtin_amdgcn_sched_barrier(0); // (the scheduler would put the weight loads first)
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int cp = 0; cp < CC / 2; ++cp)
#pragma unroll
      for (int i = 0; i < DB; ++i) wr[jj][cp][i] = *w_ptr(ubase, wlane, jj, cp, i);
  float bA[CC / 2][4], bB[CC / 2][4];
  transform(Xr, bA);

  auto chunk = [&](int c0, int buf, float (*bcur)[4], float (*bnext)[4]) {
    store_raw(Xr + (buf ^ 1) * XSZ);
    __syncthreads(); // raw(n+1) is in place; every wave has finished reading the buffer that raw(n+2) will overwrite
    fetch_raw(c0 + 2 * CC);
    transform(Xr + (buf ^ 1) * XSZ, bnext);
    const int cn = min(c0 + CC, a.Cpad - CC);
    const float *un = ubase + (long)cn * a.Mpad;
    unsigned wl = wlane;
    asm volatile("" : "+v"(wl)); // keeps the weight addresses in the form uniform pointer + lane offset
#pragma unroll
    for (int cp = 0; cp < CC / 2; ++cp)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int i = 0; i < DB; ++i) {
          acc[jj][i] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[jj][cp][i], bcur[cp][jj], acc[jj][i], 0, 0, 0);
          wr[jj][cp][i] = *w_ptr(un, wl, jj, cp, i);
        }
    // instruction order: the raw loads first, then per multiply step its weight reloads, one LDS read and two vector
    // operations of the next chunk's transform
    __builtin_amdgcn_sched_group_barrier(0x020, CC, 0);
#pragma unroll
    for (int k = 0; k < 4 * (CC / 2); ++k) {
      __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, DB, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
    }
  };
  int buf = 0;
  for (int c0 = 0; c0 < a.Cin; c0 += 2 * CC) {
    chunk(c0, buf, bA, bB);
    buf ^= 1;
    if (c0 + CC < a.Cin) {
      chunk(c0 + CC, buf, bB, bA);
      buf ^= 1;
    }
  }

  wino_store_tiles<DB>(a, smem, acc, wave, lane, m0, img, img_ok, ty, tx, G::W);
}

typedef WinoGeom<32, 4, 1, 34> WinoG32;
typedef WinoGeom<16, 8, 1, 24> WinoG16;
typedef WinoGeom<8, 8, 2, 12> WinoG8;

// ---------------------------------------------------------------------------------------------------------------
// Variant for exactly 32 input channels (output channels in blocks of 32, one run of workgroups per block), where the channel loop is only four chunks
// long and the kernels above spend more time on what surrounds it (index arithmetic, weight reloads with every
// chunk, filling and draining the pipeline once per 32 tiles) than on the multiplies.  Here the wave's share of the
// transformed weights -- 4 components x 32 channels x 32 output channels = 64 registers a lane, already laid out as
// MFMA A operands -- stays in registers for the life of a PERSISTENT workgroup, which walks over a run of groups of
// 32 tiles: the chunk pipeline (raw chunk n+1 from registers into LDS, barrier, loads of chunk n+3 into the registers
// just freed, transform of chunk n+1 interleaved with the multiplies of chunk n) runs on across group borders, so
// the first chunks of the next group are on their way while the current one is finished.  Loads are issued two
// chunks before they are needed: with two waves per SIMD one chunk of multiplies is shorter than a trip to HBM.
// The epilogue has an LDS area of its own and one barrier; the activation values backward-data needs are requested
// before the last chunk's multiplies.
// FAST selects what is fixed at compile time: 0 nothing (forward or backward-data, any pool, M <= 32, stores under
// their bounds checks); 1 forward with the 2x2 max-pool, 2 backward-data through an activation, 3 forward without a
// pool, all three for M a multiple of 32: every store is then unconditional, so the number of stores between a load and
// its use is a constant and the wait for that load does not have to drain the stores as well.
template <class G, int FAST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv_wino_res_kernel(const ConvWinoArgs a, const int n_groups, const int groups_per_wg) {
  constexpr int CC = WINO_CC, RS = G::RS, LDW = G::LDW, XSZ = CC * RS, NCH = 4, W = G::W;
  static_assert(G::NIMG == 1 && G::REAL <= 256, "a group is a band of one image; one position per thread");
  __shared__ __attribute__((aligned(16))) float smem[2 * XSZ + 8192]; // raw buffers [2][CC * RS]; epilogue [4][2][16][64]
  float *Xr = smem, *Tl = smem + 2 * XSZ;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int HW = a.H * W;
  const int m0 = blockIdx.y * 32; // block of 32 output channels (wider layers: one run of workgroups per block)
  const int g_begin = blockIdx.x * groups_per_wg, g_end = min(n_groups, g_begin + groups_per_wg);
  if (g_begin >= g_end) return;
  const bool fwd = FAST == 0 ? a.bias != nullptr : FAST != 2;
  const bool need_side = FAST == 0 ? (!fwd && a.act) : FAST == 2;
  const int pool = FAST == 0 ? a.pool : (FAST == 1 ? 1 : 0);

  // this lane's tile inside a group
  const int tyl = li / G::TW, tx = li % G::TW;
  const float *pat = Xr + lk * RS + 2 * tyl * LDW + 2 * tx;
  const int r1 = wave == 0 ? 0 : (wave == 2 ? 2 : 1);
  const int r2 = wave == 0 ? 2 : (wave == 1 ? 2 : (wave == 2 ? 1 : 3));
  const float s2 = wave == 1 ? 1.f : -1.f;

  // Epilogue addresses (FAST variants): a uniform pointer per group and accumulator row + the lane's byte offset, so
  // that no 64-bit vector arithmetic is left in the epilogue.  Lane part: output channel 8 wave + 4 lk of the block,
  // tile (tyl, tx) of the band.
  const unsigned lane_o = 4u * (unsigned)((8 * wave + 4 * lk) * HW + (2 * tyl) * W + 2 * tx);
  const unsigned lane_p = 4u * (unsigned)((8 * wave + 4 * lk) * (HW >> 2) + tyl * (W >> 1) + tx);

  // staging: thread tid owns position tid of the haloed band for the 8 channels of a chunk.  The loads are buffer
  // loads: a resource descriptor per band (it starts one pixel row above the band, so lane offsets are never
  // negative; only addresses of real pixels are ever formed from it), the channel in the scalar offset, and a lane
  // offset beyond the descriptor's range for positions that hold no input -- those read as zero without touching
  // memory, so nothing has to be masked on the way to LDS.
  const int s_rr = tid / (W + 2), s_col = tid % (W + 2);
  const bool s_in = tid < G::REAL && (unsigned)(s_col - 1) < (unsigned)W;
  const unsigned s_off = 4u * (unsigned)(s_rr * W + (s_in ? s_col - 1 : 0)); // bytes from the descriptor's base
  const int xl = tid < G::REAL ? s_rr * LDW + s_col : -1;
  const int per = a.H / G::ROWS; // bands per image
  constexpr unsigned OUTSIDE = 0x80000000u;
  struct Grp { __amdgpu_buffer_rsrc_t rs; unsigned xg; int img, row0; };
  auto setup = [&](int g) {
    Grp q;
    q.img = g / per; q.row0 = (g - q.img * per) * G::ROWS;
    const int ih = q.row0 + s_rr - 1;
    q.xg = (s_in && (unsigned)ih < (unsigned)a.H) ? s_off : OUTSIDE;
    const float *base = a.x + (long)q.img * a.Cin * HW + (q.row0 - 1) * W;
    q.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, 4 * (a.Cin * HW + W), 0x00020000);
    return q;
  };

  float xrA[CC], xrB[CC];
  auto fetch_raw = [&](const Grp &q, int c0, float *dst) {
#pragma unroll
    for (int c = 0; c < CC; ++c)
      dst[c] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(q.rs, q.xg, 4 * (c0 + c) * HW, 0));
  };
  auto store_raw = [&](float *xbuf, const float *src) {
    if (xl >= 0) {
#pragma unroll
      for (int c = 0; c < CC; ++c) xbuf[xl + c * RS] = src[c];
    }
  };
  auto transform = [&](const float *xbuf, float (*bv)[4]) {
    const float *p = pat + (xbuf - Xr);
#pragma unroll
    for (int cp = 0; cp < CC / 2; ++cp) {
      const float *q = p + 2 * cp * RS;
      const float2 a0 = *reinterpret_cast<const float2 *>(q + r1 * LDW);
      const float2 a1 = *reinterpret_cast<const float2 *>(q + r1 * LDW + 2);
      const float2 b0 = *reinterpret_cast<const float2 *>(q + r2 * LDW);
      const float2 b1 = *reinterpret_cast<const float2 *>(q + r2 * LDW + 2);
      const float t0 = fmaf(s2, b0.x, a0.x), t1 = fmaf(s2, b0.y, a0.y), t2 = fmaf(s2, b1.x, a1.x), t3 = fmaf(s2, b1.y, a1.y);
      bv[cp][0] = t0 - t2;
      bv[cp][1] = t1 + t2;
      bv[cp][2] = t2 - t1;
      bv[cp][3] = t1 - t3;
    }
  };

  Grp cur = setup(g_begin);
  fetch_raw(cur, 0, xrA);
  fetch_raw(cur, CC, xrB);
  // the wave's weights: wr[jj][channel pair] = u[(4*wave + jj)*Cpad + 2*cp + lk][m0 + li]   (Cpad = 32)
  float wr[4][NCH * CC / 2];
  {
    const float *ub = a.u + ((long)(4 * wave) * a.Cpad + lk) * a.Mpad + m0 + li;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
      for (int cp = 0; cp < NCH * CC / 2; ++cp) wr[jj][cp] = ub[((long)jj * a.Cpad + 2 * cp) * a.Mpad];
  }
  float bias_r[4];
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) bias_r[rr] = fwd ? a.bias[min(m0 + 8 * wave + 4 * lk + rr, a.M - 1)] : 0.f;

  store_raw(Xr, xrA);
  __syncthreads();
  fetch_raw(cur, 2 * CC, xrA);
  float bA[CC / 2][4], bB[CC / 2][4];
  transform(Xr, bA);

  // At the top of a group: its chunk 0 is transformed (bA), chunk 1 sits in xrB, chunk 2 is on its way into xrA.
  f32x16 acc[4];
  for (int g = g_begin; g < g_end; ++g) {
    const Grp nxt = setup(min(g + 1, g_end - 1)); // past the run's last group: re-read it (unused)
    const int img = cur.img, ty = cur.row0 / 2 + tyl;
    const long obase = ((long)img * a.M) * HW + (2 * ty) * W + 2 * tx;
    // the group's origin in the output / activation planes and in the pooled planes (uniform; FAST variants)
    const long og0 = ((long)img * a.M + m0) * HW + (long)cur.row0 * W;
    const long pg0 = ((long)img * a.M + m0) * (HW >> 2) + (long)(cur.row0 >> 1) * (W >> 1);
    float2 sd0[4], sd1[4];

    auto load_side = [&]() {
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        if (FAST != 0) {
          const char *sp = reinterpret_cast<const char *>(a.a_prev + og0 + (long)rr * HW);
          sd0[rr] = *reinterpret_cast<const float2 *>(sp + lane_o);
          sd1[rr] = *reinterpret_cast<const float2 *>(sp + lane_o + 4u * W);
        } else {
          const long o = obase + (long)min(m0 + 8 * wave + 4 * lk + rr, a.M - 1) * HW;
          sd0[rr] = *reinterpret_cast<const float2 *>(a.a_prev + o);
          sd1[rr] = *reinterpret_cast<const float2 *>(a.a_prev + o + W);
        }
      }
    };
    // chunk KC of the group: the chunk after it goes from registers (src_regs) to LDS, the chunk three ahead (chunk
    // c_next of group `from`) is requested into the same registers
    auto chunk = [&](auto kc_, float *xbuf, float *regs, const Grp &from, int c_next, float (*bcur)[4],
                     float (*bnext)[4]) {
      constexpr int KC = decltype(kc_)::value;
      store_raw(xbuf, regs);
      __syncthreads(); // the next raw chunk is in place; every wave has finished reading the buffer written after this
      fetch_raw(from, c_next, regs);
      transform(xbuf, bnext);
      if (KC == NCH - 1 && FAST == 2) load_side();
#pragma unroll
      for (int cp = 0; cp < CC / 2; ++cp)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          if (KC == 0 && cp == 0) {
            const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            acc[jj] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[jj][KC * (CC / 2) + cp], bcur[cp][jj], z, 0, 0, 0);
          } else {
            acc[jj] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[jj][KC * (CC / 2) + cp], bcur[cp][jj], acc[jj], 0, 0, 0);
          }
        }
      // instruction order: the raw loads first, then per multiply step one LDS read and two vector operations of the
      // next chunk's transform (left alone the compiler issues the sixteen multiplies in a row and the transform
      // after them, and a wave's own transform never runs in the shadow of its multiplies)
      if (FAST != 0) { // (the general variant has no registers to spare for the longer live ranges)
        __builtin_amdgcn_sched_group_barrier(0x020, CC, 0);
#pragma unroll
        for (int k = 0; k < 4 * (CC / 2); ++k) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
        }
      }
    };
    chunk(std::integral_constant<int, 0>{}, Xr + XSZ, xrB, cur, 3 * CC, bA, bB);
    chunk(std::integral_constant<int, 1>{}, Xr, xrA, nxt, 0, bB, bA);
    chunk(std::integral_constant<int, 2>{}, Xr + XSZ, xrB, nxt, CC, bA, bB);
    chunk(std::integral_constant<int, 3>{}, Xr, xrA, nxt, 2 * CC, bB, bA);

    // ---- output transform: each wave folds its own row, the four rows meet in LDS (written here, last read four
    // barriers ago), wave w finishes accumulator rows 4w .. 4w+3
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      Tl[((wave * 2 + 0) * 16 + r) * 64 + lane] = acc[0][r] + acc[1][r] + acc[2][r];
      Tl[((wave * 2 + 1) * 16 + r) * 64 + lane] = acc[1][r] - acc[2][r] - acc[3][r];
    }
    if (FAST == 0 && need_side) load_side(); // (the general variant has no registers to hold them any earlier)
    __syncthreads();
    // (the activation is fixed for the launch: one branch per group instead of two around every value)
    auto finish = [&](auto act_c) {
      constexpr int ACT = decltype(act_c)::value;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * wave + rr;
        const int m = m0 + 8 * wave + 4 * lk + rr; // accumulator row r of a lane: 8*(r/4) + 4*lk + r%4
        if (FAST == 0 && m >= a.M) continue;
        float T[4][2];
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int k = 0; k < 2; ++k) T[w][k] = Tl[((w * 2 + k) * 16 + r) * 64 + lane];
        float2 y0, y1;
        y0.x = T[0][0] + T[1][0] + T[2][0];
        y0.y = T[0][1] + T[1][1] + T[2][1];
        y1.x = T[1][0] - T[2][0] - T[3][0];
        y1.y = T[1][1] - T[2][1] - T[3][1];
        const long o = obase + (long)m * HW;
        if (fwd) {
          const float bv = bias_r[rr];
          y0.x = act_apply(ACT, y0.x + bv); y0.y = act_apply(ACT, y0.y + bv);
          y1.x = act_apply(ACT, y1.x + bv); y1.y = act_apply(ACT, y1.y + bv);
          if (pool) {
            const long pg = pg0 + (long)rr * (HW >> 2); // (uniform)
            const long po = ((long)img * a.M + m) * (HW >> 2) + ty * (W >> 1) + tx;
            float *pout = FAST != 0 ? reinterpret_cast<float *>(reinterpret_cast<char *>(a.pool_out + pg) + lane_p) : a.pool_out + po;
            if (pool == 1) {
              float best = y0.x; int bi = 0;
              if (y0.y > best) { best = y0.y; bi = 1; }
              if (y1.x > best) { best = y1.x; bi = 2; }
              if (y1.y > best) { best = y1.y; bi = 3; }
              *pout = best;
              if (FAST != 0) *(a.pool_arg + pg + (lane_p >> 2)) = (uint8_t)bi;
              else a.pool_arg[po] = (uint8_t)bi;
            } else {
              *pout = ((y0.x + y0.y) + (y1.x + y1.y)) * 0.25f;
            }
          }
        } else if (need_side) {
          y0.x *= act_deriv_from_out(ACT, sd0[rr].x); y0.y *= act_deriv_from_out(ACT, sd0[rr].y);
          y1.x *= act_deriv_from_out(ACT, sd1[rr].x); y1.y *= act_deriv_from_out(ACT, sd1[rr].y);
        }
        if (!(fwd && pool == 1)) { // (the plane before a fused max-pool is never read again)
          if (FAST != 0) {
            char *op = reinterpret_cast<char *>(a.out + og0 + (long)rr * HW); // (uniform)
            *reinterpret_cast<float2 *>(op + lane_o) = y0;
            *reinterpret_cast<float2 *>(op + lane_o + 4u * W) = y1;
          } else {
            *reinterpret_cast<float2 *>(a.out + o) = y0;
            *reinterpret_cast<float2 *>(a.out + o + W) = y1;
          }
        }
      }
    };
    if (a.act == DP_ACT_TANH_) finish(std::integral_constant<int, DP_ACT_TANH_>{});
    else if (a.act == DP_ACT_RELU_) finish(std::integral_constant<int, DP_ACT_RELU_>{});
    else finish(std::integral_constant<int, DP_ACT_NONE_>{});
    cur = nxt;
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Weight gradients of a 3x3 / stride-1 / pad-1 layer in the minimal-filtering form with the roles exchanged,
// F(3x3, 2x2): per tile the 3x3 block  G[ky][kx] = sum_{a,b} dy[a][b] xpatch[ky+a][kx+b]  is
//   A^T [ (G' dy G'^T) (.) (B^T xpatch B) ] A    with the same B^T as above and
//   G' = [1 0; 1 1; 1 -1; 0 -1]      A^T = [1 .5 .5 0; 0 .5 -.5 0; 0 .5 .5 1]
// (the transposed algorithm of F(2x2, 3x3)).  The 16 components are linear in the products, so they are summed over
// tiles and transformed back once per example or once per run of examples: 16 instead of 36 multiplies per tile and
// (d, c) pair.  MFMA: M = output channel d (32*DB per workgroup), N = input channel c (32 per workgroup), K = tile
// pair; wave w owns transform row w.  Every lane transforms its own operands from the raw planes in LDS (lanes walk
// channels; the planes sit at channel strides = 2 mod 4 words, which puts the 16 lanes served together on 32
// different banks with 8-byte reads).  Two modes:
// NORM (the norm pass, Section 1 item 2a: one gradient per example): after the last tile of an example the 16
// components are transformed back, the example's gradient goes to its row of the stored-gradient buffer in the
// parameter layout (W[d][c][3][3], then bias[d]), its squares are reduced in a fixed order into the example's slot of
// this channel block, and the accumulators start again at zero.
// Otherwise (sum over a run of examples, item 3): dy is scaled by the example's clip factor while it is staged, the
// components are summed over the whole run and transformed back once into one split-K partial (parameter layout; the
// bias gradient, the sum of the scaled dy, is accumulated while staging by the workgroups of the first channel block).
// A unit of work is 16 tiles = 64 output pixels: TR tile rows of a W-wide plane (W = 32: one tile row, 16: two, 8:
// the whole 8x8 plane); a unit's x band carries its own halo rows from the neighbouring bands (zero rows outside
// the plane) and zero halo columns, all rewritten with every unit; one barrier per unit, the next unit's planes in
// registers meanwhile.  One workgroup = one block of 32 input channels x one block of 32*DB output channels, for a
// run of examples.
struct ConvWinoWgUnitArgs {
  const float *x;      // layer input [B, C, H, W]
  const float *dy;     // [B, D, H, W]
  const float *scale;  // sum mode: clip factors s[b] (a vector of ones when nothing is clipped)
  float *slots;        // NORM: squared norms, slots[(slot0 + channel block) * slot_stride + b]
  float *gstore;       // NORM: [B][gstride], per-example gradients in the parameter layout
  float *part;         // sum mode: the run blockIdx.y writes part + blockIdx.y * part_stride
  long slot_stride, gstride, part_stride;
  int slot0;
  int B, C, D, H;      // C a multiple of 32; D a multiple of 32 * DB (NORM: D = 32 * DB), blockIdx.z = block of output
                       // channels; H a multiple of 2 * TR
  int ex_per_block;
};

template <int W_, int TR_, int DB, bool NORM>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv_wino_wgrad_unit_kernel(const ConvWinoWgUnitArgs a) {
  constexpr int W = W_, TW = W / 2, XR = 2 * TR_ + 2, LDW = W + 2;
  constexpr int XS = ((XR * LDW + 3) / 4) * 4 + 2, DS = 66; // channel strides = 2 mod 4: conflict-free 8-byte lane reads
  constexpr int XSZ = 32 * XS, DSZ = 32 * DB * DS, STAGE = XSZ + DSZ;
  constexpr int SMEM = 2 * STAGE > 12288 ? 2 * STAGE : 12288;
  constexpr int XITEMS = 32 * XR * (W / 4), XN = (XITEMS + 255) / 256, DN = 2 * DB;
  constexpr int HITEMS = 32 * XR, HN = (HITEMS + 255) / 256; // halo-column rows
  static_assert(TW * TR_ == 16, "a unit is 16 tiles");
  __shared__ __attribute__((aligned(16))) float smem[SMEM];
  __shared__ float red[4];
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c0 = blockIdx.x * 32, d0 = blockIdx.z * 32 * DB; // (the norm pass runs with one block of output channels)
  const int b0 = blockIdx.y * a.ex_per_block, b1 = min(b0 + a.ex_per_block, a.B);
  const int UPI = (a.H / 2) / TR_; // units per image
  const int HW = a.H * W;

  // staging items of a unit: x float4 (channel, band row, column group), dy float4 (channel, 16-byte part of the 64 pixels)
  int xs_l[XN], xs_rr[XN];
  unsigned xs_g[XN];
#pragma unroll
  for (int j = 0; j < XN; ++j) {
    const int q = tid + j * 256;
    const int ch = q / (XR * (W / 4)), rem = q % (XR * (W / 4)), rr = rem / (W / 4), qq = rem % (W / 4);
    xs_l[j] = q < XITEMS ? ch * XS + rr * LDW + 1 + 4 * qq : -1;
    xs_rr[j] = rr;
    xs_g[j] = 4u * (unsigned)(ch * HW + 4 * qq); // + row * W per unit
  }
  // (item j of a thread: channel (tid >> 4) + 16 j, the same part: one LDS and one memory offset serve all DN items)
  const int ds_l0 = XSZ + (tid >> 4) * DS + 4 * (tid & 15);
  const unsigned ds_g0 = 4u * (unsigned)((tid >> 4) * HW + 4 * (tid & 15));
  float4 xv[XN], dv[DN];
  float sv = 1.f; // clip factor of the example whose unit is in the registers
  // unit u = example u / UPI, band u % UPI
  auto fetch = [&](int b, int band) {
    if (!NORM) sv = a.scale[b];
    const int r0 = band * 2 * TR_;
    const float *xb = a.x + ((long)b * a.C + c0) * HW;
    const float *db = a.dy + ((long)b * a.D + d0) * HW + (long)r0 * W;
#pragma unroll
    for (int j = 0; j < XN; ++j) {
      const int ih = r0 - 1 + xs_rr[j];
      const bool ok = (XITEMS % 256 == 0 || xs_l[j] >= 0) && (unsigned)ih < (unsigned)a.H;
      const float4 v = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(xb) + (ok ? xs_g[j] + 4u * (unsigned)(ih * W) : 0u));
      xv[j] = ok ? v : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int j = 0; j < DN; ++j) dv[j] = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(db + (long)j * 16 * HW) + ds_g0);
  };
  const bool bias_block = blockIdx.x == 0; // the bias gradient is taken by the workgroups of the first channel block
  float bsum[DN];
#pragma unroll
  for (int j = 0; j < DN; ++j) bsum[j] = 0.f;
  auto store = [&](float *st) {
#pragma unroll
    for (int j = 0; j < XN; ++j)
      if (XITEMS % 256 == 0 || xs_l[j] >= 0) { // (whole rounds of the workgroup: every item is real)
        float *p = st + xs_l[j];
        p[0] = xv[j].x; p[1] = xv[j].y; p[2] = xv[j].z; p[3] = xv[j].w;
      }
#pragma unroll
    for (int j = 0; j < HN; ++j) { // zero halo columns of every band row
      const int q = tid + j * 256;
      if (q < HITEMS) {
        float *p = st + (q / XR) * XS + (q % XR) * LDW;
        p[0] = 0.f; p[W + 1] = 0.f;
      }
    }
#pragma unroll
    for (int j = 0; j < DN; ++j) {
      const float4 v = NORM ? dv[j] : make_float4(dv[j].x * sv, dv[j].y * sv, dv[j].z * sv, dv[j].w * sv);
      if (bias_block) bsum[j] += (v.x + v.y) + (v.z + v.w);
      float *p = st + ds_l0 + j * 16 * DS;
      *reinterpret_cast<float2 *>(p) = make_float2(v.x, v.y);
      *reinterpret_cast<float2 *>(p + 2) = make_float2(v.z, v.w);
    }
  };

  const int r1 = wave == 0 ? 0 : (wave == 2 ? 2 : 1);
  const int r2 = wave == 0 ? 2 : (wave == 1 ? 2 : (wave == 2 ? 1 : 3));
  const float s2 = wave == 1 ? 1.f : -1.f;
  const float ga = wave == 3 ? 0.f : 1.f;
  const float gb = wave == 0 ? 0.f : (wave == 1 ? 1.f : -1.f);
  const float *xlane = smem + li * XS + 2 * lk;
  const float *dlane = smem + XSZ + li * DS + 2 * lk;

  // (norm mode: the first tile pair of an example multiplies into a zero accumulator, so nothing is cleared here or
  // between examples)
  f32x16 acc[4][DB];
  if (!NORM) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jj][i][r] = 0.f;
  }

  float *Tl = smem; // epilogue: [wave][k][r][lane]
  if (b0 < b1) fetch(b0, 0);
  int stage = 0;
  for (int b = b0; b < b1; ++b) {
    for (int band = 0; band < UPI; ++band) {
      store(smem + stage * STAGE);
      __syncthreads(); // the unit is in place; every wave has finished reading the stage the next store overwrites
      {
        int nb = b, nband = band + 1;
        if (nband == UPI) { nband = 0; nb = min(b + 1, b1 - 1); } // (past the end: a unit is read again, unused)
        fetch(nb, nband);
      }
      const float *xp = xlane + stage * STAGE, *dp = dlane + stage * STAGE;
      // Tile pairs in a three-deep software pipeline, spelled out for the scheduler: while the MFMAs of pair kp run,
      // the operands of pair kp + 1 are transformed and the raw values of pair kp + 2 are read from LDS (left to
      // itself the compiler reads, waits, transforms and then issues two pairs' MFMAs in a row, and the matrix unit
      // idles through every read and transform).
      float2 rx[2][4], rd[2][DB][2];
      float bv[2][4], av[2][DB][4];
      auto rd_raw = [&](int kp, float2 (&x4)[4], float2 (&d2)[DB][2]) {
        const int tyl = (2 * kp) / TW, cx = 2 * ((2 * kp) % TW);
        x4[0] = *reinterpret_cast<const float2 *>(xp + (2 * tyl + r1) * LDW + cx);
        x4[1] = *reinterpret_cast<const float2 *>(xp + (2 * tyl + r1) * LDW + cx + 2);
        x4[2] = *reinterpret_cast<const float2 *>(xp + (2 * tyl + r2) * LDW + cx);
        x4[3] = *reinterpret_cast<const float2 *>(xp + (2 * tyl + r2) * LDW + cx + 2);
#pragma unroll
        for (int i = 0; i < DB; ++i) {
          d2[i][0] = *reinterpret_cast<const float2 *>(dp + 32 * i * DS + (2 * tyl) * W + cx);
          d2[i][1] = *reinterpret_cast<const float2 *>(dp + 32 * i * DS + (2 * tyl + 1) * W + cx);
        }
      };
      auto transform = [&](const float2 (&x4)[4], const float2 (&d2)[DB][2], float (&b4)[4], float (&a4)[DB][4]) {
        const float t0 = fmaf(s2, x4[2].x, x4[0].x), t1 = fmaf(s2, x4[2].y, x4[0].y);
        const float t2 = fmaf(s2, x4[3].x, x4[1].x), t3 = fmaf(s2, x4[3].y, x4[1].y);
        b4[0] = t0 - t2; b4[1] = t1 + t2; b4[2] = t2 - t1; b4[3] = t1 - t3;
#pragma unroll
        for (int i = 0; i < DB; ++i) {
          const float e0 = fmaf(gb, d2[i][1].x, ga * d2[i][0].x), e1 = fmaf(gb, d2[i][1].y, ga * d2[i][0].y);
          a4[i][0] = e0; a4[i][1] = e0 + e1; a4[i][2] = e0 - e1; a4[i][3] = e1; // (component 3 is -e1: the sign is taken back in the inverse transform)
        }
      };
      rd_raw(0, rx[0], rd[0]);
      rd_raw(1, rx[1], rd[1]);
      transform(rx[0], rd[0], bv[0], av[0]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kp = 0; kp < 8; ++kp) {
        const int cur = kp & 1, nxt = cur ^ 1;
        if (kp + 1 < 8) transform(rx[nxt], rd[nxt], bv[nxt], av[nxt]);
        if (kp + 2 < 8) rd_raw(kp + 2, rx[cur], rd[cur]);
        if (NORM && kp == 0 && band == 0) {
          // the unit opens an example: its first multiplies start from zero
          const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int i = 0; i < DB; ++i) acc[jj][i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i][jj], bv[cur][jj], z, 0, 0, 0);
        } else {
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int i = 0; i < DB; ++i) acc[jj][i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i][jj], bv[cur][jj], acc[jj][i], 0, 0, 0);
        }
        if (!(NORM && kp == 0)) {
#pragma unroll
          for (int g = 0; g < 4 * DB; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // one LDS read
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0); // three vector-ALU instructions
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      stage ^= 1;
    }
    if (!NORM) continue;
    // the example is complete: transform back, store, reduce the squares
    float *gout = a.gstore + (long)b * a.gstride;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < DB; ++i) {
      __syncthreads(); // the last unit has been read by every wave (the area below lies over both stages)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float m0 = acc[0][i][r], m1 = acc[1][i][r], m2 = acc[2][i][r], m3 = acc[3][i][r];
        const float hs = 0.5f * (m1 + m2), hd = 0.5f * (m1 - m2);
        Tl[((wave * 3 + 0) * 16 + r) * 64 + lane] = m0 + hs;
        Tl[((wave * 3 + 1) * 16 + r) * 64 + lane] = hd;
        Tl[((wave * 3 + 2) * 16 + r) * 64 + lane] = hs - m3;
      }
      __syncthreads();
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int r = 4 * wave + rr;
        const int d = 32 * i + 8 * wave + 4 * lk + rr;
        float *o = gout + ((long)d * a.C + c0 + li) * 9;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          const float T0 = Tl[((0 * 3 + k) * 16 + r) * 64 + lane], T1 = Tl[((1 * 3 + k) * 16 + r) * 64 + lane];
          const float T2 = Tl[((2 * 3 + k) * 16 + r) * 64 + lane], T3 = Tl[((3 * 3 + k) * 16 + r) * 64 + lane];
          const float hs = 0.5f * (T1 + T2), hd = 0.5f * (T1 - T2);
          const float y0 = T0 + hs, y1 = hd, y2 = hs + T3;
          o[0 * 3 + k] = y0; o[1 * 3 + k] = y1; o[2 * 3 + k] = y2;
          sq += y0 * y0 + y1 * y1 + y2 * y2;
        }
      }
    }
    // bias gradient of the example (first channel block only): 16 threads share an output channel
#pragma unroll
    for (int j = 0; j < DN; ++j) {
      float s = bsum[j];
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
      if (blockIdx.x == 0 && (tid & 15) == 0) {
        gout[(long)a.D * a.C * 9 + (tid >> 4) + 16 * j] = s;
        sq += s * s;
      }
      bsum[j] = 0.f;
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) sq += __shfl_xor(sq, o, 64);
    if (lane == 0) red[wave] = sq;
    __syncthreads(); // also: every wave is done with the epilogue area before the next unit is stored over it
    if (tid == 0) a.slots[(long)(a.slot0 + blockIdx.x) * a.slot_stride + b] = (red[0] + red[1]) + (red[2] + red[3]);
  }
  if (NORM) return;
  // sum mode: one partial in the parameter layout
  float *out = a.part + (long)blockIdx.y * a.part_stride;
#pragma unroll
  for (int i = 0; i < DB; ++i) {
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float m0 = acc[0][i][r], m1 = acc[1][i][r], m2 = acc[2][i][r], m3 = acc[3][i][r];
      const float hs = 0.5f * (m1 + m2), hd = 0.5f * (m1 - m2);
      Tl[((wave * 3 + 0) * 16 + r) * 64 + lane] = m0 + hs;
      Tl[((wave * 3 + 1) * 16 + r) * 64 + lane] = hd;
      Tl[((wave * 3 + 2) * 16 + r) * 64 + lane] = hs - m3;
    }
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int r = 4 * wave + rr;
      const int d = d0 + 32 * i + 8 * wave + 4 * lk + rr;
      float *o = out + ((long)d * a.C + c0 + li) * 9;
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const float T0 = Tl[((0 * 3 + k) * 16 + r) * 64 + lane], T1 = Tl[((1 * 3 + k) * 16 + r) * 64 + lane];
        const float T2 = Tl[((2 * 3 + k) * 16 + r) * 64 + lane], T3 = Tl[((3 * 3 + k) * 16 + r) * 64 + lane];
        const float hs = 0.5f * (T1 + T2), hd = 0.5f * (T1 - T2);
        o[0 * 3 + k] = T0 + hs; o[1 * 3 + k] = hd; o[2 * 3 + k] = hs + T3;
      }
    }
  }
  if (blockIdx.x == 0) {
#pragma unroll
    for (int j = 0; j < DN; ++j) {
      float s = bsum[j];
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o, 64);
      if ((tid & 15) == 0) out[(long)a.D * a.C * 9 + d0 + (tid >> 4) + 16 * j] = s;
    }
  }
}

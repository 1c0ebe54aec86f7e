// Networks that are one or two dense layers: the whole per-example part of the private step in one launch.
//
// For a dense layer the example's gradient is the outer product a_i (x) delta_i (plus delta_i for the bias), so
// its norm is sqrt((||a_i||^2 + 1) ||delta_i||^2) (Section 1: the per-example norm of fully connected layers)
// and everything up to the clip factor depends on that example alone: logits, loss gradient, norm and clip factor
// are computed by the wave that owns the example, and the workgroup then adds s_i a_i (x) delta_i of its examples
// into one partial of the clipped sum (Section 1, items 2-3).  The final write (finalize_kernel) sums the partials
// in a fixed order and adds the noise.  Two launches per step for softmax regression instead of four.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>

#include "gemm_tile.h" // FastDiv
#include "kernels_misc.h" // act_apply, act_deriv_from_out

#define DENSE1_THREADS 1024  // 16 waves: one row of the [d_in + 1][N] tensor per thread
#define DENSE1_MAX_IN 1023   // input features (+ the bias row): one row per thread
#define DENSE1_MAX_CLASSES 15
#define DENSE1_MAX_LDS_WORDS 14800 // in_features * (classes padded to 4 / 10 / 15 + DENSE1_EX): W transposed and one
                                   // group of inputs in 64 KB of LDS
#define DENSE1_EX 4          // examples per group
#define DENSE1_MAX_TILES 256 // partials of the clipped sum (workgroups)

struct Dense1Args {
  const float *x;    // [B][d_in]
  const float *W;    // [d_in][N]
  const float *bias; // [N]
  const int *y;      // [B]
  float *part;       // [tiles][dense1_part_stride]: partial clipped sums in the parameter layout (W then bias)
  float *norms;      // [B] unclipped norms (may be null)
  float *s;          // [B] clip factors (may be null)
  float *delta;      // [B][N] loss gradient (may be null)
  int B, d_in, N;
  int groups;        // groups of DENSE1_EX examples per workgroup
  float C;           // clip norm (private step)
  int priv;          // 0: plain sum (every factor 1)
  FastDiv dN, dD;    // division by N, by d_in
};

static inline __host__ __device__ int dense1_ldx(int d_in) { return (d_in + 3) & ~3; }
static inline __host__ __device__ int dense1_ldw(int d_in) { const int q = (d_in + 3) >> 2; return 4 * (q | 1); }
// partial rows start on 16-byte boundaries (the final write reads them with 16-byte loads)
static inline __host__ __device__ long dense1_part_stride(int d_in, int N) { return ((long)(d_in + 1) * N + 3) & ~3l; }
static inline int dense1_ncp(int n_classes) { return n_classes <= 4 ? 4 : (n_classes <= 10 ? 10 : 15); }
static inline bool dense1_fits(int d_in, int n_classes) {
  return d_in >= 1 && n_classes >= 1 && d_in <= DENSE1_MAX_IN && n_classes <= DENSE1_MAX_CLASSES &&
         (long)d_in * (dense1_ncp(n_classes) + DENSE1_EX) <= DENSE1_MAX_LDS_WORDS;
}

// Tiling shared by every caller: at most max_tiles partial rows, whole groups of DENSE1_EX examples per workgroup.
static inline void dense1_tiling(int B, int max_tiles, int *groups, int *tiles) {
  const int ngroups = (B + DENSE1_EX - 1) / DENSE1_EX;
  int t = max_tiles < DENSE1_MAX_TILES ? max_tiles : DENSE1_MAX_TILES;
  if (t < 1) t = 1;
  const int g = ngroups > 0 ? (ngroups + t - 1) / t : 1;
  *groups = g;
  *tiles = ngroups > 0 ? (ngroups + g - 1) / g : 0;
}

// One workgroup of 16 waves per run of groups of four examples.  Per group:
//   1. the four input rows go to LDS (the next group's are requested meanwhile);
//   2. lane (e, j) of every wave multiplies example e with class j's weights over the wave's sixteenth of the
//      features (lane (e, 15): with the example itself, for ||x_e||^2); the sixteen partial sums meet in LDS -- no
//      cross-lane reduction of long vectors anywhere;
//   3. wave 0 finishes the four examples: softmax, loss gradient, norm (dense identity), clip factor;
//   4. thread k adds s_e x_e[k] delta_e (k = d_in: the bias row, x = 1) of the four examples to its row of the
//      workgroup's partial clipped sum, which stays in registers over the whole run.
template <int NCP>
__global__ __launch_bounds__(DENSE1_THREADS) void dense1_fused_kernel(const Dense1Args a) {
  extern __shared__ float lds[];
  const int d_in = a.d_in, N = a.N;
  // rows of 4-float quads (16-byte LDS reads); an odd number of quads per weight row, so that the sixteen rows a
  // 16-byte read touches start in different banks
  const int ldx = dense1_ldx(d_in), ldw = dense1_ldw(d_in);
  float *xs = lds;                    // [DENSE1_EX][ldx]: the group's inputs, zero beyond d_in
  float *wt = xs + DENSE1_EX * ldx;   // [NCP][ldw]: W transposed, zero rows for the padding classes, zero beyond d_in
  float *zp = wt + NCP * ldw;         // [16 waves][64 lanes]: partial dot products
  float *dl = zp + 16 * 64;           // [DENSE1_EX][NCP]: s_e * delta_e
  float *bs = dl + DENSE1_EX * NCP;   // [16]: bias, -inf for the padding classes (their softmax term is 0)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int e = lane >> 4, jj = lane & 15;
  float acc[NCP];
#pragma unroll
  for (int j = 0; j < NCP; ++j) acc[j] = 0.f;

  // the first group's inputs (HBM: the longest latency) are requested before the weights (L2)
  const long x_total = (long)a.B * d_in;
  const int x_group = DENSE1_EX * d_in; // the rows of a group's examples are contiguous
  float xv[4];
  {
    const long base = (long)blockIdx.x * a.groups * x_group;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const int i = tid + DENSE1_THREADS * n;
      const long g = base + i;
      xv[n] = a.x[(i < x_group && g < x_total) ? g : 0]; // always a valid address; masked when stored
    }
  }
  // every other global read of the prologue is in flight before the first one is waited for: the weights (L2),
  // the bias and the first group's labels
  const int b_first = blockIdx.x * a.groups * DENSE1_EX + e;
  int yv = a.y[b_first < a.B ? b_first : 0];
  const float bv = a.bias[tid < N ? tid : 0];
  {
    const int w_total = d_in * N;
    float wv[16];
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      const int i = tid + DENSE1_THREADS * n;
      wv[n] = a.W[i < w_total ? i : 0];
    }
      // zero first: the padding rows, and the tail of every row beyond d_in (the products below run over whole quads)
    for (int i = tid; i < NCP * ldw; i += DENSE1_THREADS) wt[i] = 0.f;
    for (int i = tid; i < DENSE1_EX * ldx; i += DENSE1_THREADS) xs[i] = 0.f;
    __syncthreads();
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      const int i = tid + DENSE1_THREADS * n;
      if (i < w_total) {
        const int k = (int)a.dN.div((unsigned)i), j = i - k * N;
        wt[j * ldw + k] = wv[n];
      }
    }
  }
  if (tid < 16) bs[tid] = tid < N ? bv : -INFINITY;
  // the wave's sixteenth of the features, in whole quads
  const int kc = ((ldx >> 2) + 15) >> 4;
  const int k0 = 4 * wave * kc, k1 = min(ldx, k0 + 4 * kc);

  for (int grp = 0; grp < a.groups; ++grp) {
    const long gbase = ((long)blockIdx.x * a.groups + grp) * x_group;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const int i = tid + DENSE1_THREADS * n;
      if (i < x_group) {
        const int q = (int)a.dD.div((unsigned)i); // example of the group, feature i - q * d_in
        xs[q * ldx + (i - q * d_in)] = (gbase + i < x_total) ? xv[n] : 0.f;
      }
    }
    __syncthreads();
    const int yy = yv;
    if (grp + 1 < a.groups) {
      const long base = gbase + x_group;
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const int i = tid + DENSE1_THREADS * n;
        const long g = base + i;
        xv[n] = a.x[(i < x_group && g < x_total) ? g : 0];
      }
      const int bn = (blockIdx.x * a.groups + grp + 1) * DENSE1_EX + e;
      yv = a.y[bn < a.B ? bn : 0];
    }
    // ---- 2. partial dot products
    {
      const float *ap = xs + e * ldx;
      const float *bp = jj < NCP ? wt + jj * ldw : ap; // lane 15 of an example: the example with itself
      float z0 = 0.f, z1 = 0.f;
#pragma unroll 4
      for (int k = k0; k < k1; k += 4) {
        const float4 u = *reinterpret_cast<const float4 *>(ap + k), v = *reinterpret_cast<const float4 *>(bp + k);
        z0 = fmaf(u.x, v.x, z0); z1 = fmaf(u.y, v.y, z1); z0 = fmaf(u.z, v.z, z0); z1 = fmaf(u.w, v.w, z1);
      }
      zp[wave * 64 + lane] = z0 + z1;
    }
    __syncthreads();
    // ---- 3. wave 0: the four examples' loss gradients, norms and clip factors
    if (wave == 0) {
      float z = 0.f;
#pragma unroll
      for (int w = 0; w < 16; ++w) z += zp[w * 64 + lane];
      const int b = (blockIdx.x * a.groups + grp) * DENSE1_EX + e;
      const bool valid = b < a.B;
      const float sa = __shfl(z, (lane & 48) + 15, 64); // ||x_e||^2
      z = jj < 15 ? z + bs[jj] : -INFINITY;            // logits; padding lanes drop out of the softmax
      float mx = z;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      const float ex = expf(z - mx);
      float se = ex;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
      const float dv = ex / se - (jj == yy ? 1.f : 0.f); // delta_e[jj] (padding lanes: 0)
      float sd = dv * dv;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) sd += __shfl_xor(sd, o, 64);
      const float n = sqrtf((sa + 1.f) * sd);
      const float sc = a.priv ? fminf(1.f, a.C / n) : 1.f; // n == 0: C/0 = +inf -> 1
      if (jj < NCP) dl[e * NCP + jj] = valid ? sc * dv : 0.f;
      if (valid && jj == 0) {
        if (a.norms) a.norms[b] = n;
        if (a.s) a.s[b] = sc;
      }
      if (valid && a.delta && jj < N) a.delta[(long)b * N + jj] = dv;
    }
    __syncthreads();
    // ---- 4. the group's examples added to the partial: thread = row tid of the [d_in + 1][N] tensor
    if (tid <= d_in) {
#pragma unroll
      for (int q = 0; q < DENSE1_EX; ++q) {
        const float v = tid < d_in ? xs[q * ldx + tid] : 1.f; // the bias row multiplies a constant 1
#pragma unroll
        for (int j = 0; j < NCP; ++j) acc[j] = fmaf(v, dl[q * NCP + j], acc[j]);
      }
    }
    __syncthreads();
  }
  if (tid <= d_in) {
    float *pr = a.part + (long)blockIdx.x * dense1_part_stride(d_in, N) + (long)tid * N;
#pragma unroll
    for (int j = 0; j < NCP; ++j)
      if (j < N) pr[j] = acc[j];
  }
}

// Launches the kernel above on `st`; returns the number of partial rows written (0 for an empty batch).
static inline int launch_dense1_fused(hipStream_t st, Dense1Args a, int max_tiles) {
  int groups = 1, tiles = 0;
  dense1_tiling(a.B, max_tiles, &groups, &tiles);
  if (tiles == 0) return 0;
  a.groups = groups;
  a.dN.init(a.N);
  a.dD.init(a.d_in);
  dim3 grid(tiles), block(DENSE1_THREADS);
  const int ncp = dense1_ncp(a.N);
  const size_t smem = sizeof(float) * ((size_t)DENSE1_EX * dense1_ldx(a.d_in) + (size_t)ncp * dense1_ldw(a.d_in) + 16 * 64 +
                                       DENSE1_EX * ncp + 16);
  if (ncp == 4) hipLaunchKernelGGL(dense1_fused_kernel<4>, grid, block, smem, st, a);
  else if (ncp == 10) hipLaunchKernelGGL(dense1_fused_kernel<10>, grid, block, smem, st, a);
  else hipLaunchKernelGGL(dense1_fused_kernel<15>, grid, block, smem, st, a);
  return tiles;
}

// ---------------------------------------------------------------------------------------------------------------
// Two dense layers (hidden layer with an activation, then the logits).  The hidden layer's forward product is a
// batch-wide contraction and stays a launch of its own; everything between it and the two clipped sums depends on
// one example alone and runs here, one workgroup of 16 waves per run of groups of four examples:
//   A. hidden activations a1 = act(sum of the forward split-K partials + b1) into LDS (or read as they are);
//      partial sums of ||x_e||^2;
//   B. logits by the lane (e, j) scheme of dense1_fused_kernel over sixteenths of the hidden units, lane (e, 15)
//      taking ||a1_e||^2; wave 0 finishes softmax, delta2 and the logit layer's squared norm (dense identity);
//   C. delta1 = act'(a1) * (W2 delta2), its squared norm and the hidden layer's squared norm, the clip factor;
//      s_e * delta1 goes to memory for the hidden layer's clipped sum (a plain contraction afterwards);
//   D. thread h adds s_e a1_e[h] delta2_e (h = H: the bias row) of the four examples to its row of the
//      workgroup's partial of the logit layer's clipped sum.
struct Dense2Args {
  const float *x;      // [B][d_in]
  const float *hpart;  // forward partials of the hidden layer [ns][hstride] (ns > 0), or its finished output (ns = 0)
  long hstride; int ns;
  const float *b1;     // [H]
  const float *W2;     // [H][N]
  const float *b2;     // [N]
  const int *y;        // [B]
  float *sdelta1;      // [B][H]: s_e * delta1_e
  float *part2;        // [tiles][dense1_part_stride(H, N)]
  float *norms, *s;    // [B] (may be null)
  int B, d_in, H, N, act;
  int groups;
  float C; int priv;
  FastDiv dN;
  // head = 1: the two layers close a deeper network.  The clip factor is not known yet (the layers below add to the
  // norm), so the kernel stops after phase C: it leaves both layers' squared norms in their slots, delta1 unscaled in
  // sdelta1, the hidden activations in a1_out (when they arrived as partials) and delta2 in delta2_out for the
  // clipped sums that follow once the clip factors exist.
  // head = 2: a two-layer network whose logit layer's clipped sum is a contraction of its own, like the hidden
  // layer's: the kernel stops after phase C as well, with the clip factor applied: s * delta1 in sdelta1 and
  // s * delta2 in delta2_out, in rows of 16 floats (zero beyond N).
  int head;
  float *slot1, *slot2; // [B] squared norms of the hidden / logit layer's gradient (may be null)
  float *a1_out;        // [B][H] or null
  float *delta2_out;    // [B][d2_ld] (head = 1), [B][16] (head = 2)
  int d2_ld;            // head = 1: row length of delta2_out, N or 16 (zero beyond N)
};

template <int NCP>
__global__ __launch_bounds__(DENSE1_THREADS) void dense2_mid_kernel(const Dense2Args a) {
  extern __shared__ float lds[];
  const int H = a.H, N = a.N, d_in = a.d_in;
  const int ldh = dense1_ldx(H), ldw = dense1_ldw(H);
  float *a1s = lds;                   // [DENSE1_EX][ldh]: hidden activations, zero beyond H
  float *wt = a1s + DENSE1_EX * ldh;  // [NCP][ldw]: W2 transposed, zero rows / tails as in dense1_fused_kernel
  float *zp = wt + NCP * ldw;         // [16 waves][64 lanes]
  float *d2 = zp + 16 * 64;           // [DENSE1_EX][16]: delta2, then s * delta2
  float *bs = d2 + DENSE1_EX * 16;    // [16]: b2, -inf for the padding classes
  float *red = bs + 16;               // [16 waves][2]: partial ||delta1||^2, ||x||^2
  float *n2s = red + 32;              // [DENSE1_EX]: squared norm of the logit layer's gradient
  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
  const int q = wave >> 2; // phases A and C: the wave's example of the group
  float acc[NCP];
#pragma unroll
  for (int j = 0; j < NCP; ++j) acc[j] = 0.f;

  // What a group reads from memory -- its rows of the hidden layer's output and of x, its labels -- is requested one
  // group ahead (the first group's before W2 is staged), so that no phase starts with a round trip to memory.
  float hp[4], xv[4];
  int yv;
  auto request = [&](int grp, float (&hp_)[4], float (&xv_)[4], int &yv_) {
    const int b0 = (blockIdx.x * a.groups + grp) * DENSE1_EX, hh = tid0 & 255;
    const int bq = min(b0 + q, a.B - 1);
    const float *hr = a.hpart + (long)bq * H, *xr = a.x + (long)bq * d_in;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int h = hh + 256 * i;
      hp_[i] = hr[h < H ? h : 0];
      xv_[i] = xr[h < d_in ? h : 0];
    }
    yv_ = a.y[min(b0 + ((tid0 & 63) >> 4), a.B - 1)];
  };
  request(0, hp, xv, yv);
  const float bv = a.b2[tid0 < N ? tid0 : 0];
  {
    const int w_total = H * N;
    float wv[16];
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      const int i = tid0 + DENSE1_THREADS * n;
      wv[n] = a.W2[i < w_total ? i : 0];
    }
    for (int i = tid0; i < NCP * ldw; i += DENSE1_THREADS) wt[i] = 0.f;
    for (int i = tid0; i < DENSE1_EX * ldh; i += DENSE1_THREADS) a1s[i] = 0.f;
    __syncthreads();
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      const int i = tid0 + DENSE1_THREADS * n;
      if (i < w_total) {
        const int k = (int)a.dN.div((unsigned)i), j = i - k * N;
        wt[j * ldw + k] = wv[n];
      }
    }
  }
  if (tid0 < 16) bs[tid0] = tid0 < N ? bv : -INFINITY;
  float b1v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) b1v[i] = a.b1[(tid0 & 255) + 256 * i < H ? (tid0 & 255) + 256 * i : 0];
  const int kc = ((ldh >> 2) + 15) >> 4;
  const int k0 = 4 * wave * kc, k1 = min(ldh, k0 + 4 * kc);

  for (int grp = 0; grp < a.groups; ++grp) {
    // indices re-derived from an opaque copy of the thread index per group: the compiler otherwise keeps the
    // addresses of every phase alive across the loop and spills (and every barrier waits for scratch traffic)
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, e = lane >> 4, jj = lane & 15, hh = tid & 255;
    const int b0 = (blockIdx.x * a.groups + grp) * DENSE1_EX;
    const int bq = b0 + q;            // this thread's example in phases A and C (wave-uniform)
    const bool vq = bq < a.B;
    // ---- A. hidden activations of example bq, units hh + 256 i; ||x||^2 partial
    float a1v[4];
    {
      const long row = (long)(vq ? bq : 0) * H;
      if (a.ns > 0) {
        float pre[4] = {hp[0], hp[1], hp[2], hp[3]}; // (partial 0; the sum runs in the order of the partials)
        for (int s = 1; s < a.ns; ++s) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int h = hh + 256 * i;
            pre[i] += a.hpart[s * a.hstride + row + (h < H ? h : 0)];
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) a1v[i] = act_apply(a.act, pre[i] + b1v[i]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) a1v[i] = hp[i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int h = hh + 256 * i;
        if (h < H) a1s[q * ldh + h] = vq ? a1v[i] : 0.f;
      }
    }
    float sx = 0.f;
    {
#pragma unroll
      for (int i = 0; i < 4; ++i) sx = fmaf(hh + 256 * i < d_in ? xv[i] : 0.f, xv[i], sx);
      const float *xr = a.x + (long)(vq ? bq : 0) * d_in;
      for (int k = hh + 1024; k < d_in; k += 256) { const float v = xr[k]; sx = fmaf(v, v, sx); }
    }
    const int yy = yv;
    if (grp + 1 < a.groups) request(grp + 1, hp, xv, yv);
    __syncthreads();
    // ---- B. logits (partial dot products over the wave's sixteenth of the hidden units)
    {
      const float *ap = a1s + e * ldh;
      const float *bp = jj < NCP ? wt + jj * ldw : ap;
      float z0 = 0.f, z1 = 0.f;
#pragma unroll 4
      for (int k = k0; k < k1; k += 4) {
        const float4 u = *reinterpret_cast<const float4 *>(ap + k), v = *reinterpret_cast<const float4 *>(bp + k);
        z0 = fmaf(u.x, v.x, z0); z1 = fmaf(u.y, v.y, z1); z0 = fmaf(u.z, v.z, z0); z1 = fmaf(u.w, v.w, z1);
      }
      zp[wave * 64 + lane] = z0 + z1;
    }
    __syncthreads();
    if (wave == 0) {
      float z = 0.f;
#pragma unroll
      for (int w = 0; w < 16; ++w) z += zp[w * 64 + lane];
      const int b = b0 + e;
      const bool valid = b < a.B;
      const float sa = __shfl(z, (lane & 48) + 15, 64); // ||a1_e||^2
      z = jj < 15 ? z + bs[jj] : -INFINITY;
      float mx = z;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      const float ex = expf(z - mx);
      float se = ex;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
      const float dv = ex / se - (jj == yy ? 1.f : 0.f);
      float sd = dv * dv;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) sd += __shfl_xor(sd, o, 64);
      d2[e * 16 + jj] = valid ? dv : 0.f;
      if (jj == 0) n2s[e] = (sa + 1.f) * sd;
    }
    __syncthreads();
    // ---- C. delta1 of example bq, its norm, the clip factor
    float d1v[4];
    float sq = 0.f;
    {
      float dq[NCP];
#pragma unroll
      for (int j = 0; j < NCP; ++j) dq[j] = d2[q * 16 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int h = hh + 256 * i;
        const int hc = h < H ? h : 0;
        float t = 0.f;
#pragma unroll
        for (int j = 0; j < NCP; ++j) t = fmaf(wt[j * ldw + hc], dq[j], t);
        t *= act_deriv_from_out(a.act, a1s[q * ldh + hc]);
        d1v[i] = h < H ? t : 0.f;
        sq = fmaf(d1v[i], d1v[i], sq);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { sq += __shfl_xor(sq, o, 64); sx += __shfl_xor(sx, o, 64); }
    if (lane == 0) { red[wave * 2] = sq; red[wave * 2 + 1] = sx; }
    __syncthreads();
    float sc;
    {
      const int w0 = 4 * q;
      const float sd1 = (red[w0 * 2] + red[w0 * 2 + 2]) + (red[w0 * 2 + 4] + red[w0 * 2 + 6]);
      const float sxx = (red[w0 * 2 + 1] + red[w0 * 2 + 3]) + (red[w0 * 2 + 5] + red[w0 * 2 + 7]);
      const float n = sqrtf((sxx + 1.f) * sd1 + n2s[q]);
      sc = (a.priv && a.head != 1) ? fminf(1.f, a.C / n) : 1.f; // n == 0: C/0 = +inf -> 1
      if (a.head == 2 && vq && hh < 16) a.delta2_out[(long)bq * 16 + hh] = sc * d2[q * 16 + hh];
      if (a.head == 1) {
        if (vq && hh == 0) {
          if (a.slot1) a.slot1[bq] = (sxx + 1.f) * sd1;
          if (a.slot2) a.slot2[bq] = n2s[q];
        }
        if (vq && hh < a.d2_ld) a.delta2_out[(long)bq * a.d2_ld + hh] = d2[q * 16 + hh];
        if (vq && a.a1_out) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int h = hh + 256 * i;
            if (h < H) a.a1_out[(long)bq * H + h] = a1v[i];
          }
        }
      } else if (vq && hh == 0) {
        if (a.norms) a.norms[bq] = n;
        if (a.s) a.s[bq] = sc;
      }
      if (vq) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int h = hh + 256 * i;
          if (h < H) a.sdelta1[(long)bq * H + h] = sc * d1v[i];
        }
      }
    }
    __syncthreads(); // every thread has read delta2 before it is scaled in place
    if (a.head) continue; // (uniform; the barrier above also separates this group's LDS reads from the next group's writes)
    if (hh < 16) d2[q * 16 + hh] *= sc;
    __syncthreads();
    // ---- D. the logit layer's clipped partial: thread = row tid of [H + 1][N]
    if (tid <= H) {
#pragma unroll
      for (int p = 0; p < DENSE1_EX; ++p) {
        const float v = tid < H ? a1s[p * ldh + tid] : 1.f;
#pragma unroll
        for (int j = 0; j < NCP; ++j) acc[j] = fmaf(v, d2[p * 16 + j], acc[j]);
      }
    }
    __syncthreads();
  }
  const int tid = tid0;
  if (!a.head && tid <= H) {
    float *pr = a.part2 + (long)blockIdx.x * dense1_part_stride(H, N) + (long)tid * N;
#pragma unroll
    for (int j = 0; j < NCP; ++j)
      if (j < N) pr[j] = acc[j];
  }
}

static inline int launch_dense2_mid(hipStream_t st, Dense2Args a, int max_tiles) {
  int groups = 1, tiles = 0;
  dense1_tiling(a.B, max_tiles, &groups, &tiles);
  if (tiles == 0) return 0;
  a.groups = groups;
  a.dN.init(a.N);
  dim3 grid(tiles), block(DENSE1_THREADS);
  const int ncp = dense1_ncp(a.N);
  const size_t smem = sizeof(float) * ((size_t)DENSE1_EX * dense1_ldx(a.H) + (size_t)ncp * dense1_ldw(a.H) + 16 * 64 +
                                       DENSE1_EX * 16 + 16 + 32 + DENSE1_EX);
  if (ncp == 4) hipLaunchKernelGGL(dense2_mid_kernel<4>, grid, block, smem, st, a);
  else if (ncp == 10) hipLaunchKernelGGL(dense2_mid_kernel<10>, grid, block, smem, st, a);
  else hipLaunchKernelGGL(dense2_mid_kernel<15>, grid, block, smem, st, a);
  return tiles;
}

// ---------------------------------------------------------------------------------------------------------------
// The two batch-wide contractions of a two-layer network -- the hidden layer's forward product and its clipped sum
// -- at sizes where the whole output is a few hundred 32 x 32 tiles (512 x 512 x 784: 0.4 GFLOP, 3 us of the chip).
// Split-K partials and the launch that sums them cost more than the product itself there, so the K range is split
// INSIDE the workgroup: its four waves take every fourth 32-deep slice of K for the same 32 x 32 tile and add their
// four partial tiles through LDS at the end.  The output is complete: bias and activation (forward) or the single
// partial row the final write reads (clipped sum) are applied by the same kernel.
// A wave works alone until that last sum -- no workgroup barrier in the K loop: it loads its slice of both operands
// with 16-byte loads along whichever index is contiguous in memory (k for a row-major operand, the row for a k-major
// one), keeps the next slice in registers while the current one is multiplied, and passes the slice through an LDS
// area of its own ([k][row], row length 33), from which the lanes of v_mfma_f32_32x32x2_f32 read their operands.
// LDS operations of one wave complete in order, so one area per wave needs no double buffer.
struct SmallGemmArgs {
  const float *A; long a_sr, a_sk; // element (m, k) = A[m * a_sr + k * a_sk]; one of the two strides is 1
  const float *B; long b_sr, b_sk; // element (n, k) = B[n * b_sr + k * b_sk]; one of the two strides is 1
  const float *bias;               // [N] or null
  float *C; long c_sm, c_sn;       // C[m * c_sm + n * c_sn]
  float *C_ones;                   // row M of the output when a_ones (the bias gradient), indexed by n
  int M, N, K, act;
  int a_ones;                      // 1: A has one more row, m = M, that is constant 1 (then the grid covers M + 1 rows)
  const float *k_scale;            // [K] or null: B's element (n, k) is multiplied by k_scale[k] (the clip factors of a
                                   // clipped sum whose delta is not scaled yet); B's rows must be the contiguous index
};

typedef float sg_f32x16 __attribute__((ext_vector_type(16)));
#define SG_LD 33

// 16-byte alignment of every vector the kernel loads: base pointers, the non-unit strides and K must be multiples of
// 4 floats; an operand whose rows are the contiguous index has a row count that is one too, or rows of memory padded
// to the next multiple (its k stride covers it), so that the last group of four may be read whole
static inline bool dense_small_gemm_fits(const SmallGemmArgs &a) {
  auto al = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  const bool a_kc = a.a_sk == 1, b_kc = a.b_sk == 1;
  if (!al(a.A) || !al(a.B) || a.K < 1 || ((a_kc || b_kc) && (a.K & 3) != 0)) return false;
  if (a.k_scale && b_kc) return false;
  if (a_kc ? (a.a_sr & 3) != 0 : (a.a_sr != 1 || (a.a_sk & 3) != 0 || a.a_sk < ((a.M + 3) & ~3))) return false;
  if (b_kc ? (a.b_sr & 3) != 0 : (a.b_sr != 1 || (a.b_sk & 3) != 0 || a.b_sk < ((a.N + 3) & ~3))) return false;
  return true;
}

// One operand slice: rows r0 .. r0 + 31 (R real rows, row R the constant 1 if ONES), k0 .. k0 + 31, as four 16-byte
// items per lane.  KC: k is the contiguous index (item = row, four k); otherwise the row is (item = k, four rows).
template <bool KC>
__device__ __forceinline__ void sg_fetch(const float *P, long sr, long sk, int r0, int R, int K, int k0, int lane, float4 (&v)[4]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int it = lane + 64 * q; // 256 items
    if (KC) {
      const int row = r0 + (it >> 3), k = k0 + 4 * (it & 7);
      const bool ok = row < R && k < K;
      v[q] = *reinterpret_cast<const float4 *>(P + (ok ? (long)row * sr + k : 0));
    } else {
      const int k = k0 + (it >> 3), row = r0 + 4 * (it & 7);
      const bool ok = row < R && k < K; // (a group that crosses R reads the row's padding: see dense_small_gemm_fits)
      v[q] = *reinterpret_cast<const float4 *>(P + (ok ? (long)k * sk + row : 0));
    }
  }
}
template <bool KC>
__device__ __forceinline__ void sg_stash(float *T, int r0, int R, bool ones, int K, int k0, int lane, const float4 (&v)[4]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int it = lane + 64 * q;
    float e[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
    if (KC) {
      const int rl = it >> 3, kl = 4 * (it & 7), row = r0 + rl;
      const bool ok = row < R && k0 + kl < K, one = ones && row == R && k0 + kl < K;
#pragma unroll
      for (int j = 0; j < 4; ++j) T[(kl + j) * SG_LD + rl] = ok ? e[j] : (one ? 1.f : 0.f);
    } else {
      const int kl = it >> 3, rl = 4 * (it & 7), row = r0 + rl;
      const bool kin = k0 + kl < K;
#pragma unroll
      for (int j = 0; j < 4; ++j) T[kl * SG_LD + rl + j] = (kin && row + j < R) ? e[j] : ((ones && kin && row + j == R) ? 1.f : 0.f);
    }
  }
}

// NW waves per workgroup (the K split); LDS: NW areas of 2 x 32 x 33 floats, passed as dynamic shared memory
// A launch may carry a second product of the same operand layouts (the two clipped sums of a two-layer network):
// rows ny0 and up of the grid are its tiles.
template <bool A_KC, bool B_KC, int NW>
__global__ __launch_bounds__(64 * NW) void dense_small_gemm_kernel(const SmallGemmArgs p0, const SmallGemmArgs p1, int ny0) {
  extern __shared__ float sg_lds[]; // per wave: A slice [k][m], B slice [k][n]; after the K loop: the wave's partial tile
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lk = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool second = (int)blockIdx.y >= ny0;
  const SmallGemmArgs &a = second ? p1 : p0;
  int tm = blockIdx.x, tn = (int)blockIdx.y - (second ? ny0 : 0);
  if (!second) {
    // Workgroups go to the eight XCDs in turn, each with an L2 of its own: XCD x takes a run of consecutive tiles of
    // the list "panels of eight tile columns, row by row inside a panel", a compact block of the output, so that it
    // reads a few row strips of A and column strips of B instead of all of one operand.
    const int gx = gridDim.x, T = gx * ny0, L = blockIdx.x + gx * blockIdx.y;
    const int xcd = L & 7, i = L >> 3, qn = T >> 3, rn = T & 7;
    const int t = xcd * qn + min(xcd, rn) + i;
    const int p = t / (gx * 8), rem = t - p * (gx * 8), w = min(8, ny0 - 8 * p);
    tm = rem / w;
    tn = 8 * p + (rem - tm * w);
  }
  const int m0 = tm * 32, n0 = tn * 32;
  const int Mtot = a.M + (a.a_ones ? 1 : 0);
  if (m0 >= Mtot) return; // (the grid is as wide as the larger of the two products; uniform, before any barrier)
  float *As = sg_lds + wave * (2 * 32 * SG_LD), *Bs = As + 32 * SG_LD;
  const int n_slices = (a.K + 31) >> 5;
  sg_f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  float4 va[4], vb[4];
  float sb[4] = {1.f, 1.f, 1.f, 1.f}; // k_scale of vb's four items (an item of a row-contiguous operand has one k)
  auto fetch_scale = [&](int k0) {
    if (!B_KC && a.k_scale) {
#pragma unroll
      for (int q = 0; q < 4; ++q) sb[q] = a.k_scale[min(k0 + ((lane + 64 * q) >> 3), a.K - 1)];
    }
  };
  auto apply_scale = [&]() {
    if (!B_KC && a.k_scale) {
#pragma unroll
      for (int q = 0; q < 4; ++q) { vb[q].x *= sb[q]; vb[q].y *= sb[q]; vb[q].z *= sb[q]; vb[q].w *= sb[q]; }
    }
  };
  int sl = wave;
  if (sl < n_slices) {
    sg_fetch<A_KC>(a.A, a.a_sr, a.a_sk, m0, a.M, a.K, 32 * sl, lane, va);
    sg_fetch<B_KC>(a.B, a.b_sr, a.b_sk, n0, a.N, a.K, 32 * sl, lane, vb);
    fetch_scale(32 * sl);
  }
  for (; sl < n_slices; sl += NW) {
    apply_scale();
    sg_stash<A_KC>(As, m0, a.M, a.a_ones != 0, a.K, 32 * sl, lane, va);
    sg_stash<B_KC>(Bs, n0, a.N, false, a.K, 32 * sl, lane, vb);
    __builtin_amdgcn_wave_barrier(); // (the slice is read by other lanes of this wave: LDS operations of a wave complete in order)
    const int nx = min(sl + NW, n_slices - 1); // (past the wave's last slice: one is read again, unused)
    sg_fetch<A_KC>(a.A, a.a_sr, a.a_sk, m0, a.M, a.K, 32 * nx, lane, va);
    sg_fetch<B_KC>(a.B, a.b_sr, a.b_sk, n0, a.N, a.K, 32 * nx, lane, vb);
    fetch_scale(32 * nx);
#pragma unroll
    for (int s2 = 0; s2 < 16; ++s2)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[(2 * s2 + lk) * SG_LD + li], Bs[(2 * s2 + lk) * SG_LD + li], acc, 0, 0, 0);
    __builtin_amdgcn_wave_barrier();
  }
  // the partial tiles meet in LDS, each in its wave's own area (the wave is done with its slices): accumulator
  // register r of a lane is row 8 (r / 4) + 4 lk + r % 4, column li
#pragma unroll
  for (int r = 0; r < 16; ++r) As[(8 * (r >> 2) + 4 * lk + (r & 3)) * SG_LD + li] = acc[r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 16 / NW; ++q) {
    const int e = tid + 64 * NW * q, ml = e >> 5, nl = e & 31; // consecutive threads: consecutive n
    const int m = m0 + ml, n = n0 + nl;
    if (m < Mtot && n < a.N) {
      const float *rp = sg_lds + ml * SG_LD + nl;
      float v[NW];
#pragma unroll
      for (int w = 0; w < NW; ++w) v[w] = rp[w * (2 * 32 * SG_LD)];
#pragma unroll
      for (int h = 1; h < NW; h *= 2) // a fixed tree: (0+1) + (2+3) ...
#pragma unroll
        for (int w = 0; w + h < NW; w += 2 * h) v[w] += v[w + h];
      float r = v[0];
      if (a.bias) r += a.bias[n];
      r = act_apply(a.act, r);
      if (m < a.M) a.C[(long)m * a.c_sm + (long)n * a.c_sn] = r;
      else a.C_ones[n] = r;
    }
  }
}

#define SG_WAVES 8
static inline size_t dense_small_gemm_lds_bytes() { return sizeof(float) * SG_WAVES * 2 * 32 * SG_LD; }
// once per device before the first launch (the LDS areas of eight waves exceed the default 64 KB limit)
static inline bool dense_small_gemm_prepare() {
  const int bytes = (int)dense_small_gemm_lds_bytes();
  const hipFuncAttribute at = hipFuncAttributeMaxDynamicSharedMemorySize;
  return hipFuncSetAttribute((const void *)dense_small_gemm_kernel<true, true, SG_WAVES>, at, bytes) == hipSuccess &&
         hipFuncSetAttribute((const void *)dense_small_gemm_kernel<true, false, SG_WAVES>, at, bytes) == hipSuccess &&
         hipFuncSetAttribute((const void *)dense_small_gemm_kernel<false, true, SG_WAVES>, at, bytes) == hipSuccess &&
         hipFuncSetAttribute((const void *)dense_small_gemm_kernel<false, false, SG_WAVES>, at, bytes) == hipSuccess;
}

// b: a second product in the same launch, or null; both must have the same contiguous indices
static inline void launch_dense_small_gemm(hipStream_t st, const SmallGemmArgs &a, const SmallGemmArgs *b = nullptr) {
  const int Mtot = a.M + (a.a_ones ? 1 : 0), Mtot2 = b ? b->M + (b->a_ones ? 1 : 0) : 0;
  const int ny0 = (a.N + 31) / 32, ny1 = b ? (b->N + 31) / 32 : 0;
  dim3 grid((std::max(Mtot, Mtot2) + 31) / 32, ny0 + ny1), block(64 * SG_WAVES);
  const size_t lds = dense_small_gemm_lds_bytes();
  const bool a_kc = a.a_sk == 1, b_kc = a.b_sk == 1;
  const SmallGemmArgs &a2 = b ? *b : a;
  if (a_kc && b_kc) hipLaunchKernelGGL((dense_small_gemm_kernel<true, true, SG_WAVES>), grid, block, lds, st, a, a2, ny0);
  else if (a_kc) hipLaunchKernelGGL((dense_small_gemm_kernel<true, false, SG_WAVES>), grid, block, lds, st, a, a2, ny0);
  else if (b_kc) hipLaunchKernelGGL((dense_small_gemm_kernel<false, true, SG_WAVES>), grid, block, lds, st, a, a2, ny0);
  else hipLaunchKernelGGL((dense_small_gemm_kernel<false, false, SG_WAVES>), grid, block, lds, st, a, a2, ny0);
}

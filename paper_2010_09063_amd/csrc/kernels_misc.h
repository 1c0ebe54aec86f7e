// Small kernels of the private step: loss gradient, pooling, dense per-example
// norms, clip factors, and the final write with fused Philox noise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_tile.h" // FastDiv

#define DP_ACT_NONE_ 0
#define DP_ACT_RELU_ 1
#define DP_ACT_TANH_ 2

// tanh and the logistic function from one hardware exp2 and one hardware reciprocal
// (v_exp_f32, v_rcp_f32: about 1 ulp each).  Absolute error is at the 1e-7 level, the same
// size as fp32 rounding of the result, far inside the 1e-4 bar on the aggregated gradient;
// the library versions cost several times the MFMA time of a small tile's epilogue.
__device__ __forceinline__ float fast_tanh(float x) {
  const float t = __builtin_amdgcn_exp2f(-2.885390081777927f * fabsf(x)); // exp(-2|x|)
  const float r = (1.f - t) * __builtin_amdgcn_rcpf(1.f + t);
  return copysignf(r, x);
}
__device__ __forceinline__ float fast_sigmoid(float x) {
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

__device__ __forceinline__ float act_apply(int act, float z) {
  if (act == DP_ACT_RELU_) return z > 0.f ? z : 0.f;
  if (act == DP_ACT_TANH_) return fast_tanh(z);
  return z;
}
// derivative expressed through the activation's output a = act(z)
__device__ __forceinline__ float act_deriv_from_out(int act, float a) {
  if (act == DP_ACT_RELU_) return a > 0.f ? 1.f : 0.f;
  if (act == DP_ACT_TANH_) return 1.f - a * a;
  return 1.f;
}

// i = (z * Y + y) * X + x  ->  (x, y, z); 32-bit arithmetic with precomputed reciprocals when the range allows
struct Split3 { FastDiv dX, dY; };
__device__ __forceinline__ void split3(long i, long total, int X, int Y, const Split3 &d, int &x, int &y, long &z) {
  if (total < (1l << 31)) {
    const unsigned u = (unsigned)i, r = d.dX.div(u), r2 = d.dY.div(r);
    x = (int)(u - r * (unsigned)X);
    y = (int)(r - r2 * (unsigned)Y);
    z = r2;
  } else {
    x = (int)(i % X);
    const long r = i / X;
    y = (int)(r % Y);
    z = r / Y;
  }
}

// delta_i = softmax(logits_i) - onehot(y_i): gradient of one example's own
// cross-entropy (DPSGD item 2a: the objective at (x_i, y_i), not a batch mean).
__global__ void softmax_xent_grad_kernel(const float *__restrict__ logits, const int *__restrict__ y,
                                         float *__restrict__ g, int B, int K) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const float *z = logits + (long)b * K;
  float mx = z[0];
  for (int k = 1; k < K; ++k) mx = fmaxf(mx, z[k]);
  float se = 0.f;
  for (int k = 0; k < K; ++k) se += expf(z[k] - mx);
  float inv = 1.f / se;
  int yy = y[b];
  for (int k = 0; k < K; ++k) g[(long)b * K + k] = expf(z[k] - mx) * inv - (k == yy ? 1.f : 0.f);
}

// max-pool forward; arg = window offset kh*KW+kw of the first maximum.  K_ / S_: window and stride as compile-time
// constants for the common 2x2 / stride-1 pool (0: taken from the arguments).
template <int K_, int S_>
__global__ void maxpool_fwd_kernel(const float *__restrict__ in, float *__restrict__ out,
                                   uint8_t *__restrict__ arg, long total, int H, int W, int OH, int OW,
                                   int KH_, int KW_, int Sa, Split3 dv) {
  const int KH = K_ ? K_ : KH_, KW = K_ ? K_ : KW_, S = S_ ? S_ : Sa;
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int ow, oh;
  long bc;
  split3(i, total, OW, OH, dv, ow, oh, bc);
  const float *p = in + (bc * H + (long)oh * S) * W + (long)ow * S;
  float best = p[0];
  int bi = 0;
#pragma unroll
  for (int kh = 0; kh < KH; ++kh)
#pragma unroll
    for (int kw = 0; kw < KW; ++kw) {
      float v = p[kh * W + kw];
      if (v > best) { best = v; bi = kh * KW + kw; }
    }
  out[i] = best;
  arg[i] = (uint8_t)bi;
}

// max-pool backward in gather form (no atomics): every input position sums the
// output gradients of the windows whose recorded maximum it is, then applies the
// derivative of the activation that produced the pool's input.
template <int K_, int S_>
__global__ void maxpool_bwd_kernel(const float *__restrict__ gout, const uint8_t *__restrict__ arg,
                                   const float *__restrict__ a_in, float *__restrict__ gin, long total, int H,
                                   int W, int OH, int OW, int KH_, int KW_, int Sa, int act, Split3 dv, FastDiv dS) {
  const int KH = K_ ? K_ : KH_, KW = K_ ? K_ : KW_, S = S_ ? S_ : Sa;
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int iw, ih;
  long bc;
  split3(i, total, W, H, dv, iw, ih, bc);
  float acc = 0.f;
  int oh_lo = ih - KH + 1; oh_lo = oh_lo > 0 ? (S_ == 1 ? oh_lo : (int)dS.div((unsigned)(oh_lo + S - 1))) : 0;
  int ow_lo = iw - KW + 1; ow_lo = ow_lo > 0 ? (S_ == 1 ? ow_lo : (int)dS.div((unsigned)(ow_lo + S - 1))) : 0;
  int oh_hi = min(S_ == 1 ? ih : (int)dS.div((unsigned)ih), OH - 1), ow_hi = min(S_ == 1 ? iw : (int)dS.div((unsigned)iw), OW - 1);
  const long obase = bc * OH * OW; // (windows of one plane: 32-bit offsets from here)
  for (int oh = oh_lo; oh <= oh_hi; ++oh)
    for (int ow = ow_lo; ow <= ow_hi; ++ow) {
      const long o = obase + oh * OW + ow;
      int want = (ih - oh * S) * KW + (iw - ow * S);
      if ((int)arg[o] == want) acc += gout[o];
    }
  gin[i] = acc * act_deriv_from_out(act, a_in[i]);
}

// 2x2 / stride-2 pooling with even H and W (the common case): one thread per window,
// 8-byte accesses to the two input rows, no divisions by the window geometry.
__global__ void maxpool2x2_fwd_kernel(const float *__restrict__ in, float *__restrict__ out,
                                      uint8_t *__restrict__ arg, long total, int OW, int W) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const long row = i / OW;           // (b, c, oh) flattened: input rows 2*row and 2*row+1
  const int ow = (int)(i - row * OW);
  const float2 t = *reinterpret_cast<const float2 *>(in + (2 * row) * W + 2 * ow);
  const float2 u = *reinterpret_cast<const float2 *>(in + (2 * row + 1) * W + 2 * ow);
  float best = t.x; int bi = 0;
  if (t.y > best) { best = t.y; bi = 1; }
  if (u.x > best) { best = u.x; bi = 2; }
  if (u.y > best) { best = u.y; bi = 3; }
  out[i] = best;
  arg[i] = (uint8_t)bi;
}

// Backward: the gradient of a window goes to the position of its (first) maximum, times the derivative of the
// activation that produced the pooled plane.  That derivative is a function of the activation's OUTPUT at that
// position, which is the pooled value itself -- so the kernel reads the pooled plane (a quarter of the words) instead
// of the activation plane: bit-identical, and a third less memory traffic.
__global__ void maxpool2x2_bwd_kernel(const float *__restrict__ gout, const uint8_t *__restrict__ arg,
                                      const float *__restrict__ pooled, float *__restrict__ gin, long total, int OW,
                                      int W, int act) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const long row = i / OW;
  const int ow = (int)(i - row * OW);
  const float g = gout[i] * act_deriv_from_out(act, pooled[i]);
  const int bi = arg[i];
  const long o0 = (2 * row) * W + 2 * ow, o1 = o0 + W;
  float2 r0, r1;
  r0.x = bi == 0 ? g : 0.f;
  r0.y = bi == 1 ? g : 0.f;
  r1.x = bi == 2 ? g : 0.f;
  r1.y = bi == 3 ? g : 0.f;
  *reinterpret_cast<float2 *>(gin + o0) = r0;
  *reinterpret_cast<float2 *>(gin + o1) = r1;
}
// The same for an even number of windows per row: a thread takes two neighbouring windows (8-byte reads, 16-byte stores).
__global__ void maxpool2x2_bwd2_kernel(const float *__restrict__ gout, const uint8_t *__restrict__ arg,
                                       const float *__restrict__ pooled, float *__restrict__ gin, long pairs, int OW2,
                                       int W, int act) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pairs) return;
  const long row = i / OW2;
  const int op = (int)(i - row * OW2);
  const float2 gg = *reinterpret_cast<const float2 *>(gout + 2 * i);
  const float2 pv = *reinterpret_cast<const float2 *>(pooled + 2 * i);
  const unsigned short ab = *reinterpret_cast<const unsigned short *>(arg + 2 * i);
  const float g0 = gg.x * act_deriv_from_out(act, pv.x), g1 = gg.y * act_deriv_from_out(act, pv.y);
  const int b0 = ab & 255, b1 = ab >> 8;
  const long o0 = (2 * row) * W + 4 * op, o1 = o0 + W;
  float4 r0, r1;
  r0.x = b0 == 0 ? g0 : 0.f; r0.y = b0 == 1 ? g0 : 0.f; r0.z = b1 == 0 ? g1 : 0.f; r0.w = b1 == 1 ? g1 : 0.f;
  r1.x = b0 == 2 ? g0 : 0.f; r1.y = b0 == 3 ? g0 : 0.f; r1.z = b1 == 2 ? g1 : 0.f; r1.w = b1 == 3 ? g1 : 0.f;
  *reinterpret_cast<float4 *>(gin + o0) = r0;
  *reinterpret_cast<float4 *>(gin + o1) = r1;
}

// Backward-data of a strided convolution, second half: the first half is the per-example product
// cols[b][(c, kh, kw)][p] = sum_d W[d][c][kh][kw] Delta[b][d][p] (a plain contraction, no gather).  Here every
// input position sums the columns of the windows that hold it (gather form, no atomics) and applies the derivative
// of the activation that produced the layer's input.  One thread per input element.
struct Col2imDiv { FastDiv dW, dH, dC, dS; };
__global__ void conv_col2im_kernel(const float *__restrict__ cols, const float *__restrict__ a_in,
                                   float *__restrict__ gin, long total, int C, int H, int W, int OH, int OW, int KH,
                                   int KW, int S, int PAD, int act, Col2imDiv dv) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int iw, ih, c;
  long b;
  if (total < (1l << 31)) { // 32-bit index arithmetic with precomputed reciprocals
    const unsigned u = (unsigned)i;
    unsigned r = dv.dW.div(u);
    iw = (int)(u - r * (unsigned)W);
    unsigned r2 = dv.dH.div(r);
    ih = (int)(r - r2 * (unsigned)H);
    const unsigned r3 = dv.dC.div(r2);
    c = (int)(r2 - r3 * (unsigned)C);
    b = r3;
  } else {
    iw = (int)(i % W);
    long r = i / W;
    ih = (int)(r % H);
    r /= H;
    c = (int)(r % C);
    b = r / C;
  }
  const int P = OH * OW, KK = KH * KW;
  const float *cb = cols + ((long)b * C + c) * KK * P;
  // only the taps whose window row / column lands on this position: kh = (ih + PAD) mod S, then every S-th
  const int ihp = ih + PAD, iwp = iw + PAD;
  const int qh = (int)dv.dS.div((unsigned)ihp), qw = (int)dv.dS.div((unsigned)iwp);
  const int kh0 = ihp - qh * S, kw0 = iwp - qw * S;
  float acc = 0.f;
  for (int kh = kh0, oh = qh; kh < KH && oh >= 0; kh += S, --oh) {
    if (oh >= OH) continue;
    for (int kw = kw0, ow = qw; kw < KW && ow >= 0; kw += S, --ow) {
      if (ow >= OW) continue;
      acc += cb[(long)(kh * KW + kw) * P + oh * OW + ow];
    }
  }
  gin[i] = a_in != nullptr ? acc * act_deriv_from_out(act, a_in[i]) : acc;
}

// Average pool (Appendix B, CIFAR10 network): the plain mean of a KH x KW window, no padding.  A window that
// covers the whole plane is the global average pool.
__global__ void avgpool_fwd_kernel(const float *__restrict__ in, float *__restrict__ out, long total, int H, int W,
                                   int OH, int OW, int KH, int KW, int S, Split3 dv) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int ow, oh;
  long bc;
  split3(i, total, OW, OH, dv, ow, oh, bc);
  const float *p = in + (bc * H + (long)oh * S) * W + (long)ow * S;
  float acc = 0.f;
  for (int kh = 0; kh < KH; ++kh)
    for (int kw = 0; kw < KW; ++kw) acc += p[kh * W + kw];
  out[i] = acc / (float)(KH * KW);
}

// Gather form of the backward pass: an input position sums 1/(KH*KW) of the gradient of every window that
// holds it, then applies the derivative of the activation that produced the pool's input.
__global__ void avgpool_bwd_kernel(const float *__restrict__ gout, const float *__restrict__ a_in,
                                   float *__restrict__ gin, long total, int H, int W, int OH, int OW, int KH, int KW,
                                   int S, int act, Split3 dv, FastDiv dS) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int iw, ih;
  long bc;
  split3(i, total, W, H, dv, iw, ih, bc);
  float acc = 0.f;
  int oh_lo = ih - KH + 1; oh_lo = oh_lo > 0 ? (int)dS.div((unsigned)(oh_lo + S - 1)) : 0;
  int ow_lo = iw - KW + 1; ow_lo = ow_lo > 0 ? (int)dS.div((unsigned)(ow_lo + S - 1)) : 0;
  int oh_hi = min((int)dS.div((unsigned)ih), OH - 1), ow_hi = min((int)dS.div((unsigned)iw), OW - 1);
  for (int oh = oh_lo; oh <= oh_hi; ++oh)
    for (int ow = ow_lo; ow <= ow_hi; ++ow) acc += gout[(bc * OH + oh) * OW + ow];
  gin[i] = acc / (float)(KH * KW) * act_deriv_from_out(act, a_in[i]);
}

// 2x2 / stride-2 average pool with even H and W: one thread per window, 8-byte accesses.
__global__ void avgpool2x2_fwd_kernel(const float *__restrict__ in, float *__restrict__ out, long total, int OW,
                                      int W) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const long row = i / OW;
  const int ow = (int)(i - row * OW);
  const float2 t = *reinterpret_cast<const float2 *>(in + (2 * row) * W + 2 * ow);
  const float2 u = *reinterpret_cast<const float2 *>(in + (2 * row + 1) * W + 2 * ow);
  out[i] = ((t.x + t.y) + (u.x + u.y)) * 0.25f;
}

__global__ void avgpool2x2_bwd_kernel(const float *__restrict__ gout, const float *__restrict__ a_in,
                                      float *__restrict__ gin, long total, int OW, int W, int act) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const long row = i / OW;
  const int ow = (int)(i - row * OW);
  const float g = gout[i] * 0.25f;
  const long o0 = (2 * row) * W + 2 * ow, o1 = o0 + W;
  const float2 t = *reinterpret_cast<const float2 *>(a_in + o0);
  const float2 u = *reinterpret_cast<const float2 *>(a_in + o1);
  float2 r0, r1;
  r0.x = g * act_deriv_from_out(act, t.x); r0.y = g * act_deriv_from_out(act, t.y);
  r1.x = g * act_deriv_from_out(act, u.x); r1.y = g * act_deriv_from_out(act, u.y);
  *reinterpret_cast<float2 *>(gin + o0) = r0;
  *reinterpret_cast<float2 *>(gin + o1) = r1;
}

// Clipped sum of stored per-example gradients (Section 1, items 2b-3): sum over a split's examples of
// s[b] * g[b][n], where a row of g is in the accumulator order of the convolution weight-gradient kernel
// ([channel block][wave group][tap slot][16 registers][64 lanes], then the bias).  Thread = one stored word n
// (consecutive lanes read consecutive words), blockIdx.y = split; the result goes to the parameter layout
// part[split][(d*C + c)*KK + tap] (bias: D*C*KK + d); padding slots are skipped.
struct GradOrder {
  int C, D, KK;       // layer shape
  int NBW, WN, NW;    // tap slots per wave group, wave groups along the taps, wave groups per channel block
  int flat;           // 1: one wave group whose lane column is the flattened (channel, tap) index;
                      // 2: the rows are in the parameter layout already;
                      // 3: rows are [D][C*KK + 1], the bias gradient being the last column
  long n_w;           // flat 0 / 1: stored words before the bias
  long n_total;       // words per stored row
};
__global__ __launch_bounds__(256) void weighted_sum_kernel(const float *__restrict__ g, long gstride,
                                                           const float *__restrict__ s, float *__restrict__ part,
                                                           long pstride, GradOrder o, int B, int ex_per_split) {
  const long n = (long)blockIdx.x * 256 + threadIdx.x;
  if (n >= o.n_total) return;
  long p;
  if (o.flat == 2) {
    p = n;
  } else if (o.flat == 3) {
    const int ckk = o.C * o.KK;
    const long m = n / (ckk + 1);
    const int col = (int)(n - m * (ckk + 1));
    p = col < ckk ? m * ckk + col : (long)o.D * ckk + m;
  } else if (n >= o.n_w) {
    p = (long)o.D * o.C * o.KK + (n - o.n_w);
  } else {
    const int lane = (int)(n & 63), r = (int)((n >> 6) & 15);
    const long t = n >> 10;
    const int j = (int)(t % o.NBW);
    const long t2 = t / o.NBW;
    const int grp = (int)(t2 % o.NW), cbi = (int)(t2 / o.NW);
    const int wd = grp / o.WN, wn = grp % o.WN;
    const int li = lane & 31, lk = lane >> 5;
    const int d = wd * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
    if (d >= o.D) return;
    if (o.flat) {
      if (li >= o.C * o.KK) return;
      p = (long)d * o.C * o.KK + li;
    } else {
      const int c = cbi * 32 + li, tap = wn * o.NBW + j;
      if (c >= o.C || tap >= o.KK) return;
      p = ((long)d * o.C + c) * o.KK + tap;
    }
  }
  const int b0 = blockIdx.y * ex_per_split, b1 = min(B, b0 + ex_per_split);
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int b = b0;
  for (; b + 4 <= b1; b += 4) {
    const float v0 = g[(long)b * gstride + n], v1 = g[(long)(b + 1) * gstride + n], v2 = g[(long)(b + 2) * gstride + n],
                v3 = g[(long)(b + 3) * gstride + n];
    a0 = fmaf(s[b], v0, a0); a1 = fmaf(s[b + 1], v1, a1); a2 = fmaf(s[b + 2], v2, a2); a3 = fmaf(s[b + 3], v3, a3);
  }
  for (; b < b1; ++b) a0 = fmaf(s[b], g[(long)b * gstride + n], a0);
  part[(long)blockIdx.y * pstride + p] = (a0 + a1) + (a2 + a3);
}

// Dense layer: ||g_i||^2 = (||a_i||^2 + 1) ||delta_i||^2 without forming the outer
// product (Section 1: per-example norms for fully-connected layers).  One wave per example.
__global__ void dense_norm_kernel(const float *__restrict__ a, int d_in, const float *__restrict__ delta, int d_out,
                                  float *__restrict__ slot, int B) {
  int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (wave >= B) return;
  float sa = 0.f, sd = 0.f;
  for (int k = lane; k < d_in; k += 64) { float v = a[(long)wave * d_in + k]; sa += v * v; }
  for (int k = lane; k < d_out; k += 64) { float v = delta[(long)wave * d_out + k]; sd += v * v; }
  for (int o = 32; o > 0; o >>= 1) { sa += __shfl_xor(sa, o, 64); sd += __shfl_xor(sd, o, 64); }
  if (lane == 0) slot[wave] = (sa + 1.f) * sd;
}

// n_i = sqrt(sum over all layers' partial squared norms); s_i = min(1, C / n_i)  (DPSGD item 2b)
__global__ void clip_factor_kernel(const float *__restrict__ slots, int n_slots, long slot_stride, float C,
                                   float *__restrict__ norms, float *__restrict__ s, int B) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  float n2 = 0.f;
  for (int k = 0; k < n_slots; ++k) n2 += slots[k * slot_stride + b];
  float n = sqrtf(n2);
  norms[b] = n;
  s[b] = fminf(1.f, C / n); // n == 0: C/0 = +inf -> 1
}

// out[i] = act(sum_s part[s*stride + i] + bias[i % N]): epilogue of a split-K dense forward
__global__ void bias_act_reduce_kernel(const float *__restrict__ part, int nsplit, long stride,
                                       const float *__restrict__ bias, int act, float *__restrict__ out, long total,
                                       int N) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  float a0 = 0.f, a1 = 0.f;
  int s = 0;
  for (; s + 1 < nsplit; s += 2) { a0 += part[s * stride + i]; a1 += part[(s + 1) * stride + i]; }
  if (s < nsplit) a0 += part[s * stride + i];
  out[i] = act_apply(act, a0 + a1 + bias[i % N]);
}

// Last dense layer (no activation, at most 64 classes), one wave per example, three small launches in one:
//   logits   z[n] = sum of the forward split-K partials + bias[n]   (part == nullptr: z is already in a)
//   loss     g = softmax(z) - onehot(y)                             (Section 1, item 2a: the example's own loss)
//   norm     slot[b] = (||a_in||^2 + 1) ||g||^2                     (dense identity; slot == nullptr: skipped)
//   clip     norms[b], s[b] as clip_factor_kernel computes them      (only when this slot is the whole norm, i.e.
//                                                                      the model is this one layer; else null)
__global__ __launch_bounds__(256) void logits_loss_norm_kernel(const float *__restrict__ part, int nsplit, long stride,
                                                               const float *__restrict__ bias, const int *__restrict__ y,
                                                               const float *__restrict__ a_in, int d_in,
                                                               float *__restrict__ a, float *__restrict__ g,
                                                               float *__restrict__ slot, float *__restrict__ norms,
                                                               float *__restrict__ s_out, float C, int B, int N) {
  const int b = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (b >= B) return;
  const bool on = lane < N;
  float z = 0.f;
  if (on) {
    const long i = (long)b * N + lane;
    if (part != nullptr) {
      float a0 = 0.f, a1 = 0.f;
      int s = 0;
      for (; s + 1 < nsplit; s += 2) { a0 += part[s * stride + i]; a1 += part[(s + 1) * stride + i]; }
      if (s < nsplit) a0 += part[s * stride + i];
      z = a0 + a1 + bias[lane];
      a[i] = z;
    } else {
      z = a[i];
    }
  }
  float mx = on ? z : -INFINITY;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  const float e = on ? expf(z - mx) : 0.f;
  float se = e;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
  const float gv = on ? e * (1.f / se) - (lane == y[b] ? 1.f : 0.f) : 0.f;
  if (on) g[(long)b * N + lane] = gv;
  if (slot == nullptr) return;
  float sd = gv * gv, sa = 0.f;
  for (int k = lane; k < d_in; k += 64) { const float v = a_in[(long)b * d_in + k]; sa += v * v; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { sd += __shfl_xor(sd, o, 64); sa += __shfl_xor(sa, o, 64); }
  if (lane == 0) {
    const float n2 = (sa + 1.f) * sd;
    slot[b] = n2;
    if (s_out != nullptr) {
      const float n = sqrtf(n2);
      norms[b] = n;
      s_out[b] = fminf(1.f, C / n); // n == 0: C/0 = +inf -> 1
    }
  }
}

// zeroes p[0:n] and q[0:m] (one launch for the two buffers the embedding's clipped sum starts from)
__global__ void fill_zero_kernel(float *__restrict__ p, long n, float *__restrict__ q, long m) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
  else if (i - n < m) q[i - n] = 0.f;
}

// ---------------------------------------------------------------- noise

// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// four standard normals of block `blk`: uniforms ((r >> 9) + 1/2) 2^-23 (exact in
// fp32, never 0 or 1), two Box-Muller pairs.
__device__ __forceinline__ void normal4(uint64_t blk, uint32_t k0, uint32_t k1, float z[4]) {
  uint32_t r[4];
  philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, k0, k1, r);
  float u[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) u[q] = ((float)(r[q] >> 9) + 0.5f) * (1.0f / 8388608.0f);
  float r0 = sqrtf(-2.f * logf(u[0])), r1 = sqrtf(-2.f * logf(u[2]));
  float s, c;
  sincospif(2.f * u[1], &s, &c);
  z[0] = r0 * c; z[1] = r0 * s;
  sincospif(2.f * u[3], &s, &c);
  z[2] = r1 * c; z[3] = r1 * s;
}

// Final write (DPSGD item 3): out[j] = sum over split-K partials of the clipped sum + sigma*C*z_j.
// A thread owns the four coordinates of one Philox block (all four normals of the block are used, 16-byte loads
// and stores where the rows allow).  The parameter vector is cut into regions of consecutive tensors whose partial
// rows are summed the same way: a workgroup of a region owns 256 / SG blocks and splits the partial rows SG ways
// -- 16 for tensors cut into many splits (short dependent chains), 4 for a few rows, 1 (every lane draws noise, no
// LDS pass) where a tensor arrives complete.  Every sum runs in a fixed order.
#define DP_MAX_SEG 24
struct FinalizeSeg {
  long p_off, n;     // segment [p_off, p_off + n) of the flat parameter vector
  const float *part; // [nsplit][stride]
  long stride;
  int nsplit;
};
struct FinalizeRegion {
  long blk0, blk1; // Philox blocks [blk0, blk1): those whose first coordinate lies in the region's tensors
  int wg0;         // first workgroup of the region
  int sg;          // split groups of its workgroups: 1, 4 or 16
  int seg0;        // first tensor of the region
};
struct FinalizeArgs {
  int nseg;
  FinalizeSeg seg[DP_MAX_SEG];
  int nreg;
  FinalizeRegion reg[DP_MAX_SEG];
};

// theta != null: the parameter update of DPSGD item 4 is fused into the same write,
// theta[j] -= step * (sum + noise) with step = learning rate / batch; out may then be null.
template <int DP_FIN_SG>
__device__ __forceinline__ void finalize_body(const FinalizeArgs &fa, const FinalizeRegion &rg, float4 *red,
                                              float *__restrict__ out, long P, float noise_std, uint32_t k0, uint32_t k1,
                                              float *__restrict__ theta, float step) {
  constexpr int DP_FIN_BLK = 256 / DP_FIN_SG;
  const int cb = threadIdx.x & (DP_FIN_BLK - 1);
  const int sg = threadIdx.x / DP_FIN_BLK;
  const long blk = rg.blk0 + (long)((int)blockIdx.x - rg.wg0) * DP_FIN_BLK + cb, j0 = blk * 4;
  const bool live = blk < rg.blk1; // (blk1 * 4 < P + 4: a live block has at least one coordinate)
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (live) {
    int si = rg.seg0;
    while (si < fa.nseg - 1 && j0 >= fa.seg[si].p_off + fa.seg[si].n) ++si;
    const FinalizeSeg &g = fa.seg[si];
    const float *p = g.part + (j0 - g.p_off);
    const long st = g.stride;
    const int ns = g.nsplit;
    if (j0 + 3 < g.p_off + g.n && (((uintptr_t)p | (uintptr_t)(st * 4)) & 15) == 0) {
      // the block lies inside one tensor and its rows are 16-byte aligned
      float4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
      int s = sg;
      for (; s + 3 * DP_FIN_SG < ns; s += 4 * DP_FIN_SG) { // four rows in flight
        const float4 v0 = *reinterpret_cast<const float4 *>(p + s * st);
        const float4 v1 = *reinterpret_cast<const float4 *>(p + (s + DP_FIN_SG) * st);
        const float4 v2 = *reinterpret_cast<const float4 *>(p + (s + 2 * DP_FIN_SG) * st);
        const float4 v3 = *reinterpret_cast<const float4 *>(p + (s + 3 * DP_FIN_SG) * st);
        a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
        a1.x += v1.x; a1.y += v1.y; a1.z += v1.z; a1.w += v1.w;
        a2.x += v2.x; a2.y += v2.y; a2.z += v2.z; a2.w += v2.w;
        a3.x += v3.x; a3.y += v3.y; a3.z += v3.z; a3.w += v3.w;
      }
      for (; s < ns; s += DP_FIN_SG) {
        const float4 v0 = *reinterpret_cast<const float4 *>(p + s * st);
        a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
      }
      a0.x += a2.x; a0.y += a2.y; a0.z += a2.z; a0.w += a2.w;
      a1.x += a3.x; a1.y += a3.y; a1.z += a3.z; a1.w += a3.w;
      acc[0] = a0.x + a1.x; acc[1] = a0.y + a1.y; acc[2] = a0.z + a1.z; acc[3] = a0.w + a1.w;
    } else {
      // a block that straddles two tensors, or unaligned rows: coordinate by coordinate
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const long j = j0 + q;
        if (j >= P) break;
        int sj = si;
        while (sj < fa.nseg - 1 && j >= fa.seg[sj].p_off + fa.seg[sj].n) ++sj;
        const FinalizeSeg &h = fa.seg[sj];
        const float *pj = h.part + (j - h.p_off);
        float a0 = 0.f, a1 = 0.f;
        int s = sg;
        for (; s + DP_FIN_SG < h.nsplit; s += 2 * DP_FIN_SG) { a0 += pj[s * h.stride]; a1 += pj[(s + DP_FIN_SG) * h.stride]; }
        if (s < h.nsplit) a0 += pj[s * h.stride];
        acc[q] = a0 + a1;
      }
    }
  }
  if (DP_FIN_SG > 1) {
    if (sg > 0) red[(sg - 1) * DP_FIN_BLK + cb] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    __syncthreads();
  }
  if (sg == 0 && live) {
#pragma unroll
    for (int q = 0; q < DP_FIN_SG - 1; ++q) {
      const float4 v = red[q * DP_FIN_BLK + cb];
      acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    }
    if (noise_std > 0.f) {
      float z[4];
      normal4((uint64_t)blk, k0, k1, z);
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] = fmaf(noise_std, z[q], acc[q]);
    }
    const bool whole = j0 + 3 < P;
    if (out) {
      if (whole && ((uintptr_t)(out + j0) & 15) == 0) *reinterpret_cast<float4 *>(out + j0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
      else
        for (int q = 0; q < 4 && j0 + q < P; ++q) out[j0 + q] = acc[q];
    }
    if (theta) {
      if (whole && ((uintptr_t)(theta + j0) & 15) == 0) {
        float4 t = *reinterpret_cast<float4 *>(theta + j0);
        t.x -= step * acc[0]; t.y -= step * acc[1]; t.z -= step * acc[2]; t.w -= step * acc[3];
        *reinterpret_cast<float4 *>(theta + j0) = t;
      } else {
        for (int q = 0; q < 4 && j0 + q < P; ++q) theta[j0 + q] -= step * acc[q];
      }
    }
  }
}

__global__ __launch_bounds__(256) void finalize_kernel(const FinalizeArgs fa, float *__restrict__ out, long P,
                                                        float noise_std, uint32_t k0, uint32_t k1,
                                                        float *__restrict__ theta, float step) {
  __shared__ float4 red[240];
  int r = 0;
  while (r < fa.nreg - 1 && (int)blockIdx.x >= fa.reg[r + 1].wg0) ++r; // (the same for the whole workgroup)
  const FinalizeRegion &rg = fa.reg[r];
  if (rg.sg == 16) finalize_body<16>(fa, rg, red, out, P, noise_std, k0, k1, theta, step);
  else if (rg.sg == 4) finalize_body<4>(fa, rg, red, out, P, noise_std, k0, k1, theta, step);
  else finalize_body<1>(fa, rg, red, out, P, noise_std, k0, k1, theta, step);
}

// The launch: the regions (runs of tensors that take the same number of split groups) and their workgroups.  The
// tensors of fa lie one after the other in [0, P).  Sixteen split groups (64 coordinates per workgroup) where a
// tensor has many partial rows, or a few in a short vector (which would otherwise leave most CUs without a
// workgroup); four for a few rows; one (1,024 coordinates) for a tensor that arrives in at most two rows.
static inline void launch_finalize(hipStream_t st, FinalizeArgs &fa, float *out, long P, float noise_std, uint32_t k0,
                                   uint32_t k1, float *theta, float step) {
  fa.nreg = 0;
  int wg = 0;
  for (int i = 0; i < fa.nseg; ++i) {
    const FinalizeSeg &g = fa.seg[i];
    const int ns = g.nsplit;
    const int sg = (ns >= 24 || (P < 100000 && ns >= 3)) ? 16 : ns >= 3 ? 4 : 1;
    const long b0 = (g.p_off + 3) / 4, b1 = i == fa.nseg - 1 ? (P + 3) / 4 : (g.p_off + g.n + 3) / 4;
    if (fa.nreg > 0 && fa.reg[fa.nreg - 1].sg == sg) { fa.reg[fa.nreg - 1].blk1 = b1; continue; }
    if (fa.nreg > 0) {
      const FinalizeRegion &q = fa.reg[fa.nreg - 1];
      wg += (int)((q.blk1 - q.blk0 + 256 / q.sg - 1) / (256 / q.sg));
    }
    FinalizeRegion &r = fa.reg[fa.nreg++];
    r.blk0 = fa.nreg == 1 ? 0 : b0; r.blk1 = b1; r.wg0 = wg; r.sg = sg; r.seg0 = i;
  }
  if (fa.nreg > 0) {
    const FinalizeRegion &q = fa.reg[fa.nreg - 1];
    wg += (int)((q.blk1 - q.blk0 + 256 / q.sg - 1) / (256 / q.sg));
  }
  if (wg == 0) return;
  dim3 grid((unsigned)wg), block(256);
  hipLaunchKernelGGL(finalize_kernel, grid, block, 0, st, fa, out, P, noise_std, k0, k1, theta, step);
}

// Sequence kernels: the LSTM recurrence (forward and back-propagation through
// time) and the embedding layer's per-example norm / clipped scatter-add.
//
// The recurrence is a chain of T dependent (examples x H)*(H x 4H) products; per step it is far too small for a
// tiled contraction, and examples are independent.  Each workgroup of LSTM_THREADS threads therefore owns one
// example for the whole sequence and keeps W_hh in registers (forward: a quarter of the rows for the four gate
// columns of one hidden unit per thread, summed over a quad of lanes with DPP moves; backward: one gate's part
// of a row per thread), so a step costs no weight traffic at all: only the hidden state goes through LDS
// (broadcast reads).  A step is a chain of dependent phases, so what bounds it is latency: eight waves per
// example (two per SIMD) overlap each other's LDS reads, and every global load is issued a whole step before its
// value is used.  The input projection x_t W_ih + b and the input / weight gradients are hoisted out of the loop
// into the tiled MFMA contraction.  The [B, T, 4H] buffer is reused in place: input projection -> activated
// gates (forward) -> gate gradients (backward).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_misc.h"

#define LSTM_THREADS 512

// x_{b,t} = E[tok[b,t]]: the embedding lookup, written once per step so that the three
// contractions that read it (input projection, per-example and clipped weight gradient)
// address it directly instead of chasing the token id first.
__global__ void emb_gather_kernel(const int *__restrict__ tok, const float *__restrict__ table,
                                  float *__restrict__ xseq, long rows, int D) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * D) return;
  long r = i / D;
  int e = (int)(i - r * D);
  xseq[i] = table[(long)tok[r] * D + e];
}

// The same lookup for rows that are whole 16-byte groups (D a multiple of 4, both pointers 16-byte aligned): a thread
// copies four coordinates, a row's groups lie in consecutive threads.
__global__ void emb_gather4_kernel(const int *__restrict__ tok, const float4 *__restrict__ table,
                                   float4 *__restrict__ xseq, long rows, int D4) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * D4) return;
  const long r = i / D4;
  const int e = (int)(i - r * D4);
  xseq[i] = table[(long)tok[r] * D4 + e];
}

__device__ __forceinline__ float sigmoidf_(float v) { return fast_sigmoid(v); }

// Mean over the T step vectors of a sequence (embedding network, Appendix B): out[b, e] = (1/T) sum_t in[b, t, e].
// One workgroup per example: thread (tl, e) sums the steps tl, tl + ntl, ... of coordinate e (consecutive threads
// read consecutive coordinates of one step), the ntl partial sums of a coordinate are added in a fixed order.
__global__ __launch_bounds__(256) void seq_mean_fwd_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                            int T, int D) {
  __shared__ float part[256];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int dp = D < 256 ? D : 256, ntl = 256 / dp;
  const int e_l = tid % dp, tl = tid / dp;
  const float *p = in + (long)b * T * D;
  for (int e0 = 0; e0 < D; e0 += dp) {
    const int e = e0 + e_l;
    float s = 0.f;
    if (tl < ntl && e < D)
      for (int t = tl; t < T; t += ntl) s += p[(long)t * D + e];
    part[tid] = s;
    __syncthreads();
    if (tl == 0 && e < D) {
      float tot = 0.f;
      for (int q = 0; q < ntl; ++q) tot += part[q * dp + e_l];
      out[(long)b * D + e] = tot / (float)T;
    }
    __syncthreads();
  }
}

// ... and its gradient: every step receives g[b, e] / T.  One thread per (b, t, e).
__global__ void seq_mean_bwd_kernel(const float *__restrict__ g, float *__restrict__ gin, long n, int T, int D) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const long bt = i / D;
  const int e = (int)(i - bt * D);
  const long b = bt / T;
  gin[i] = g[b * D + e] / (float)T;
}

// Lane-relative access on a uniform base pointer with an unsigned byte offset: one address register per access
// (a signed or pre-scaled index would be widened to 64 bits per lane).
__device__ __forceinline__ float &lane_at(float *base, unsigned byte_off) {
  return *reinterpret_cast<float *>(reinterpret_cast<char *>(base) + byte_off);
}
__device__ __forceinline__ float lane_ld(const float *base, unsigned byte_off) {
  return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(base) + byte_off);
}

// Quad-lane helpers: the four lanes 4u .. 4u+3 exchange values with DPP moves (no LDS, no barrier).
__device__ __forceinline__ float quad_xor1(float v) { // lanes swap within pairs: quad_perm [1,0,3,2]
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_xor2(float v) { // pairs swap: quad_perm [2,3,0,1]
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
}
template <int Q>
__device__ __forceinline__ float quad_bcast(float v) { // every lane of the quad gets lane Q's value
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), Q * 0x55, 0xF, 0xF, true));
}

// Forward.  gates: in  x_t W_ih + b for every (b, t); out activated i, f, g, o.
// hs, cs: [B, T, H] hidden and cell states; hlast [B, H] = h_T (null: not wanted).  H <= 128, HP >= H.
// Thread (u = tid / 4, q = tid % 4) belongs to hidden unit u and holds, for all four gates
// of that unit, the quarter q of the rows of W_hh (k in [q*QL, q*QL + QL)).  A step is then: quarter product (QL
// broadcast words of h from LDS instead of all H), sum over the quad with two DPP exchanges per gate, lane q
// activates and stores gate q, the quad shares the four activated gates, every lane updates the unit's cell
// state, lane 0 publishes h.  h is double-buffered in LDS, so ONE barrier per step suffices: a step reads one
// buffer and writes the other, and every wave has finished reading a buffer before the barrier after which it is
// written again.
template <int HP>
__global__ __launch_bounds__(LSTM_THREADS) void lstm_fwd_kernel(float *__restrict__ gates, const float *__restrict__ Whh,
                                                                      float *__restrict__ hs, float *__restrict__ cs,
                                                                      float *__restrict__ hlast, int B, int T, int H) {
  constexpr int QL = (HP + 3) / 4;        // rows of W_hh per quarter
  constexpr int QLP = (QL + 3) & ~3;      // the quarter's stride in LDS (16-byte aligned)
  __shared__ __attribute__((aligned(16))) float h_s[2][4 * QLP];
  const int tid = threadIdx.x;
  const int b = blockIdx.x; // the grid is exactly B workgroups
  const int G = 4 * H;
  const int u = tid >> 2, q = tid & 3;
  const bool unit_ok = u < H;
  const int ul = unit_ok ? u : 0;
  float w[4][QL];
#pragma unroll
  for (int g = 0; g < 4; ++g)
#pragma unroll
    for (int i = 0; i < QL; ++i) {
      const int k = q * QL + i;
      w[g][i] = (unit_ok && k < H) ? Whh[(long)k * G + g * H + ul] : 0.f;
    }
  for (int i = tid; i < 2 * 4 * QLP; i += LSTM_THREADS) (&h_s[0][0])[i] = 0.f;
  float c_reg = 0.f;
  const unsigned colb = 4u * (q * H + ul), ub = 4u * ul;
  const int hpos = (ul / QL) * QLP + ul % QL; // where unit u's h sits in a buffer
  float *const grow0 = gates + (long)b * T * G;
  float *const hrow0 = hs + (long)b * T * H, *const crow0 = cs + (long)b * T * H;
  __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): the weight loads end here, not at their first use inside the loop
  __syncthreads();
  auto step = [&](const int t, const float xcur, float &xnext, const float *hin, float *hout) {
    unsigned colx = colb, ux = ub; // (re-materialised inside the loop: hoisted, they would be widened to 64 bits)
    asm volatile("" : "+v"(colx), "+v"(ux));
    xnext = lane_ld(grow0 + (long)min(t + 1, T - 1) * G, colx);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const float *hq = hin + q * QLP;
#pragma unroll
    for (int i = 0; i + 4 <= QL; i += 4) {
      const float4 h4 = *reinterpret_cast<const float4 *>(hq + i);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        acc[g] = fmaf(h4.x, w[g][i], acc[g]); acc[g] = fmaf(h4.y, w[g][i + 1], acc[g]);
        acc[g] = fmaf(h4.z, w[g][i + 2], acc[g]); acc[g] = fmaf(h4.w, w[g][i + 3], acc[g]);
      }
    }
#pragma unroll
    for (int i = QL & ~3; i < QL; ++i) {
      const float hv = hq[i];
#pragma unroll
      for (int g = 0; g < 4; ++g) acc[g] = fmaf(hv, w[g][i], acc[g]);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      acc[g] += quad_xor1(acc[g]);
      acc[g] += quad_xor2(acc[g]);
    }
    // lane q activates gate q (order i, f, g, o: gate 2 is the tanh one)
    const float mine = q == 0 ? acc[0] : (q == 1 ? acc[1] : (q == 2 ? acc[2] : acc[3]));
    const float pre = mine + xcur;
    const float v = q == 2 ? fast_tanh(pre) : sigmoidf_(pre);
    if (unit_ok) lane_at(grow0 + (long)t * G, colx) = v;
    const float gi = quad_bcast<0>(v), gf = quad_bcast<1>(v), gg = quad_bcast<2>(v), go = quad_bcast<3>(v);
    c_reg = gf * c_reg + gi * gg;
    const float h = go * fast_tanh(c_reg);
    if (unit_ok && q == 0) {
      hout[hpos] = h;
      lane_at(hrow0 + (long)t * H, ux) = h;
      lane_at(crow0 + (long)t * H, ux) = c_reg;
      if (hlast != nullptr && t == T - 1) lane_at(hlast + (long)b * H, ux) = h;
    }
    __syncthreads();
  };
  float xa = lane_ld(grow0, colb), xb;
  int t = 0;
  for (; t + 1 < T; t += 2) {
    step(t, xa, xb, h_s[0], h_s[1]);
    step(t + 1, xb, xa, h_s[1], h_s[0]);
  }
  if (t < T) step(t, xa, xb, h_s[0], h_s[1]);
}

// Back-propagation through time.  gates: in activated gates, out d(loss)/d(gate pre-activations).
// One workgroup per example; thread (k = tid % 128, q = tid / 128) owns W_hh[k][qH .. qH + H), the columns of
// gate q, and computes that gate's share of dL/dh_{t-1}[k].
// SEQ = false: the loss sees h_T only, dh_out is [B, H].  SEQ = true: the layer's output is every h_t,
// dh_out is [B, T, H] and step t adds its own share to what the later steps send back.
template <int HP, bool SEQ>
__global__ __launch_bounds__(LSTM_THREADS, (HP <= 100 ? 4 : 2)) void lstm_bwd_kernel(float *__restrict__ gates, const float *__restrict__ cs,
                                                                 const float *__restrict__ Whh,
                                                                 const float *__restrict__ dh_out, int B, int T, int H) {
  __shared__ __attribute__((aligned(16))) float dg_s[4 * HP]; // gate-major, each gate padded to HP (zeros)
  __shared__ float part_s[4][128];
  const int tid = threadIdx.x;
  const int b = blockIdx.x; // the grid is exactly B workgroups
  const int G = 4 * H;
  const int k = tid & 127, q = tid >> 7;
  float w[HP];
#pragma unroll
  for (int j = 0; j < HP; ++j) w[j] = (k < H && j < H) ? Whh[(long)k * G + q * H + j] : 0.f;
  for (int i = tid; i < 4 * HP; i += LSTM_THREADS) dg_s[i] = 0.f;
  for (int i = tid; i < 4 * 128; i += LSTM_THREADS) (&part_s[0][0])[i] = 0.f;
  const bool upd_thread = tid < H;
  const int ur = upd_thread ? tid : 0;
  const unsigned urb = 4u * ur;
  float *const grow0 = gates + (long)b * T * G;
  const float *const crow0 = cs + (long)b * T * H;
  const float *const drow0 = SEQ ? dh_out + (long)b * T * H : dh_out + (long)b * H;
  // Operands of the step being processed, held by the cell-update threads only.  They are declared without a
  // value and loaded and used inside the same branch: an initial value, a load under one branch used under
  // another, or a loaded value copied into a second variable would each be waited for at once, not at the use.
  float gi, gf, gg, go, cp, dh_own, ct;
  float dc = 0.f;
  if (upd_thread) {
    const float *g = grow0 + (long)(T - 1) * G;
    gi = lane_ld(g, urb); gf = lane_ld(g + H, urb); gg = lane_ld(g + 2 * H, urb); go = lane_ld(g + 3 * H, urb);
    ct = lane_ld(crow0 + (long)(T - 1) * H, urb);
    cp = lane_ld(crow0 + (long)max(T - 2, 0) * H, urb); // c_{t-1}; unused at t = 0
    dh_own = SEQ ? lane_ld(drow0 + (long)(T - 1) * H, urb) : lane_ld(drow0, urb);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): the weight loads end here, not at their first use inside the loop
  __syncthreads();
  for (int t = T - 1; t >= 0; --t) {
    if (upd_thread) { // (the waves without a cell-update thread skip this)
      // (lane offset re-materialised inside the loop: hoisted out of it, it would be widened to 64 bits)
      unsigned urx = urb;
      asm volatile("" : "+v"(urx));
      // what the later steps send back (zero at the last step: part_s starts cleared) plus the loss's own share
      float dh = (part_s[0][ur] + part_s[1][ur]) + (part_s[2][ur] + part_s[3][ur]);
      if (SEQ || t == T - 1) dh += dh_own;
      const float cprev = t > 0 ? cp : 0.f;
      const float tc = fast_tanh(ct);
      const float dct = dc + dh * go * (1.f - tc * tc);
      const float d_o = dh * tc * go * (1.f - go);
      const float d_i = dct * gg * gi * (1.f - gi);
      const float d_f = dct * cprev * gf * (1.f - gf);
      const float d_g = dct * gi * (1.f - gg * gg);
      dc = dct * gf;
      float *g = grow0 + (long)t * G;
      lane_at(g, urx) = d_i; lane_at(g + H, urx) = d_f; lane_at(g + 2 * H, urx) = d_g; lane_at(g + 3 * H, urx) = d_o;
      dg_s[ur] = d_i; dg_s[HP + ur] = d_f; dg_s[2 * HP + ur] = d_g; dg_s[3 * HP + ur] = d_o;
      // operands of step t - 1 (row clamped at the first step) into the registers just freed; they land while
      // the product below runs
      const int tn = max(t - 1, 0);
      const float *gn = grow0 + (long)tn * G;
      gi = lane_ld(gn, urx); gf = lane_ld(gn + H, urx); gg = lane_ld(gn + 2 * H, urx); go = lane_ld(gn + 3 * H, urx);
      ct = lane_ld(crow0 + (long)tn * H, urx); // (loaded again rather than copied from cp: see above)
      cp = lane_ld(crow0 + (long)max(tn - 1, 0) * H, urx);
      if (SEQ) dh_own = lane_ld(drow0 + (long)tn * H, urx);
    }
    __syncthreads();
    if (t > 0) {
      float acc = 0.f; // (two waves per SIMD alternate, which covers the latency of the dependent chain)
#pragma unroll
      for (int j = 0; j < HP; j += 4) {
        const float4 d4 = *reinterpret_cast<const float4 *>(&dg_s[q * HP + j]);
        acc = fmaf(d4.x, w[j], acc); acc = fmaf(d4.y, w[j + 1], acc);
        acc = fmaf(d4.z, w[j + 2], acc); acc = fmaf(d4.w, w[j + 3], acc);
      }
      part_s[q][k] = acc;
    }
    __syncthreads();
  }
}

// Embedding layer, per-example squared norm: row v of g_i is the sum of dx_{i,t}
// over the steps t whose token is v, so repeated tokens are added before squaring.
// One workgroup per example: bitonic sort of (token, t) keys in LDS, then a chunked
// segmented sum over the sorted steps.
#define EMB_TMAX 1024
#define EMB_NC 16 // chunks of the sorted steps
// Bitonic sort of KPT*256 keys, element m*256 + tid in kr[m]: exchanges at distance >= 256 stay inside the thread,
// distances 64 and 128 go through LDS (3 such passes for 256 keys), the shorter ones are wave shuffles.
template <int KPT>
__device__ __forceinline__ void emb_sort_keys(uint32_t (&kr)[KPT], uint32_t *key, const int tid) {
  constexpr int N = KPT * 256;
#pragma unroll
  for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      if (j >= 256) {
#pragma unroll
        for (int m = 0; m < KPT; ++m) {
          const int pm = m ^ (j >> 8);
          if (pm > m) {
            const bool up = (((m << 8) + tid) & k) == 0;
            const uint32_t a = kr[m], c = kr[pm];
            if ((a > c) == up) { kr[m] = c; kr[pm] = a; }
          }
        }
      } else {
        if (j >= 64) {
#pragma unroll
          for (int m = 0; m < KPT; ++m) key[(m << 8) + tid] = kr[m];
          __syncthreads();
        }
#pragma unroll
        for (int m = 0; m < KPT; ++m) {
          const int i = (m << 8) + tid;
          const uint32_t other = j >= 64 ? key[i ^ j] : (uint32_t)__shfl_xor((int)kr[m], j, 64);
          const bool keep_min = ((i & j) == 0) == ((i & k) == 0);
          kr[m] = keep_min ? min(kr[m], other) : max(kr[m], other);
        }
        if (j >= 64) __syncthreads();
      }
    }
  }
}

template <int KPT>
__global__ __launch_bounds__(256) void emb_norm_kernel(const int *__restrict__ tok, const float *__restrict__ dx,
                                                        float *__restrict__ slot, int T, int D) {
  __shared__ uint32_t key[EMB_TMAX];
  __shared__ float red[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  uint32_t kr[KPT];
#pragma unroll
  for (int m = 0; m < KPT; ++m) {
    const int i = (m << 8) + tid;
    kr[m] = i < T ? (((uint32_t)tok[(long)b * T + i] << 10) | (uint32_t)i) : 0xFFFFFFFFu;
  }
  emb_sort_keys<KPT>(kr, key, tid);
#pragma unroll
  for (int m = 0; m < KPT; ++m) key[(m << 8) + tid] = kr[m];
  __syncthreads();
  // Segmented sum over the sorted steps, in a fixed order.  The T steps are cut into EMB_NC chunks; a work item
  // (coordinate e, chunk c) walks its chunk: runs of one token that lie inside the chunk are squared at once, the
  // part before the chunk's first run start (lead) and after its last one (tail) are left for the pass below,
  // where one thread per coordinate stitches the chunks together.  (A single walk over all T steps per
  // coordinate leaves all but D threads idle behind T dependent loads.)
  constexpr int ET = 128;                 // coordinates per tile
  __shared__ float lead[EMB_NC][ET], tail[EMB_NC][ET];
  __shared__ int has_head[EMB_NC];
  const int L = (T + EMB_NC - 1) / EMB_NC;
  float tot = 0.f;
  for (int e0 = 0; e0 < D; e0 += ET) {
    const int de = min(ET, D - e0);
    for (int it = tid; it < de * EMB_NC; it += 256) {
      const int c = it / de, e = e0 + (it - c * de);
      const int p0 = c * L, p1 = min(T, p0 + L);
      float acc = 0.f, ld = 0.f;
      bool seen = false;
      uint32_t prev = p0 > 0 && p0 < p1 ? key[p0 - 1] >> 10 : 0xFFFFFFFFu; // (no token has this value: step 0 is a head)
      for (int pb = p0; pb < p1; pb += 8) { // eight loads in flight, then their sums in order
        float v[8];
        uint32_t kk[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          kk[j] = key[min(pb + j, p1 - 1)];
          v[j] = dx[((long)b * T + (kk[j] & 1023u)) * D + e];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (pb + j < p1) {
            const uint32_t tk = kk[j] >> 10;
            if (tk != prev) {
              if (seen) tot += acc * acc; else ld = acc;
              acc = 0.f; seen = true; prev = tk;
            }
            acc += v[j];
          }
      }
      lead[c][e - e0] = seen ? ld : acc;
      tail[c][e - e0] = seen ? acc : 0.f;
      if (e == e0) has_head[c] = seen;
    }
    __syncthreads();
    if (tid < de) {
      float carry = 0.f;
      for (int c = 0; c < EMB_NC; ++c) {
        carry += lead[c][tid];
        if (has_head[c]) { tot += carry * carry; carry = tail[c][tid]; }
      }
      tot += carry * carry;
    }
    __syncthreads();
  }
  for (int o = 32; o > 0; o >>= 1) tot += __shfl_xor(tot, o, 64);
  if ((tid & 63) == 0) red[tid >> 6] = tot;
  __syncthreads();
  if (tid == 0) slot[b] = red[0] + red[1] + red[2] + red[3];
}

// Clipped sum of the embedding gradient, G_E[v, :] = sum over steps (b, t) with
// tok[b, t] = v of s_b * dx[b, t, :], as a segmented reduction instead of one float
// atomic per element: the steps are bucketed by token with a counting sort (integer
// atomics only), every bucket is cut into chunks of EMB_CH steps, and one workgroup
// sums one chunk.  A token that fits in one chunk is written with plain stores; only
// the few hot tokens that span several chunks combine with fp32 atomics.
#define EMB_CH 64

#define EMB_LDS_V 12288 // vocabularies up to this size get a per-workgroup LDS histogram

// count[v] += occurrences of v.  A Zipf-distributed batch sends a large share of its
// steps to a handful of tokens, and same-address global atomics serialise, so each
// workgroup of 1024 steps first counts in LDS and issues one global atomic per
// distinct token it saw (the thread that hit the LDS bin first owns the flush).
__global__ __launch_bounds__(1024) void emb_count_kernel(const int *__restrict__ tok, int *__restrict__ count, long n,
                                                          int V) {
  extern __shared__ int bins[];
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (V > EMB_LDS_V) { if (i < n) atomicAdd(&count[tok[i]], 1); return; }
  for (int v = threadIdx.x; v < V; v += 1024) bins[v] = 0;
  __syncthreads();
  int t = -1, old = -1;
  if (i < n) { t = tok[i]; old = atomicAdd(&bins[t], 1); }
  __syncthreads();
  if (old == 0) atomicAdd(&count[t], bins[t]);
}

// one workgroup of 1024: exclusive scans of count[v] (-> start[v]) and of the chunk
// counts ceil(count[v]/EMB_CH) (-> chunk0[v]); start[V], chunk0[V] hold the totals;
// cursor[v] is reset to 0 for the fill pass.
__global__ __launch_bounds__(1024) void emb_scan_kernel(const int *__restrict__ count, int *__restrict__ start,
                                                         int *__restrict__ chunk0, int *__restrict__ cursor, int V) {
  __shared__ int wa[16], wb[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (V + 1023) / 1024;
  const int lo = min(V, tid * per), hi = min(V, lo + per);
  int a = 0, b = 0;
  for (int v = lo; v < hi; ++v) { a += count[v]; b += (count[v] + EMB_CH - 1) / EMB_CH; }
  // inclusive scan of the 1024 range totals: shuffles inside a wave, then the 16 wave totals
  int ia = a, ib = b;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int xa = __shfl_up(ia, o, 64), xb = __shfl_up(ib, o, 64);
    if (lane >= o) { ia += xa; ib += xb; }
  }
  if (lane == 63) { wa[wave] = ia; wb[wave] = ib; }
  __syncthreads();
  if (wave == 0) {
    int ta = lane < 16 ? wa[lane] : 0, tb = lane < 16 ? wb[lane] : 0;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int xa = __shfl_up(ta, o, 64), xb = __shfl_up(tb, o, 64);
      if (lane >= o) { ta += xa; tb += xb; }
    }
    if (lane < 16) { wa[lane] = ta; wb[lane] = tb; }
  }
  __syncthreads();
  const int offa = wave > 0 ? wa[wave - 1] : 0, offb = wave > 0 ? wb[wave - 1] : 0;
  int ra = offa + ia - a, rb = offb + ib - b; // exclusive prefix of this thread's range
  for (int v = lo; v < hi; ++v) {
    start[v] = ra; chunk0[v] = rb; cursor[v] = 0;
    ra += count[v]; rb += (count[v] + EMB_CH - 1) / EMB_CH;
  }
  if (tid == 1023) { start[V] = wa[15]; chunk0[V] = wb[15]; }
}

// list[start[v] + rank] = step index, rank unique within the bucket: the workgroup reserves a
// range of its bucket with one global atomic per distinct token, steps take their rank in LDS.
__global__ __launch_bounds__(1024) void emb_fill_kernel(const int *__restrict__ tok, const int *__restrict__ start,
                                                         int *__restrict__ cursor, int *__restrict__ list, long n,
                                                         int V) {
  extern __shared__ int bins[];
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (V > EMB_LDS_V) {
    if (i < n) { const int v = tok[i]; list[start[v] + atomicAdd(&cursor[v], 1)] = (int)i; }
    return;
  }
  for (int v = threadIdx.x; v < V; v += 1024) bins[v] = 0;
  __syncthreads();
  int t = -1, old = -1;
  if (i < n) { t = tok[i]; old = atomicAdd(&bins[t], 1); }
  __syncthreads();
  if (old == 0) bins[t] = atomicAdd(&cursor[t], bins[t]); // the bin now holds this workgroup's base rank
  __syncthreads();
  if (i < n) list[start[t] + bins[t] + old] = (int)i;
}

// The three kernels above in one launch, for small batches (up to 2^15 steps, vocabularies that fit the LDS
// histogram): count in LDS, scan, then hand out the positions of every bucket from LDS cursors.  One workgroup walks
// through all the steps twice, so its time grows with the batch -- measured 98 us at 131,072 Zipf-distributed steps
// (the hot tokens serialise the LDS atomics) against 57 us for the three launches -- while three launches cost
// 15-20 us each however small the batch; hence the limit.  The order of the steps inside a bucket depends on the
// order in which the LDS atomics retire, as it does with the three-kernel route.
#define EMB_ONE_MAX_ROWS (1 << 15)
__global__ __launch_bounds__(1024) void emb_bucket_one_kernel(const int *__restrict__ tok, int *__restrict__ start,
                                                               int *__restrict__ chunk0, int *__restrict__ list, int n,
                                                               int V) {
  extern __shared__ int bins[]; // [V]
  __shared__ int wa[16], wb[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int v = tid; v < V; v += 1024) bins[v] = 0;
  __syncthreads();
  for (int i = tid; i < n; i += 1024) atomicAdd(&bins[tok[i]], 1);
  __syncthreads();
  // exclusive scans of the counts and of the chunk counts; every thread owns a run of consecutive tokens
  const int per = (V + 1023) / 1024;
  const int lo = min(V, tid * per), hi = min(V, lo + per);
  int a = 0, b = 0;
  for (int v = lo; v < hi; ++v) { const int c = bins[v]; a += c; b += (c + EMB_CH - 1) / EMB_CH; }
  int ia = a, ib = b;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int xa = __shfl_up(ia, o, 64), xb = __shfl_up(ib, o, 64);
    if (lane >= o) { ia += xa; ib += xb; }
  }
  if (lane == 63) { wa[wave] = ia; wb[wave] = ib; }
  __syncthreads();
  if (wave == 0) {
    int ta = lane < 16 ? wa[lane] : 0, tb = lane < 16 ? wb[lane] : 0;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int xa = __shfl_up(ta, o, 64), xb = __shfl_up(tb, o, 64);
      if (lane >= o) { ta += xa; tb += xb; }
    }
    if (lane < 16) { wa[lane] = ta; wb[lane] = tb; }
  }
  __syncthreads();
  int ra = (wave > 0 ? wa[wave - 1] : 0) + ia - a, rb = (wave > 0 ? wb[wave - 1] : 0) + ib - b;
  for (int v = lo; v < hi; ++v) {
    const int c = bins[v];
    start[v] = ra; chunk0[v] = rb;
    bins[v] = ra; // the bucket's cursor for the fill pass
    ra += c; rb += (c + EMB_CH - 1) / EMB_CH;
  }
  if (tid == 1023) { start[V] = wa[15]; chunk0[V] = wb[15]; }
  __syncthreads();
  for (int i = tid; i < n; i += 1024) list[atomicAdd(&bins[tok[i]], 1)] = i;
}

// one workgroup per chunk; workgroups past the last chunk exit.  acc must be zero
// on entry (rows of tokens that do not occur stay zero).
__global__ __launch_bounds__(256) void emb_reduce_kernel(const int *__restrict__ start, const int *__restrict__ chunk0,
                                                          const int *__restrict__ list, const float *__restrict__ dx,
                                                          const float *__restrict__ scale, float *__restrict__ acc,
                                                          int V, int T, int D) {
  __shared__ int ent[EMB_CH];
  __shared__ float sc[EMB_CH];
  __shared__ float part[256];
  const int chunk = blockIdx.x;
  if (chunk >= chunk0[V]) return;
  // token whose chunk range contains `chunk`: last v with chunk0[v] <= chunk
  int lo = 0, hi = V;
  while (hi - lo > 1) { int mid = (lo + hi) >> 1; if (chunk0[mid] <= chunk) lo = mid; else hi = mid; }
  const int v = lo, ci = chunk - chunk0[v];
  const int cnt = start[v + 1] - start[v];
  const int e0 = ci * EMB_CH, n = min(EMB_CH, cnt - e0);
  const int tid = threadIdx.x;
  if (tid < n) {
    const int en = list[start[v] + e0 + tid];
    ent[tid] = en;
    sc[tid] = scale ? scale[en / T] : 1.f;
  }
  __syncthreads();
  // two groups of 128 threads each take every other step; thread e < D of a group owns coordinate e
  const int grp = tid >> 7, e = tid & 127;
  for (int ebase = 0; ebase < D; ebase += 128) {
    float a = 0.f;
    if (ebase + e < D)
      for (int i = grp; i < n; i += 2) a += sc[i] * dx[(long)ent[i] * D + ebase + e];
    part[tid] = a;
    __syncthreads();
    if (grp == 0 && ebase + e < D) {
      const float tot = part[e] + part[128 + e];
      float *dst = acc + (long)v * D + ebase + e;
      if (cnt <= EMB_CH) *dst = tot; else unsafeAtomicAdd(dst, tot);
    }
    __syncthreads();
  }
}

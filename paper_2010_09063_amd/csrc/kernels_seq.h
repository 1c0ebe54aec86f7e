// Sequence kernels: the LSTM recurrence (forward and back-propagation through
// time) and the embedding layer's per-example norm / clipped scatter-add.
//
// The recurrence is a chain of T dependent (examples x H)*(H x 4H) products; per
// step it is far too small for a tiled contraction, and examples are
// independent.  Each workgroup therefore owns LSTM_NE examples for the whole
// sequence and keeps W_hh in registers (two gate columns per thread forward, half
// a row per thread backward), so a step costs no weight traffic at all: only the
// hidden state goes through LDS (broadcast reads).  The input projection
// x_t W_ih + b and the input / weight gradients are hoisted out of the loop into
// the tiled MFMA contraction.  The [B, T, 4H] buffer is reused in place: input
// projection -> activated gates (forward) -> gate gradients (backward).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_misc.h"

#define LSTM_NE 2

__device__ __forceinline__ float sigmoidf_(float v) { return fast_sigmoid(v); }

// Forward.  gates: in  x_t W_ih + b for every (b, t); out activated i, f, g, o.
// hs, cs: [B, T, H] hidden and cell states; hlast [B, H] = h_T.
// Thread j < 2H owns columns j and j + 2H of W_hh (H <= 128, HP = H rounded up to 4).
template <int HP>
__global__ __launch_bounds__(256) void lstm_fwd_kernel(float *__restrict__ gates, const float *__restrict__ Whh,
                                                        float *__restrict__ hs, float *__restrict__ cs,
                                                        float *__restrict__ hlast, int B, int T, int H) {
  __shared__ __attribute__((aligned(16))) float h_s[LSTM_NE][HP];
  __shared__ float gact[LSTM_NE][4 * HP];
  const int tid = threadIdx.x;
  const int b0 = blockIdx.x * LSTM_NE;
  const int G = 4 * H;
  const bool col_thread = tid < 2 * H;
  const int c0 = tid, c1 = tid + 2 * H;
  float w0[HP], w1[HP];
#pragma unroll
  for (int k = 0; k < HP; ++k) {
    w0[k] = (col_thread && k < H) ? Whh[(long)k * G + c0] : 0.f;
    w1[k] = (col_thread && k < H) ? Whh[(long)k * G + c1] : 0.f;
  }
  for (int i = tid; i < LSTM_NE * HP; i += 256) (&h_s[0][0])[i] = 0.f;
  // cell-update role: thread (e, r)
  const int ue = tid / H, ur = tid - ue * H;
  const bool upd_thread = tid < LSTM_NE * H && (b0 + ue) < B;
  float c_reg = 0.f;
  float xp[LSTM_NE][2];
#pragma unroll
  for (int e = 0; e < LSTM_NE; ++e) {
    const bool ok = col_thread && (b0 + e) < B;
    xp[e][0] = ok ? gates[((long)(b0 + e) * T) * G + c0] : 0.f;
    xp[e][1] = ok ? gates[((long)(b0 + e) * T) * G + c1] : 0.f;
  }
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    float acc[LSTM_NE][2];
#pragma unroll
    for (int e = 0; e < LSTM_NE; ++e) { acc[e][0] = xp[e][0]; acc[e][1] = xp[e][1]; }
    if (t + 1 < T) {
#pragma unroll
      for (int e = 0; e < LSTM_NE; ++e) {
        const bool ok = col_thread && (b0 + e) < B;
        xp[e][0] = ok ? gates[((long)(b0 + e) * T + t + 1) * G + c0] : 0.f;
        xp[e][1] = ok ? gates[((long)(b0 + e) * T + t + 1) * G + c1] : 0.f;
      }
    }
    if (t > 0) {
#pragma unroll
      for (int k = 0; k < HP; k += 4) {
#pragma unroll
        for (int e = 0; e < LSTM_NE; ++e) {
          const float4 h4 = *reinterpret_cast<const float4 *>(&h_s[e][k]);
          acc[e][0] = fmaf(h4.x, w0[k], acc[e][0]); acc[e][1] = fmaf(h4.x, w1[k], acc[e][1]);
          acc[e][0] = fmaf(h4.y, w0[k + 1], acc[e][0]); acc[e][1] = fmaf(h4.y, w1[k + 1], acc[e][1]);
          acc[e][0] = fmaf(h4.z, w0[k + 2], acc[e][0]); acc[e][1] = fmaf(h4.z, w1[k + 2], acc[e][1]);
          acc[e][0] = fmaf(h4.w, w0[k + 3], acc[e][0]); acc[e][1] = fmaf(h4.w, w1[k + 3], acc[e][1]);
        }
      }
    }
    if (col_thread) {
      // columns [0,H) i, [H,2H) f, [2H,3H) g, [3H,4H) o: c0 < 2H is i or f, c1 = c0+2H is g or o
      const bool c1_is_g = c1 < 3 * H;
#pragma unroll
      for (int e = 0; e < LSTM_NE; ++e) {
        const float v0 = sigmoidf_(acc[e][0]);
        const float v1 = c1_is_g ? fast_tanh(acc[e][1]) : sigmoidf_(acc[e][1]);
        gact[e][c0] = v0; gact[e][c1] = v1;
        if (b0 + e < B) {
          gates[((long)(b0 + e) * T + t) * G + c0] = v0;
          gates[((long)(b0 + e) * T + t) * G + c1] = v1;
        }
      }
    }
    __syncthreads();
    if (upd_thread) {
      const float gi = gact[ue][ur], gf = gact[ue][H + ur], gg = gact[ue][2 * H + ur], go = gact[ue][3 * H + ur];
      c_reg = gf * c_reg + gi * gg;
      const float h = go * fast_tanh(c_reg);
      h_s[ue][ur] = h;
      const long o = ((long)(b0 + ue) * T + t) * H + ur;
      hs[o] = h; cs[o] = c_reg;
      if (t == T - 1) hlast[(long)(b0 + ue) * H + ur] = h;
    }
    __syncthreads();
  }
}

// Back-propagation through time.  gates: in activated gates, out d(loss)/d(gate
// pre-activations).  Thread (k = tid % 128, q = tid / 128) owns W_hh[k][q*2H .. q*2H+2H).
template <int HP>
__global__ __launch_bounds__(256) void lstm_bwd_kernel(float *__restrict__ gates, const float *__restrict__ cs,
                                                        const float *__restrict__ Whh,
                                                        const float *__restrict__ dh_last, int B, int T, int H) {
  constexpr int DG_LD = 2 * HP; // per half, padded so that float4 reads stay aligned
  __shared__ __attribute__((aligned(16))) float dg_s[LSTM_NE][2 * DG_LD];
  __shared__ float part_s[LSTM_NE][2][128];
  const int tid = threadIdx.x;
  const int b0 = blockIdx.x * LSTM_NE;
  const int G = 4 * H;
  const int k = tid & 127, q = tid >> 7;
  float w[DG_LD];
#pragma unroll
  for (int j = 0; j < DG_LD; ++j) w[j] = (k < H && j < 2 * H) ? Whh[(long)k * G + q * 2 * H + j] : 0.f;
  for (int i = tid; i < LSTM_NE * 2 * DG_LD; i += 256) (&dg_s[0][0])[i] = 0.f;
  const int ue = tid / H, ur = tid - ue * H;
  const bool upd_thread = tid < LSTM_NE * H && (b0 + ue) < B;
  const long ub = b0 + ue;
  float dc = 0.f;
  float gi = 0.f, gf = 0.f, gg = 0.f, go = 0.f, ct = 0.f, cp = 0.f;
  if (upd_thread) {
    const long o = (ub * T + (T - 1));
    gi = gates[o * G + ur]; gf = gates[o * G + H + ur]; gg = gates[o * G + 2 * H + ur]; go = gates[o * G + 3 * H + ur];
    ct = cs[o * H + ur]; cp = T > 1 ? cs[(o - 1) * H + ur] : 0.f;
  }
  __syncthreads();
  for (int t = T - 1; t >= 0; --t) {
    if (upd_thread) {
      const float dh = (t == T - 1) ? dh_last[ub * H + ur] : part_s[ue][0][ur] + part_s[ue][1][ur];
      const float tc = fast_tanh(ct);
      const float dct = dc + dh * go * (1.f - tc * tc);
      const float d_o = dh * tc * go * (1.f - go);
      const float d_i = dct * gg * gi * (1.f - gi);
      const float d_f = dct * cp * gf * (1.f - gf);
      const float d_g = dct * gi * (1.f - gg * gg);
      dc = dct * gf;
      const long o = (ub * T + t) * G;
      gates[o + ur] = d_i; gates[o + H + ur] = d_f; gates[o + 2 * H + ur] = d_g; gates[o + 3 * H + ur] = d_o;
      // columns [0,2H) = i,f go to half 0; [2H,4H) = g,o to half 1
      dg_s[ue][ur] = d_i; dg_s[ue][H + ur] = d_f;
      dg_s[ue][DG_LD + ur] = d_g; dg_s[ue][DG_LD + H + ur] = d_o;
      if (t > 0) { // operands of the next iteration; they land while the product below runs
        const long on = (ub * T + (t - 1));
        gi = gates[on * G + ur]; gf = gates[on * G + H + ur]; gg = gates[on * G + 2 * H + ur];
        go = gates[on * G + 3 * H + ur];
        ct = cp; cp = t > 1 ? cs[(on - 1) * H + ur] : 0.f;
      }
    }
    __syncthreads();
    if (t > 0) {
      float acc[LSTM_NE];
#pragma unroll
      for (int e = 0; e < LSTM_NE; ++e) acc[e] = 0.f;
#pragma unroll
      for (int j = 0; j < DG_LD; j += 4) {
#pragma unroll
        for (int e = 0; e < LSTM_NE; ++e) {
          const float4 d4 = *reinterpret_cast<const float4 *>(&dg_s[e][q * DG_LD + j]);
          acc[e] = fmaf(d4.x, w[j], acc[e]); acc[e] = fmaf(d4.y, w[j + 1], acc[e]);
          acc[e] = fmaf(d4.z, w[j + 2], acc[e]); acc[e] = fmaf(d4.w, w[j + 3], acc[e]);
        }
      }
#pragma unroll
      for (int e = 0; e < LSTM_NE; ++e) part_s[e][q][k] = acc[e];
    }
    __syncthreads();
  }
}

// Embedding layer, per-example squared norm: row v of g_i is the sum of dx_{i,t}
// over the steps t whose token is v, so repeated tokens are added before squaring.
// One workgroup per example: bitonic sort of (token, t) keys in LDS, then every
// thread walks the sorted steps for its embedding coordinate(s).
#define EMB_TMAX 1024
__global__ __launch_bounds__(256) void emb_norm_kernel(const int *__restrict__ tok, const float *__restrict__ dx,
                                                        float *__restrict__ slot, int T, int TP, int D) {
  __shared__ uint32_t key[EMB_TMAX];
  __shared__ float red[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < TP; i += 256) key[i] = i < T ? (((uint32_t)tok[(long)b * T + i] << 10) | (uint32_t)i) : 0xFFFFFFFFu;
  __syncthreads();
  for (int k = 2; k <= TP; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < TP; i += 256) {
        int l = i ^ j;
        if (l > i) {
          uint32_t a = key[i], c = key[l];
          bool up = (i & k) == 0;
          if ((a > c) == up) { key[i] = c; key[l] = a; }
        }
      }
      __syncthreads();
    }
  float tot = 0.f;
  for (int e = tid; e < D; e += 256) {
    float acc = 0.f;
    uint32_t prev = key[0] >> 10;
    for (int p = 0; p < T; ++p) {
      const uint32_t kk = key[p];
      const uint32_t v = kk >> 10;
      if (v != prev) { tot += acc * acc; acc = 0.f; prev = v; }
      acc += dx[((long)b * T + (kk & 1023u)) * D + e];
    }
    tot += acc * acc;
  }
  for (int o = 32; o > 0; o >>= 1) tot += __shfl_xor(tot, o, 64);
  if ((tid & 63) == 0) red[tid >> 6] = tot;
  __syncthreads();
  if (tid == 0) slot[b] = red[0] + red[1] + red[2] + red[3];
}

// Clipped sum of the embedding gradient: acc[tok[b,t], :] += s_b * dx[b, t, :]
// (hardware fp32 atomics; acc is zeroed before the launch).
__global__ void emb_scatter_kernel(const int *__restrict__ tok, const float *__restrict__ dx,
                                   const float *__restrict__ scale, float *__restrict__ acc, long rows, int T,
                                   int D) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * D) return;
  long row = i / D;
  int e = (int)(i - row * D);
  float s = scale ? scale[row / T] : 1.f;
  unsafeAtomicAdd(&acc[(long)tok[row] * D + e], s * dx[i]);
}

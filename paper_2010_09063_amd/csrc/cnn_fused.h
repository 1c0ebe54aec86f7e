// The small MNIST-shaped CNN (1x28x28 -> conv 16 ch 8x8 / 2 pad 3 -> 2x2 / 1 max-pool -> conv 32 ch 4x4 / 2 ->
// 2x2 / 1 max-pool -> fc 32 -> fc 10; 26,010 parameters, Section 3's architectures paragraph and Appendix B) as ONE
// launch per private step plus the final write.
//
// Everything one example needs fits a compute unit: 45 KB of activations and backprops and 37 KB of convolution
// weights in LDS; the first fully connected layer's 64 KB of weights come from the L2.  A workgroup of 16 waves therefore takes whole examples, one
// after the other: forward, loss gradient, backward-data, the example's full gradient g_i (Section 1, item 2a), its
// norm and clip factor (item 2b), and adds s_i g_i to a partial clipped sum that lives in registers for the whole
// run (item 3) -- each thread owns 26 coordinates of the parameter vector.  The five convolution contractions run on
// v_mfma_f32_16x16x4_f32 with operands read straight from the LDS images (patches are never formed); pools, the
// fully connected layers and all reductions are plain vector code.  The workgroups' partial sums are added, in a
// fixed order, by the final write, which also adds the noise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels_misc.h"

typedef float cnn_f32x4 __attribute__((ext_vector_type(4)));

namespace cnnf {
// geometry
constexpr int H0 = 28, XP = 34;                    // input plane, padded plane (pad 3 each side)
constexpr int D1 = 16, K1 = 8, O1 = 14, P1 = 196;  // conv1: channels, filter, output plane
constexpr int Q1 = 13, R1 = 169;                   // pool1 output plane
constexpr int D2 = 32, K2 = 4, O2 = 5, P2 = 25, CK2 = 256; // conv2 (16 input channels x 4 x 4)
constexpr int Q2 = 4, F = 512;                     // pool2 output plane, flattened features
constexpr int HID = 32, NC = 10;
constexpr int LW2 = 257;                           // row length of W2 in LDS (odd: 16 rows on 16 banks)
// parameter offsets
constexpr int OFF_W1 = 0, OFF_B1 = 1024, OFF_W2 = 1040, OFF_B2 = OFF_W2 + 8192, OFF_W3 = OFF_B2 + 32;
constexpr int OFF_B3 = OFF_W3 + F * HID, OFF_W4 = OFF_B3 + HID, OFF_B4 = OFF_W4 + HID * NC, NPARAM = OFF_B4 + NC;
static_assert(NPARAM == 26010, "parameter count of the network");
// LDS layout (floats)
constexpr int L_XP = 0;                       // [34][34] zero-padded input
constexpr int L_A1 = L_XP + XP * XP;          // [16][196] conv1 activations, later Delta1
constexpr int L_P1 = L_A1 + D1 * P1;          // [16][169] pool1 output
constexpr int L_DP1 = L_P1 + D1 * R1;         // [16][169] gradient w.r.t. pool1 output
constexpr int L_A2 = L_DP1 + D1 * R1;         // [32][25] conv2 activations, later Delta2
constexpr int L_P2 = L_A2 + D2 * P2;          // [512] pool2 output
constexpr int L_DP2 = L_P2 + F;               // [512]
constexpr int L_A3 = L_DP2 + F;               // [32]
constexpr int L_D3 = L_A3 + HID;              // [32]
constexpr int L_D4 = L_D3 + HID;              // [16]
constexpr int L_RED = L_D4 + 16;              // [16 waves] + scalars
constexpr int L_SC = L_RED + 32;              // [4]: clip factor, ...
constexpr int L_W2 = L_SC + 4;                // [32][257]
constexpr int L_B = L_W2 + D2 * LW2;          // b1[16] b2[32] b3[32] b4[10] W4[320] -> 410
constexpr int L_W1 = L_B + 416;               // [16][65] conv1 weights (odd rows: 16 channels on 16 banks)
constexpr int L_COLS = L_W1 + 16 * 65 + 4;    // [256][25] columns of conv2 backward-data; also the K-split partials
constexpr int L_ARG1 = L_COLS + CK2 * P2;     // pool1 arg-max bytes (2704) as words of 4
constexpr int L_ARG2 = L_ARG1 + (D1 * R1 + 3) / 4;
constexpr int L_END = L_ARG2 + F / 4;
constexpr size_t LDS_BYTES = sizeof(float) * (size_t)L_END;
static_assert(D2 * 32 * 4 <= CK2 * P2 && D1 * 64 * 4 <= CK2 * P2, "the K-split partials fit the column buffer");
constexpr int THREADS = 1024;
} // namespace cnnf

struct CnnFusedArgs {
  const float *params; // [26010]
  const float *x;      // [B][784]
  const int *y;        // [B]
  float *part;         // [gridDim.x][pstride]
  long pstride;
  float *norms, *s;    // [B] (may be null)
  int B, act1, act2, act3;
  float C;
  int priv;
};

__global__ __launch_bounds__(cnnf::THREADS) void cnn_small_fused_kernel(const CnnFusedArgs a) {
  using namespace cnnf;
  extern __shared__ float lds[];
  float *xp = lds + L_XP, *a1 = lds + L_A1, *p1 = lds + L_P1, *dp1 = lds + L_DP1, *a2 = lds + L_A2, *p2 = lds + L_P2;
  float *dp2 = lds + L_DP2, *a3 = lds + L_A3, *d3 = lds + L_D3, *d4 = lds + L_D4, *red = lds + L_RED, *scl = lds + L_SC;
  float *w2s = lds + L_W2, *bb = lds + L_B, *cols = lds + L_COLS, *w1s = lds + L_W1;
  uint8_t *arg1 = reinterpret_cast<uint8_t *>(lds + L_ARG1), *arg2 = reinterpret_cast<uint8_t *>(lds + L_ARG2);
  const float *b1 = bb, *b2 = bb + 16, *b3 = bb + 48, *b4 = bb + 80, *w4 = bb + 96; // W4[n][j] at w4[n * 10 + j]
  const int tid0 = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);

  // ---- once per workgroup: weights into LDS / registers, zero border of the padded input
  for (int i = tid0; i < XP * XP; i += THREADS) xp[i] = 0.f;
  for (int i = tid0; i < D2 * CK2; i += THREADS) w2s[(i >> 8) * LW2 + (i & 255)] = a.params[OFF_W2 + i];
  if (tid0 < 16) bb[tid0] = a.params[OFF_B1 + tid0];
  if (tid0 < 32) { bb[16 + tid0] = a.params[OFF_B2 + tid0]; bb[48 + tid0] = a.params[OFF_B3 + tid0]; }
  if (tid0 < 10) bb[80 + tid0] = a.params[OFF_B4 + tid0];
  if (tid0 < 320) bb[96 + tid0] = a.params[OFF_W4 + tid0];
  w1s[(tid0 >> 6) * 65 + (tid0 & 63)] = a.params[OFF_W1 + tid0];

  // partial clipped sum of this workgroup's examples, by owner thread
  float acc1 = 0.f, accb = 0.f, acc4 = 0.f; // conv1 weight (d = tid0 / 64, tap = tid0 % 64); one bias (see the end); fc2 weight
  float acc2[2][4], acc3[16];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc2[i][r] = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc3[i] = 0.f;
  float accb2 = 0.f, accb3 = 0.f, accb4 = 0.f;

  float xnext = (tid0 < H0 * H0 && (int)blockIdx.x < a.B) ? a.x[(long)blockIdx.x * (H0 * H0) + tid0] : 0.f;
  int ynext = a.y[(int)blockIdx.x < a.B ? blockIdx.x : 0];
  __syncthreads();

  for (int ex = blockIdx.x; ex < a.B; ex += gridDim.x) {
    // The thread index is made opaque once per example: every phase derives its indices from it again (a few integer
    // operations) instead of the compiler keeping dozens of loop-invariant addresses alive across the whole loop,
    // which spilled registers to scratch memory -- and every barrier waits for outstanding scratch traffic.
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, i16 = lane & 15, kq = lane >> 4;
    const int fn = tid & 31, fk = tid >> 5; // fc1: output unit, block of 16 input features
    // ---- input into the padded plane; the next example's pixels are requested now
    if (tid < H0 * H0) xp[(tid / H0 + 3) * XP + tid % H0 + 3] = xnext;
    const int yy = ynext;
    __syncthreads();
    // ---- conv1 forward: [16 x 64] x [64 x 196]; wave = block of 16 positions
    if (wave < 13) {
      const int n = wave * 16 + i16, nn = n < P1 ? n : P1 - 1;
      const int base = (2 * (nn / O1)) * XP + 2 * (nn % O1);
      cnn_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        const int k = 4 * ks + kq; // tap (kh, kw) = (k / 8, k % 8)
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(w1s[i16 * 65 + k], xp[base + (k >> 3) * XP + (k & 7)], d, 0, 0, 0);
      }
      if (n < P1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) a1[(4 * kq + r) * P1 + n] = act_apply(a.act1, d[r] + b1[4 * kq + r]);
      }
    }
    __syncthreads();
    // ---- pool1 forward (2x2, stride 1): first maximum in row-major window order
    for (int i = tid; i < D1 * R1; i += THREADS) {
      const int c = i / R1, q = i - c * R1, qh = q / Q1, qw = q - qh * Q1;
      const float *w = a1 + c * P1 + qh * O1 + qw;
      float best = w[0]; int bi = 0;
      if (w[1] > best) { best = w[1]; bi = 1; }
      if (w[O1] > best) { best = w[O1]; bi = 2; }
      if (w[O1 + 1] > best) { best = w[O1 + 1]; bi = 3; }
      p1[i] = best; arg1[i] = (uint8_t)bi;
    }
    __syncthreads();
    // ---- conv2 forward: [32 x 256] x [256 x 25]; wave = (output block, quarter of K); partials meet in LDS
    {
      const int mb = wave & 1, nb = (wave >> 1) & 1, kp = wave >> 2;
      const int p = nb * 16 + i16, pp = p < P2 ? p : P2 - 1;
      const int pbase = (2 * (pp / O2)) * Q1 + 2 * (pp % O2) + kq; // + kw = kq
      const float *wrow = w2s + (mb * 16 + i16) * LW2 + kq;
      cnn_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int ks = kp * 16 + j; // k = 4 ks + kq = c * 16 + kh * 4 + kw: c = ks / 4, kh = ks % 4, kw = kq
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(wrow[4 * ks], p1[(ks >> 2) * R1 + (ks & 3) * Q1 + pbase], d, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) cols[kp * 1024 + (mb * 16 + 4 * kq + r) * 32 + p] = d[r];
    }
    __syncthreads();
    if (tid < D2 * P2) {
      const int d = tid / P2, p = tid - d * P2;
      const int o = d * 32 + p;
      a2[tid] = act_apply(a.act2, (cols[o] + cols[1024 + o]) + (cols[2048 + o] + cols[3072 + o]) + b2[d]);
    }
    __syncthreads();
    // the thread's sixteen weights of the first fully connected layer (the same every example; 64 KB in all, read
    // from the L2 rather than held in registers through the convolution phases)
    float w3r[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) w3r[i] = a.params[OFF_W3 + (fk * 16 + i) * HID + fn];
    // ---- pool2 forward
    if (tid < F) {
      const int c = tid >> 4, qh = (tid >> 2) & 3, qw = tid & 3;
      const float *w = a2 + c * P2 + qh * O2 + qw;
      float best = w[0]; int bi = 0;
      if (w[1] > best) { best = w[1]; bi = 1; }
      if (w[O2] > best) { best = w[O2]; bi = 2; }
      if (w[O2 + 1] > best) { best = w[O2 + 1]; bi = 3; }
      p2[tid] = best; arg2[tid] = (uint8_t)bi;
    }
    __syncthreads();
    // ---- fc1 forward: thread (unit fn, block fk of 16 features); 32 partial sums per unit meet in LDS
    {
      float z = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) z = fmaf(p2[fk * 16 + i], w3r[i], z);
      cols[fk * 32 + fn] = z;
    }
    __syncthreads();
    if (tid < HID) {
      float z0 = 0.f, z1 = 0.f;
#pragma unroll
      for (int k = 0; k < 32; k += 2) { z0 += cols[k * 32 + tid]; z1 += cols[(k + 1) * 32 + tid]; }
      a3[tid] = act_apply(a.act3, z0 + z1 + b3[tid]);
    }
    __syncthreads();
    // ---- fc2, loss gradient, the two dense layers' squared norms, delta3 (wave 0)
    if (wave == 0) {
      float sp2 = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) { const float v = p2[lane + 64 * i]; sp2 = fmaf(v, v, sp2); }
      const float a3v = a3[lane & 31];
      float sa3 = lane < 32 ? a3v * a3v : 0.f;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) { sp2 += __shfl_xor(sp2, o, 64); sa3 += __shfl_xor(sa3, o, 64); }
      float z = -INFINITY;
      if (lane < NC) {
        z = b4[lane];
#pragma unroll
        for (int n = 0; n < HID; ++n) z = fmaf(a3[n], w4[n * NC + lane], z);
      }
      float mx = z;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      mx = __shfl(mx, 0, 64);
      const float e = lane < NC ? expf(z - mx) : 0.f;
      float se = e;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
      se = __shfl(se, 0, 64);
      const float dv = lane < NC ? e / se - (lane == yy ? 1.f : 0.f) : 0.f;
      float sd4 = dv * dv;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) sd4 += __shfl_xor(sd4, o, 64);
      sd4 = __shfl(sd4, 0, 64);
      if (lane < 16) d4[lane] = dv;
      // delta3[n] = act'(a3[n]) * sum_j W4[n][j] delta4[j]
      float t = 0.f;
#pragma unroll
      for (int j = 0; j < NC; ++j) t = fmaf(w4[(lane & 31) * NC + j], __shfl(dv, j, 64), t);
      t *= act_deriv_from_out(a.act3, a3v);
      if (lane < 32) d3[lane] = t;
      float sd3 = lane < 32 ? t * t : 0.f;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) sd3 += __shfl_xor(sd3, o, 64);
      if (lane == 0) scl[1] = (sp2 + 1.f) * sd3 + (sa3 + 1.f) * sd4; // dense identity, both layers
    }
    __syncthreads();
    // ---- fc1 backward-data: dp2[k] = sum_n W3[k][n] delta3[n] from the weights the thread already holds: thread
    // (unit fn, features fk*16 ..) has the sixteen products W3[k][fn] delta3[fn]; the 32 lanes of a feature block
    // add them up by a halving exchange (16 + 8 + 4 + 2 + 1 lanes apart: each step a lane keeps half of its values
    // and receives the partner's sums for them), 16 exchanges instead of 80, in a fixed order
    {
      const float dn = d3[fn];
      const bool b4 = lane & 16, b3 = lane & 8, b2 = lane & 4, b1 = lane & 2;
      float u8[8], u4[4], u2[2];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float lo = w3r[j] * dn, hi = w3r[8 + j] * dn;
        u8[j] = (b4 ? hi : lo) + __shfl_xor(b4 ? lo : hi, 16, 64);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) u4[j] = (b3 ? u8[4 + j] : u8[j]) + __shfl_xor(b3 ? u8[j] : u8[4 + j], 8, 64);
#pragma unroll
      for (int j = 0; j < 2; ++j) u2[j] = (b2 ? u4[2 + j] : u4[j]) + __shfl_xor(b2 ? u4[j] : u4[2 + j], 4, 64);
      float u1 = (b1 ? u2[1] : u2[0]) + __shfl_xor(b1 ? u2[0] : u2[1], 2, 64);
      u1 += __shfl_xor(u1, 1, 64);
      if ((lane & 1) == 0) dp2[fk * 16 + (b4 ? 8 : 0) + (b3 ? 4 : 0) + (b2 ? 2 : 0) + (b1 ? 1 : 0)] = u1;
    }
    __syncthreads();
    // ---- pool2 backward (gather over the windows that hold the position) and conv2's activation derivative
    if (tid < D2 * P2) {
      const int d = tid / P2, p = tid - d * P2, ph = p / O2, pw = p - ph * O2;
      float g = 0.f;
#pragma unroll
      for (int dh = 0; dh < 2; ++dh)
#pragma unroll
        for (int dw = 0; dw < 2; ++dw) {
          const int qh = ph - dh, qw = pw - dw; // window whose element (dh, dw) is this position
          if (qh >= 0 && qh < Q2 && qw >= 0 && qw < Q2) {
            const int o = d * 16 + qh * 4 + qw;
            if (arg2[o] == dh * 2 + dw) g += dp2[o];
          }
        }
      a2[tid] = g * act_deriv_from_out(a.act2, a2[tid]); // Delta2 in place
    }
    __syncthreads();
    // ---- conv2 backward-data, first half: cols[k][p] = sum_d W2[d][k] Delta2[d][p]; wave = 16 rows k
    {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const int p = nb * 16 + i16, pp = p < P2 ? p : P2 - 1;
        cnn_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const int dd = 4 * ks + kq;
          d = __builtin_amdgcn_mfma_f32_16x16x4f32(w2s[dd * LW2 + wave * 16 + i16], a2[dd * P2 + pp], d, 0, 0, 0);
        }
        if (p < P2) {
#pragma unroll
          for (int r = 0; r < 4; ++r) cols[(wave * 16 + 4 * kq + r) * P2 + p] = d[r];
        }
      }
    }
    __syncthreads();
    // ---- second half: every pool1-output position gathers the columns of the windows that hold it
    for (int i = tid; i < D1 * R1; i += THREADS) {
      const int c = i / R1, q = i - c * R1, ih = q / Q1, iw = q - ih * Q1;
      float g = 0.f;
#pragma unroll
      for (int eh = 0; eh < 2; ++eh)
#pragma unroll
        for (int ew = 0; ew < 2; ++ew) {
          const int kh = (ih & 1) + 2 * eh, kw = (iw & 1) + 2 * ew; // taps of the same parity as the position
          const int oh = (ih - kh) >> 1, ow = (iw - kw) >> 1;
          if (ih >= kh && iw >= kw && oh < O2 && ow < O2) g += cols[(c * 16 + kh * 4 + kw) * P2 + oh * O2 + ow];
        }
      dp1[i] = g;
    }
    __syncthreads();
    // ---- pool1 backward and conv1's activation derivative: Delta1 in place
    for (int i = tid; i < D1 * P1; i += THREADS) {
      const int c = i / P1, p = i - c * P1, oh = p / O1, ow = p - oh * O1;
      float g = 0.f;
#pragma unroll
      for (int dh = 0; dh < 2; ++dh)
#pragma unroll
        for (int dw = 0; dw < 2; ++dw) {
          const int qh = oh - dh, qw = ow - dw;
          if (qh >= 0 && qh < Q1 && qw >= 0 && qw < Q1) {
            const int o = c * R1 + qh * Q1 + qw;
            if (arg1[o] == dh * 2 + dw) g += dp1[o];
          }
        }
      a1[i] = g * act_deriv_from_out(a.act1, a1[i]);
    }
    __syncthreads();
    // the next example's pixels and label are requested here, ahead of the longest phase: every barrier waits for
    // outstanding loads, so a request made at the top of the example would be waited for at once
    {
      const int nx = ex + gridDim.x;
      xnext = a.x[(tid < H0 * H0 && nx < a.B) ? (long)nx * (H0 * H0) + tid : 0];
      ynext = a.y[nx < a.B ? nx : 0];
    }
    // ---- conv1 weight gradient: [16 x 196] x [196 x 64]; wave = (block of 16 taps, quarter of the positions)
    {
      const int nb = wave & 3, kp = wave >> 2;
      const int tap = nb * 16 + i16, tbase = (tap >> 3) * XP + (tap & 7);
      const int ks0 = kp == 0 ? 0 : 1 + 12 * kp; // 13, 12, 12, 12 of the 49 steps: 13 issued, the last one empty for three quarters
      const int last = kp == 0 ? 13 : 12;
      int p = 4 * ks0 + kq, oh = p / O1, ow = p - oh * O1;
      cnn_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 13; ++j) {
        const bool on = j < last;
        const int pc = on ? p : 0;
        const float av = a1[i16 * P1 + pc], bv = xp[(2 * oh) * XP + 2 * ow + tbase];
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(on ? av : 0.f, bv, d, 0, 0, 0);
        p += 4; ow += 4;
        if (ow >= O1) { ow -= O1; ++oh; }
        if (!on) { oh = 0; ow = 0; }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) cols[kp * 1024 + (4 * kq + r) * 64 + tap] = d[r];
    }
    // ---- conv2 weight gradient: [32 x 25] x [25 x 256]; wave = 16 columns k = (c = wave, kh, kw); stays in registers
    float g2[2][4];
    {
      const int kh = i16 >> 2, kw = i16 & 3;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        cnn_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 7; ++ks) {
          const int p = 4 * ks + kq, pp = p < P2 ? p : P2 - 1;
          const float av = a2[(mb * 16 + i16) * P2 + pp];
          d = __builtin_amdgcn_mfma_f32_16x16x4f32(p < P2 ? av : 0.f,
                                                   p1[wave * R1 + (2 * (pp / O2) + kh) * Q1 + 2 * (pp % O2) + kw], d, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) g2[mb][r] = d[r];
      }
    }
    // bias gradients: conv1 (wave d sums its channel), conv2 (thread d < 32)
    float gb1 = 0.f;
    {
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) { const int p = lane + 64 * i; t += p < P1 ? a1[wave * P1 + p] : 0.f; }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, 64);
      gb1 = t; // every lane of wave d holds the bias gradient of channel d
    }
    float gb2 = 0.f;
    if (tid < D2) {
#pragma unroll
      for (int p = 0; p < P2; ++p) gb2 += a2[tid * P2 + p];
    }
    __syncthreads();
    const float g1 = (cols[tid] + cols[1024 + tid]) + (cols[2048 + tid] + cols[3072 + tid]); // (d, tap) = (tid / 64, tid % 64)
    // ---- the example's squared norm: convolution coordinates here, dense layers by the identity (scl[1])
    {
      float q = g1 * g1;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) q = fmaf(g2[mb][r], g2[mb][r], q);
      if (lane == 0) q = fmaf(gb1, gb1, q);
      if (tid < D2) q = fmaf(gb2, gb2, q);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
      if (lane == 0) red[wave] = q;
    }
    __syncthreads();
    float sc;
    {
      float q = scl[1];
#pragma unroll
      for (int w = 0; w < 16; ++w) q += red[w];
      const float n = sqrtf(q);
      sc = a.priv ? fminf(1.f, a.C / n) : 1.f; // n == 0: C/0 = +inf -> 1
      if (tid == 0) {
        if (a.norms) a.norms[ex] = n;
        if (a.s) a.s[ex] = sc;
      }
    }
    // ---- s_i g_i into the partial clipped sum
    acc1 = fmaf(sc, g1, acc1);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc2[mb][r] = fmaf(sc, g2[mb][r], acc2[mb][r]);
    accb = fmaf(sc, gb1, accb);
    accb2 = fmaf(sc, gb2, accb2);
    {
      const float sd = sc * d3[fn];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc3[i] = fmaf(p2[fk * 16 + i], sd, acc3[i]);
      if (tid < HID) accb3 = fmaf(sc, d3[tid], accb3);
      if (tid < HID * NC) acc4 = fmaf(sc * a3[tid / NC], d4[tid % NC], acc4);
      if (tid < NC) accb4 = fmaf(sc, d4[tid], accb4);
    }
    __syncthreads(); // before the next example overwrites the LDS images
  }
  // ---- the workgroup's partial, in the parameter layout
  const int tid = tid0, lane = tid & 63, i16 = lane & 15, kq = lane >> 4, fn = tid & 31, fk = tid >> 5;
  float *pr = a.part + (long)blockIdx.x * a.pstride;
  pr[OFF_W1 + tid] = acc1;
  if (lane == 0) pr[OFF_B1 + wave] = accb;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int r = 0; r < 4; ++r) pr[OFF_W2 + (mb * 16 + 4 * kq + r) * CK2 + wave * 16 + i16] = acc2[mb][r];
  if (tid < D2) pr[OFF_B2 + tid] = accb2;
#pragma unroll
  for (int i = 0; i < 16; ++i) pr[OFF_W3 + (fk * 16 + i) * HID + fn] = acc3[i];
  if (tid < HID) pr[OFF_B3 + tid] = accb3;
  if (tid < HID * NC) pr[OFF_W4 + tid] = acc4;
  if (tid < NC) pr[OFF_B4 + tid] = accb4;
}

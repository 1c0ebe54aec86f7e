// Operand functors for gemm_tile_kernel.  An operand names element (f, k) where f is
// the fixed dimension (row m of A or column n of B) and k the contracted one.
//   scalar staging:  FC fctx(z, f, F), KC kctx(z, k, kend), float load(FC, KC)
//   float4 staging:  groups of four consecutive indices along the contiguous dimension
//                    (first index a multiple of 4): fctx4 / kctx4 and float4 load4
// Elements outside the operand read as 0.  kLanesAlongK tells the tile loader which
// index consecutive lanes should walk so that global loads coalesce; kVec selects the
// float4 loaders.
//
// Every load here is UNCONDITIONAL: an invalid element selects a safe address (the
// operand's base) and the value is discarded afterwards.  A load under a branch makes
// the compiler wait for all outstanding loads where the paths join, which serialises
// the whole tile fetch; with selects the fetch of a tile stays one burst of loads.
// For the same reason float4 vs. scalar staging is a template parameter chosen on the
// host (`can_vec`: 16-byte aligned base, sizes multiples of 4), not a run-time branch.
#pragma once
#include <type_traits>

#include "gemm_tile.h"

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
DEVI float4 f4scale(float4 v, float s) { v.x *= s; v.y *= s; v.z *= s; v.w *= s; return v; }

// ---------------------------------------------------------------- plain matrices

// element (f, k) = ptr[z*zstride + f*ld + k]            (k contiguous)
template <bool VEC>
struct OpRowMajor {
  static constexpr bool kLanesAlongK = true, kVec = VEC;
  const float *ptr;
  long zstride;
  int ld;
  static bool can_vec(const float *p, int ld_, long zs, int K) {
    return aligned16(p) && (ld_ & 3) == 0 && (zs & 3) == 0 && (K & 3) == 0;
  }
  void set(const float *p, int ld_, long zs = 0) { ptr = p; ld = ld_; zstride = zs; }
  struct FC { const float *row; };
  struct KC { int k; };
  typedef KC KC4;
  DEVI FC fctx(int z, int f, int F) const {
    FC c; c.row = f < F ? ptr + z * zstride + (long)f * ld : nullptr; return c;
  }
  DEVI KC kctx(int, int k, int kend) const { KC c; c.k = k < kend ? k : -1; return c; }
  DEVI KC4 kctx4(int, int k, int kend) const { KC c; c.k = k < kend ? k : -1; return c; } // K % 4 == 0
  typedef bool Post;
  typedef bool Post4;
  DEVI Post post(const FC &f, const KC &k) const { return f.row && k.k >= 0; }
  DEVI Post4 post4(const FC &f, const KC4 &k) const { return f.row && k.k >= 0; }
  DEVI float raw(const FC &f, const KC &k, Post ok) const { return *(ok ? f.row + k.k : ptr); }
  DEVI float4 raw4(const FC &f, const KC4 &k, Post4 ok) const {
    return *reinterpret_cast<const float4 *>(ok ? f.row + k.k : ptr);
  }
  DEVI float finish(float v, Post ok) const { return ok ? v : 0.f; }
  DEVI float4 finish4(float4 v, Post4 ok) const { return ok ? v : f4zero(); }
};

// element (f, k) = ptr[z*zstride + k*ld + f] * scale[k / scale_div]    (f contiguous);
// with ones_row, f == F-1 is a row of ones (times the scale): the bias column.
// SCALED operands always carry a valid scale pointer (a vector of ones when nothing is clipped).
template <bool VEC, bool SCALED>
struct OpKMajor {
  static constexpr bool kLanesAlongK = false, kVec = VEC;
  const float *ptr;
  long zstride;
  int ld;
  const float *scale; // indexed by z when by_z, else by k / scale_div
  FastDiv scale_div;
  int ones_row, by_z;
  // real = number of rows that live in memory (F minus the ones row)
  static bool can_vec(const float *p, int ld_, long zs, int real) {
    return aligned16(p) && (ld_ & 3) == 0 && (zs & 3) == 0 && (real & 3) == 0;
  }
  void set(const float *p, int ld_, long zs = 0) {
    ptr = p; ld = ld_; zstride = zs; scale = nullptr; scale_div.init(1); ones_row = 0; by_z = 0;
  }
  struct FC { int f, one; };
  struct FC4 { int f, n, one; }; // n = 4 (whole group in memory) or 0; index of the ones row within the group or -1
  struct KC { const float *row; float s; };
  DEVI FC fctx(int, int f, int F) const {
    FC c; c.one = (ones_row && f == F - 1); c.f = (f < F && !c.one) ? f : -1; return c;
  }
  DEVI FC4 fctx4(int, int f, int F) const {
    FC4 c; c.f = f;
    const int real = F - (ones_row ? 1 : 0);
    c.n = f + 3 < real ? 4 : 0; // real % 4 == 0: a group is whole or empty
    c.one = (ones_row && F - 1 >= f && F - 1 < f + 4) ? F - 1 - f : -1;
    return c;
  }
  DEVI KC kctx(int z, int k, int kend) const {
    KC c;
    const bool ok = k < kend;
    c.row = ok ? ptr + z * zstride + (long)k * ld : nullptr;
    if (SCALED) {
      const float sv = scale[ok ? (by_z ? z : (int)scale_div.div((uint32_t)k)) : 0];
      c.s = ok ? sv : 0.f;
    } else c.s = ok ? 1.f : 0.f;
    return c;
  }
  struct Post { float s; int mode; };  // mode 1: value * s; 2: the ones row (= s); 0: zero
  struct Post4 { float s; int ok, one; };
  DEVI Post post(const FC &f, const KC &k) const {
    Post p; p.s = k.s; // 0 for an invalid k
    p.mode = (k.row && f.f >= 0) ? 1 : (f.one ? 2 : 0);
    return p;
  }
  DEVI Post4 post4(const FC4 &f, const KC &k) const {
    Post4 p; p.s = k.s; p.ok = k.row && f.n == 4; p.one = f.one; return p;
  }
  DEVI float raw(const FC &f, const KC &k, const Post &p) const { return *(p.mode == 1 ? k.row + f.f : ptr); }
  DEVI float4 raw4(const FC4 &f, const KC &k, const Post4 &p) const {
    return *reinterpret_cast<const float4 *>(p.ok ? k.row + f.f : ptr);
  }
  DEVI float finish(float v, const Post &p) const { return p.mode == 1 ? v * p.s : (p.mode == 2 ? p.s : 0.f); }
  DEVI float4 finish4(float4 v, const Post4 &p) const {
    v = p.ok ? f4scale(v, p.s) : f4zero();
    if (p.one == 0) v.x = p.s;
    if (p.one == 1) v.y = p.s;
    if (p.one == 2) v.z = p.s;
    if (p.one == 3) v.w = p.s;
    return v;
  }
};

// ---------------------------------------------------------------- convolution

struct ConvGeom {
  int C, H, W;        // input
  int D, OH, OW;      // output
  int KH, KW, S, PAD;
  int CKK, P;         // C*KH*KW, OH*OW
  FastDiv dP, dOW, dKK, dKW, dHW, dW;
};

// im2col patch element: pixel q = (b, oh, ow), tap t = (c, kh, kw)
//   x[b, c, oh*S - PAD + kh, ow*S - PAD + kw], 0 outside the image;
// tap == CKK (when has_ones) is the constant 1 that carries the bias.
// PIX_FIXED: the pixel is the fixed dimension (forward), else the tap is (weight gradient).
// In batched launches (by_z) pixel q is local to image z.
template <bool PIX_FIXED>
struct OpConvPatch {
  static constexpr bool kLanesAlongK = !PIX_FIXED, kVec = false; // lanes always walk pixels
  const float *x;
  ConvGeom g;
  int has_ones, by_z;
  struct Pix { const float *base; int ih0, iw0; };
  struct Tap { int off, kh, kw; };
  typedef typename std::conditional<PIX_FIXED, Pix, Tap>::type FC;
  typedef typename std::conditional<PIX_FIXED, Tap, Pix>::type KC;
  DEVI Pix pix(int z, int q, int Q) const {
    Pix c;
    if (q < Q) {
      int b = by_z ? z : (int)g.dP.div(q);
      int p = by_z ? q : q - b * g.P;
      int oh = (int)g.dOW.div(p), ow = p - oh * g.OW;
      c.ih0 = oh * g.S - g.PAD; c.iw0 = ow * g.S - g.PAD;
      c.base = x + (long)b * g.C * g.H * g.W + c.ih0 * g.W + c.iw0;
    } else { c.base = nullptr; c.ih0 = c.iw0 = 0; }
    return c;
  }
  DEVI Tap tap(int t, int Tn) const {
    Tap c;
    if (t < Tn && t < g.CKK) {
      int ch = (int)g.dKK.div(t), r = t - ch * g.KH * g.KW;
      c.kh = (int)g.dKW.div(r); c.kw = r - c.kh * g.KW;
      c.off = ch * g.H * g.W + c.kh * g.W + c.kw;
    } else if (t < Tn && has_ones) { c.off = -1; c.kh = c.kw = 0; }
    else { c.off = -2; c.kh = c.kw = 0; }
    return c;
  }
  DEVI FC fctx(int z, int f, int F) const {
    if constexpr (PIX_FIXED) return pix(z, f, F); else return tap(f, F);
  }
  DEVI KC kctx(int z, int k, int kend) const {
    if constexpr (PIX_FIXED) return tap(k, kend); else return pix(z, k, kend);
  }
  typedef int Post; // 1: the pixel; 2: the constant 1 of the bias tap; 0: zero
  DEVI Post pst(const Pix &p, const Tap &t) const {
    const int ih = p.ih0 + t.kh, iw = p.iw0 + t.kw;
    const bool ok = p.base && t.off >= 0 && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
    return ok ? 1 : ((p.base && t.off == -1) ? 2 : 0);
  }
  DEVI Post post(const FC &f, const KC &k) const {
    if constexpr (PIX_FIXED) return pst(f, k); else return pst(k, f);
  }
  DEVI float raw(const FC &f, const KC &k, Post m) const {
    if constexpr (PIX_FIXED) return *(m == 1 ? f.base + k.off : x); else return *(m == 1 ? k.base + f.off : x);
  }
  DEVI float finish(float v, Post m) const { return m == 1 ? v : (m == 2 ? 1.f : 0.f); }
};

// element (d, q) = T[b, d, p] * scale[b]  for pixel q = (b, p); T is [B, D, P].  Lanes walk pixels.
struct OpChanPix {
  static constexpr bool kLanesAlongK = true, kVec = false;
  const float *t;
  const float *scale; // always valid (ones when nothing is clipped)
  int D, P, by_z;
  FastDiv dP;
  struct FC { int off; };
  struct KC { const float *base; float s; };
  DEVI FC fctx(int, int f, int F) const { FC c; c.off = f < F ? f * P : -1; return c; }
  DEVI KC kctx(int z, int k, int kend) const {
    KC c;
    const bool ok = k < kend;
    const int kk = ok ? k : 0;
    const int b = by_z ? z : (int)dP.div(kk);
    const int p = by_z ? kk : kk - b * P;
    c.base = ok ? t + (long)b * D * P + p : nullptr;
    const float sv = scale[ok ? b : 0];
    c.s = ok ? sv : 0.f;
    return c;
  }
  struct Post { float s; int ok; };
  DEVI Post post(const FC &f, const KC &k) const { Post p; p.s = k.s; p.ok = k.base && f.off >= 0; return p; }
  DEVI float raw(const FC &f, const KC &k, const Post &p) const { return *(p.ok ? k.base + f.off : t); }
  DEVI float finish(float v, const Post &p) const { return p.ok ? v * p.s : 0.f; }
};

// backward-data A operand: element (c, k=(d,kh,kw)) = W[d, c, kh, kw]
struct OpConvWeightT {
  static constexpr bool kLanesAlongK = true, kVec = false;
  const float *w;
  ConvGeom g;
  struct FC { int off; };
  struct KC { int off; };
  DEVI FC fctx(int, int f, int F) const { FC c; c.off = f < F ? f * g.KH * g.KW : -1; return c; }
  DEVI KC kctx(int, int k, int kend) const {
    KC c;
    if (k < kend) { int d = (int)g.dKK.div(k), r = k - d * g.KH * g.KW; c.off = d * g.CKK + r; }
    else c.off = -1;
    return c;
  }
  typedef bool Post;
  DEVI Post post(const FC &f, const KC &k) const { return f.off >= 0 && k.off >= 0; }
  DEVI float raw(const FC &f, const KC &k, Post ok) const { return w[ok ? f.off + k.off : 0]; }
  DEVI float finish(float v, Post ok) const { return ok ? v : 0.f; }
};

// backward-data B operand: fixed = input pixel (b, ih, iw), k = (d, kh, kw):
//   Delta[b, d, (ih+PAD-kh)/S, (iw+PAD-kw)/S] where the divisions are exact and in range.
struct OpConvDeltaGather {
  static constexpr bool kLanesAlongK = false, kVec = false;
  const float *delta;
  ConvGeom g;
  FastDiv dS; // stride
  struct FC { const float *base; int ihp, iwp; };
  struct KC { int off, kh, kw; };
  DEVI FC fctx(int, int f, int F) const {
    FC c;
    if (f < F) {
      int b = (int)g.dHW.div(f), r = f - b * g.H * g.W;
      int ih = (int)g.dW.div(r), iw = r - ih * g.W;
      c.base = delta + (long)b * g.D * g.P; c.ihp = ih + g.PAD; c.iwp = iw + g.PAD;
    } else { c.base = nullptr; c.ihp = c.iwp = 0; }
    return c;
  }
  DEVI KC kctx(int, int k, int kend) const {
    KC c;
    if (k < kend) {
      int d = (int)g.dKK.div(k), r = k - d * g.KH * g.KW;
      c.kh = (int)g.dKW.div(r); c.kw = r - c.kh * g.KW; c.off = d * g.P;
    } else { c.off = -1; c.kh = c.kw = 0; }
    return c;
  }
  typedef int Post; // offset of the element inside delta's image block, or -1
  DEVI Post post(const FC &f, const KC &k) const {
    const int th = f.ihp - k.kh, tw = f.iwp - k.kw;
    // S == 1 divides trivially; the multiply-shift division is exact for any S
    const int oh = (int)dS.div((uint32_t)max(th, 0)), ow = (int)dS.div((uint32_t)max(tw, 0));
    const bool ok = f.base && k.off >= 0 && th >= 0 && tw >= 0 && oh * g.S == th && ow * g.S == tw &&
                    oh < g.OH && ow < g.OW;
    return ok ? k.off + oh * g.OW + ow : -1;
  }
  DEVI float raw(const FC &f, const KC &, Post o) const { return *(o >= 0 ? f.base + o : delta); }
  DEVI float finish(float v, Post o) const { return o >= 0 ? v : 0.f; }
};

// ---------------------------------------------------------------- LSTM

// weight-gradient A operand of the LSTM: fixed r in [0, Din+H], k = step (b, t):
//   r < Din        x_{b,t}[r]      = xin[(b,t)*Din + r]   (the gathered embedding rows)
//   r < Din + H    h_{b,t-1}[r-Din] (0 at t = 0), hs is [B, T, H]
//   r == Din + H   1               (bias)
// all times scale[b] (always a valid pointer).  In batched launches (by_z) k = t within example z.
// float4 staging needs Din % 4 == 0 and H % 4 == 0: a group then lies inside x, inside h,
// or is the tail group that starts with the ones row.
template <bool VEC>
struct OpLstmIn {
  static constexpr bool kLanesAlongK = false, kVec = VEC;
  const float *xin;
  const float *hs;
  const float *scale;
  int Din, H, T, by_z;
  FastDiv dT;
  static bool can_vec(const float *x, const float *h, int Din_, int H_) {
    return aligned16(x) && aligned16(h) && (Din_ & 3) == 0 && (H_ & 3) == 0;
  }
  void set(const float *xin_, const float *hs_, const float *scale_, int Din_, int H_, int T_, int by_z_) {
    xin = xin_; hs = hs_; scale = scale_; Din = Din_; H = H_; T = T_; by_z = by_z_; dT.init(T_);
  }
  struct FC { int r; };
  typedef FC FC4;
  struct KC { const float *xrow; const float *hrow; float s; };
  DEVI FC fctx(int, int f, int F) const { FC c; c.r = f < F ? f : -1; return c; }
  DEVI FC4 fctx4(int, int f, int F) const { FC c; c.r = f < F ? f : -1; return c; }
  DEVI KC kctx(int z, int k, int kend) const {
    KC c;
    const bool ok = k < kend;
    const int kk = ok ? k : 0;
    const int b = by_z ? z : (int)dT.div(kk);
    const int t = by_z ? kk : kk - b * T;
    const long bt = (long)b * T + t;
    c.xrow = ok ? xin + bt * Din : nullptr;
    c.hrow = (ok && t > 0) ? hs + (bt - 1) * H : nullptr;
    const float sv = scale[ok ? b : 0];
    c.s = ok ? sv : 0.f;
    return c;
  }
  struct Post { float s; int mode; }; // mode 1: x row; 2: h row; 3: the ones row; 0: zero
  typedef Post Post4;
  DEVI Post post(const FC &f, const KC &k) const {
    Post p; p.s = k.s;
    p.mode = (k.xrow && f.r >= 0 && f.r < Din) ? 1
           : ((k.hrow && f.r >= Din && f.r < Din + H) ? 2 : ((k.xrow && f.r == Din + H) ? 3 : 0));
    return p;
  }
  DEVI Post4 post4(const FC4 &f, const KC &k) const {
    Post p; p.s = k.s;
    p.mode = (k.xrow && f.r >= 0 && f.r + 3 < Din) ? 1
           : ((k.hrow && f.r >= Din && f.r + 3 < Din + H) ? 2 : ((k.xrow && f.r == Din + H) ? 3 : 0));
    return p; // mode 3: the ones row opens the tail group, the other three are past the operand
  }
  DEVI const float *addr(int r, const KC &k, int mode) const {
    return mode == 1 ? k.xrow + r : (mode == 2 ? k.hrow + (r - Din) : xin);
  }
  DEVI float raw(const FC &f, const KC &k, const Post &p) const { return *addr(f.r, k, p.mode); }
  DEVI float4 raw4(const FC4 &f, const KC &k, const Post4 &p) const {
    return *reinterpret_cast<const float4 *>(addr(f.r, k, p.mode));
  }
  DEVI float finish(float v, const Post &p) const {
    return (p.mode == 1 || p.mode == 2) ? v * p.s : (p.mode == 3 ? p.s : 0.f);
  }
  DEVI float4 finish4(float4 v, const Post4 &p) const {
    if (p.mode == 1 || p.mode == 2) return f4scale(v, p.s);
    float4 z = f4zero();
    if (p.mode == 3) z.x = p.s;
    return z;
  }
};

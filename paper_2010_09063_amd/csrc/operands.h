// Operand functors for gemm_tile_kernel.  An operand names element (f, k) where f is
// the fixed dimension (row m of A or column n of B) and k the contracted one.
//   FC fctx(z, f, F)    context of fixed index f (invalid if f >= F)
//   KC kctx(z, k, kend) context of contracted index k (invalid if k >= kend)
//   float load(FC, KC)  the element, 0 where invalid / padded
// kLanesAlongK tells the tile loader which index consecutive lanes should walk so
// that global loads coalesce.
#pragma once
#include "gemm_tile.h"

// ---------------------------------------------------------------- plain matrices
//
// Vector operands (kVec) are staged as float4 items along their contiguous
// dimension: kctx4 / fctx4 give the context of a group of four consecutive
// indices (first index a multiple of 4) and load4 returns the four elements.
// `vec` is set on the host when base pointer, leading dimension and batch
// stride keep every group 16-byte aligned; otherwise load4 falls back to four
// guarded scalar loads.

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// element (f, k) = ptr[z*zstride + f*ld + k]            (k contiguous)
struct OpRowMajor {
  static constexpr bool kLanesAlongK = true, kVec = true;
  const float *ptr;
  long zstride;
  int ld, vec;
  void set(const float *p, int ld_, long zs = 0) {
    ptr = p; ld = ld_; zstride = zs;
    vec = aligned16(p) && (ld_ & 3) == 0 && (zs & 3) == 0;
  }
  struct FC { const float *row; };
  struct KC4 { int k, n; };
  DEVI FC fctx(int z, int f, int F) const {
    FC c; c.row = f < F ? ptr + z * zstride + (long)f * ld : nullptr; return c;
  }
  DEVI KC4 kctx4(int, int k, int kend) const { KC4 c; c.k = k; c.n = min(4, kend - k); return c; }
  DEVI float4 load4(const FC &f, const KC4 &k) const {
    if (!f.row || k.n <= 0) return f4zero();
    if (vec && k.n == 4) return *reinterpret_cast<const float4 *>(f.row + k.k);
    float4 v = f4zero();
    v.x = f.row[k.k];
    if (k.n > 1) v.y = f.row[k.k + 1];
    if (k.n > 2) v.z = f.row[k.k + 2];
    if (k.n > 3) v.w = f.row[k.k + 3];
    return v;
  }
};

// element (f, k) = ptr[z*zstride + k*ld + f] * scale[k / scale_div]    (f contiguous);
// with ones_row, f == F-1 is a row of ones (times the scale): the bias column.
struct OpKMajor {
  static constexpr bool kLanesAlongK = false, kVec = true;
  const float *ptr;
  long zstride;
  int ld, vec;
  const float *scale; // nullable; indexed by z when by_z, else by k / scale_div
  FastDiv scale_div;
  int ones_row, by_z;
  void set(const float *p, int ld_, long zs = 0) {
    ptr = p; ld = ld_; zstride = zs; scale = nullptr; scale_div.init(1); ones_row = 0; by_z = 0;
    vec = aligned16(p) && (ld_ & 3) == 0 && (zs & 3) == 0;
  }
  struct FC4 { int f, n, one; }; // n real rows in the group, index of the ones row within it (or -1)
  struct KC { const float *row; float s; };
  DEVI FC4 fctx4(int, int f, int F) const {
    FC4 c; c.f = f;
    const int real = F - (ones_row ? 1 : 0);
    c.n = max(0, min(4, real - f));
    c.one = (ones_row && F - 1 >= f && F - 1 < f + 4) ? F - 1 - f : -1;
    return c;
  }
  DEVI KC kctx(int z, int k, int kend) const {
    KC c;
    if (k < kend) {
      c.row = ptr + z * zstride + (long)k * ld;
      c.s = scale ? scale[by_z ? z : (int)scale_div.div((uint32_t)k)] : 1.f;
    } else { c.row = nullptr; c.s = 0.f; }
    return c;
  }
  DEVI float4 load4(const FC4 &f, const KC &k) const {
    if (!k.row) return f4zero();
    float4 v;
    if (vec && f.n == 4) v = *reinterpret_cast<const float4 *>(k.row + f.f);
    else {
      v.x = f.n > 0 ? k.row[f.f] : (f.one == 0 ? 1.f : 0.f);
      v.y = f.n > 1 ? k.row[f.f + 1] : (f.one == 1 ? 1.f : 0.f);
      v.z = f.n > 2 ? k.row[f.f + 2] : (f.one == 2 ? 1.f : 0.f);
      v.w = f.n > 3 ? k.row[f.f + 3] : (f.one == 3 ? 1.f : 0.f);
    }
    v.x *= k.s; v.y *= k.s; v.z *= k.s; v.w *= k.s;
    return v;
  }
};

// element (f, k) = table[idx[f]*ld + k]: gathered rows (embedding lookup fused into the operand)
struct OpGatherRows {
  static constexpr bool kLanesAlongK = true, kVec = true;
  const float *table;
  const int *idx;
  int ld, vec;
  void set(const float *t, const int *i, int ld_) { table = t; idx = i; ld = ld_; vec = aligned16(t) && (ld_ & 3) == 0; }
  struct FC { const float *row; };
  struct KC4 { int k, n; };
  DEVI FC fctx(int, int f, int F) const {
    FC c; c.row = f < F ? table + (long)idx[f] * ld : nullptr; return c;
  }
  DEVI KC4 kctx4(int, int k, int kend) const { KC4 c; c.k = k; c.n = min(4, kend - k); return c; }
  DEVI float4 load4(const FC &f, const KC4 &k) const {
    if (!f.row || k.n <= 0) return f4zero();
    if (vec && k.n == 4) return *reinterpret_cast<const float4 *>(f.row + k.k);
    float4 v = f4zero();
    v.x = f.row[k.k];
    if (k.n > 1) v.y = f.row[k.k + 1];
    if (k.n > 2) v.z = f.row[k.k + 2];
    if (k.n > 3) v.w = f.row[k.k + 3];
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
  DEVI float ld(const Pix &p, const Tap &t) const {
    if (!p.base || t.off == -2) return 0.f;
    if (t.off == -1) return 1.f;
    int ih = p.ih0 + t.kh, iw = p.iw0 + t.kw;
    return ((unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W) ? p.base[t.off] : 0.f;
  }
  DEVI float load(const FC &f, const KC &k) const {
    if constexpr (PIX_FIXED) return ld(f, k); else return ld(k, f);
  }
};

// element (d, q) = T[b, d, p] * scale[b]  for pixel q = (b, p); T is [B, D, P].  Lanes walk pixels.
struct OpChanPix {
  static constexpr bool kLanesAlongK = true, kVec = false;
  const float *t;
  const float *scale; // nullable
  int D, P, by_z;
  FastDiv dP;
  struct FC { int off; };
  struct KC { const float *base; float s; };
  DEVI FC fctx(int, int f, int F) const { FC c; c.off = f < F ? f * P : -1; return c; }
  DEVI KC kctx(int z, int k, int kend) const {
    KC c;
    if (k < kend) {
      int b = by_z ? z : (int)dP.div(k);
      int p = by_z ? k : k - b * P;
      c.base = t + (long)b * D * P + p;
      c.s = scale ? scale[b] : 1.f;
    } else { c.base = nullptr; c.s = 0.f; }
    return c;
  }
  DEVI float load(const FC &f, const KC &k) const { return (k.base && f.off >= 0) ? k.base[f.off] * k.s : 0.f; }
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
  DEVI float load(const FC &f, const KC &k) const { return (f.off >= 0 && k.off >= 0) ? w[f.off + k.off] : 0.f; }
};

// backward-data B operand: fixed = input pixel (b, ih, iw), k = (d, kh, kw):
//   Delta[b, d, (ih+PAD-kh)/S, (iw+PAD-kw)/S] where the divisions are exact and in range.
struct OpConvDeltaGather {
  static constexpr bool kLanesAlongK = false, kVec = false;
  const float *delta;
  ConvGeom g;
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
  DEVI float load(const FC &f, const KC &k) const {
    if (!f.base || k.off < 0) return 0.f;
    int th = f.ihp - k.kh, tw = f.iwp - k.kw;
    if (th < 0 || tw < 0) return 0.f;
    int oh = th, ow = tw;
    if (g.S != 1) {
      oh = th / g.S; ow = tw / g.S;
      if (oh * g.S != th || ow * g.S != tw) return 0.f;
    }
    if (oh >= g.OH || ow >= g.OW) return 0.f;
    return f.base[k.off + oh * g.OW + ow];
  }
};

// ---------------------------------------------------------------- LSTM

// weight-gradient A operand of the LSTM: fixed r in [0, Din+H], k = step (b, t):
//   r < Din        x_{b,t}[r]      = table[tok[b,t]*Din + r]   (or xin[(b,t)*Din + r] if no table)
//   r < Din + H    h_{b,t-1}[r-Din] (0 at t = 0), hs is [B, T, H]
//   r == Din + H   1               (bias)
// all times scale[b].  In batched launches (by_z) k = t within example z.
struct OpLstmIn {
  static constexpr bool kLanesAlongK = false, kVec = true;
  const float *table; const int *tok;
  const float *hs;
  const float *scale;
  int Din, H, T, by_z, vec;
  FastDiv dT;
  void set(const float *table_, const int *tok_, const float *hs_, const float *scale_, int Din_, int H_, int T_,
           int by_z_) {
    table = table_; tok = tok_; hs = hs_; scale = scale_; Din = Din_; H = H_; T = T_; by_z = by_z_; dT.init(T_);
    vec = aligned16(table_) && aligned16(hs_) && (Din_ & 3) == 0 && (H_ & 3) == 0;
  }
  struct FC4 { int r, n; };
  struct KC { const float *xrow; const float *hrow; float s; int valid; };
  DEVI FC4 fctx4(int, int f, int F) const { FC4 c; c.r = f; c.n = max(0, min(4, F - f)); return c; }
  DEVI KC kctx(int z, int k, int kend) const {
    KC c;
    if (k < kend) {
      int b = by_z ? z : (int)dT.div(k);
      int t = by_z ? k : k - b * T;
      long bt = (long)b * T + t;
      c.xrow = table + (long)tok[bt] * Din;
      c.hrow = t > 0 ? hs + (bt - 1) * H : nullptr;
      c.s = scale ? scale[b] : 1.f;
      c.valid = 1;
    } else { c.xrow = c.hrow = nullptr; c.s = 0.f; c.valid = 0; }
    return c;
  }
  DEVI float one(int r, const KC &k) const {
    if (r < Din) return k.xrow[r];
    if (r < Din + H) return k.hrow ? k.hrow[r - Din] : 0.f;
    return 1.f;
  }
  DEVI float4 load4(const FC4 &f, const KC &k) const {
    if (!k.valid || f.n <= 0) return f4zero();
    float4 v;
    if (vec && f.r + 3 < Din) v = *reinterpret_cast<const float4 *>(k.xrow + f.r);
    else if (vec && f.r >= Din && f.r + 3 < Din + H)
      v = k.hrow ? *reinterpret_cast<const float4 *>(k.hrow + (f.r - Din)) : f4zero();
    else {
      v.x = one(f.r, k);
      v.y = f.n > 1 ? one(f.r + 1, k) : 0.f;
      v.z = f.n > 2 ? one(f.r + 2, k) : 0.f;
      v.w = f.n > 3 ? one(f.r + 3, k) : 0.f;
    }
    v.x *= k.s; v.y *= k.s; v.z *= k.s; v.w *= k.s;
    return v;
  }
};

/*
 * CPU oracle for one private gradient step of DPSGD.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * build, link or call this file.  It shares no code with the GPU library: the
 * structs below are this file's own.
 *
 * What it computes (paper, Section 1, the enumerated DPSGD procedure, items 2-3):
 *   for every example i of the minibatch, on its own:
 *       g_i   = gradient of the example's own loss w.r.t. all parameters   (2a)
 *       if ||g_i||_2 > C rescale g_i so that its norm is C                 (2b)
 *   sum the clipped gradients and add Gaussian noise N(0, sigma^2 C^2 I)   (3)
 * Examples are processed one at a time with explicit backprop, the way the
 * for-loop library of Section 2.1 ("PyVacy") does; per-layer gradients follow
 * the transposed-Jacobian formula of Section 2.1 ("BackPACK"): the gradient of a
 * layer's parameters is that layer's parameter-Jacobian transposed, applied to
 * the example's backpropagated signal.
 *
 * All arithmetic is fp64; the result is rounded to fp32 once at the end.
 * OpenMP is used over examples only (each thread owns whole examples); partial
 * sums are combined in thread order, so a run is deterministic for a fixed
 * thread count.
 *
 * Readings taken where the paper is silent (each is listed in the design notes):
 *   - "aggregate" = sum, not mean; noise std = sigma*C on every coordinate;
 *   - clip factor min(1, C/||g||), 1 when ||g|| = 0; one global norm over all tensors;
 *   - softmax cross-entropy on logits for one example, no 1/B;
 *   - conv = cross-correlation with zero padding, out = floor((H+2p-K)/s)+1;
 *   - ReLU'(0) = 0; max-pool sends the gradient to the first maximum in
 *     row-major window order;
 *   - LSTM: i,f,o = sigmoid, g = tanh, c_t = f*c_{t-1} + i*g, h_t = o*tanh(c_t),
 *     h_0 = c_0 = 0, one bias of size 4H, gate order i,f,g,o; the layer's output is h_T
 *     or, for the sequence variant of Appendix B, every h_t;
 *   - average pools (Appendix B) take the plain mean of a window, no padding; the global one
 *     is the window that covers the whole plane;
 *   - noise: Philox4x32-10 (Salmon et al., SC'11), key = seed (lo, hi),
 *     counter = (block lo, block hi, 0, 0); four normals per block from two
 *     Box-Muller pairs; uniform u = ((r >> 9) + 1/2) * 2^-23.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OR_DENSE = 0, OR_CONV2D = 1, OR_MAXPOOL2D = 2, OR_EMBEDDING = 3, OR_LSTM_LAST = 4, OR_SEQ_MEAN = 5,
       OR_LSTM_SEQ = 6, OR_AVGPOOL2D = 7 };
enum { OR_ACT_NONE = 0, OR_ACT_RELU = 1, OR_ACT_TANH = 2 };

typedef struct {
  int kind, act;
  int d_in, d_out;                      /* dense; lstm: d_in = input width, d_out = hidden */
  int c_in, c_out, kh, kw, stride, pad; /* conv; pool uses kh = kw = window, stride      */
  int vocab, dim;                       /* embedding                                      */
} or_layer;

typedef struct {
  int n_layers;
  const or_layer *layers;
  int in_c, in_h, in_w; /* image input (a feature vector is in_c x 1 x 1) */
  int seq_len;          /* > 0: the input is seq_len int32 token ids      */
  int n_classes;
} or_model;

/* ---------------------------------------------------------------- shapes */

typedef struct { int c, h, w; } shp; /* sequences: c = T, h = D, w = 1; vectors: c = D, h = w = 1 */

static int shp_size(shp s) { return s.c * s.h * s.w; }

static shp out_shape(const or_layer *L, shp in, int seq_len) {
  shp o = in;
  switch (L->kind) {
  case OR_DENSE: o.c = L->d_out; o.h = o.w = 1; break;
  case OR_CONV2D:
    o.c = L->c_out;
    o.h = (in.h + 2 * L->pad - L->kh) / L->stride + 1;
    o.w = (in.w + 2 * L->pad - L->kw) / L->stride + 1;
    break;
  case OR_MAXPOOL2D:
  case OR_AVGPOOL2D:
    o.h = (in.h - L->kh) / L->stride + 1;
    o.w = (in.w - L->kw) / L->stride + 1;
    break;
  case OR_EMBEDDING: o.c = seq_len; o.h = L->dim; o.w = 1; break;
  case OR_LSTM_LAST: o.c = L->d_out; o.h = o.w = 1; break;
  case OR_SEQ_MEAN: o.c = in.h; o.h = o.w = 1; break; /* [T, D] -> [D] */
  case OR_LSTM_SEQ: o.c = in.c; o.h = L->d_out; o.w = 1; break; /* [T, D] -> [T, H] */
  }
  return o;
}

static long layer_params(const or_layer *L) {
  switch (L->kind) {
  case OR_DENSE: return (long)L->d_in * L->d_out + L->d_out;
  case OR_CONV2D: return (long)L->c_out * L->c_in * L->kh * L->kw + L->c_out;
  case OR_EMBEDDING: return (long)L->vocab * L->dim;
  case OR_LSTM_LAST:
  case OR_LSTM_SEQ: return (long)L->d_in * 4 * L->d_out + (long)L->d_out * 4 * L->d_out + 4 * L->d_out;
  default: return 0;
  }
}

long oracle_num_params(const or_model *m) {
  long p = 0;
  for (int l = 0; l < m->n_layers; ++l) p += layer_params(&m->layers[l]);
  return p;
}

/* ---------------------------------------------------------------- helpers */

static double act_f(int act, double z) {
  if (act == OR_ACT_RELU) return z > 0 ? z : 0;
  if (act == OR_ACT_TANH) return tanh(z);
  return z;
}
static double act_df(int act, double z) {
  if (act == OR_ACT_RELU) return z > 0 ? 1.0 : 0.0;
  if (act == OR_ACT_TANH) { double t = tanh(z); return 1.0 - t * t; }
  return 1.0;
}
static double sigm(double v) { return 1.0 / (1.0 + exp(-v)); }

/* Per-example scratch: for every layer its pre-activation z and output a; the
 * pool's argmax; the LSTM's per-step gates and states. */
typedef struct {
  int n_layers;
  shp *shape;     /* output shape of each layer                   */
  double **z;     /* pre-activation (dense, conv)                 */
  double **a;     /* layer output                                 */
  int **arg;      /* pool: flat input index of each output's max  */
  double **lstm;  /* lstm: [T][6][H] = i,f,g,o,c,h                */
  double *in0;    /* the example's input as doubles (images)      */
  double *d_a, *d_b; /* two gradient buffers of the largest size  */
  long max_act;
  long ties;      /* number of pool windows whose maximum is not unique */
  double margin;  /* smallest distance of the current example from a decision an fp32 forward pass may take the other
                   * way: (maximum - runner-up) over its max-pool windows, |z| over its non-zero ReLU pre-activations */
} scratch;

static scratch *scratch_new(const or_model *m) {
  scratch *s = (scratch *)calloc(1, sizeof(scratch));
  int L = m->n_layers;
  s->n_layers = L;
  s->shape = (shp *)calloc(L, sizeof(shp));
  s->z = (double **)calloc(L, sizeof(double *));
  s->a = (double **)calloc(L, sizeof(double *));
  s->arg = (int **)calloc(L, sizeof(int *));
  s->lstm = (double **)calloc(L, sizeof(double *));
  shp cur = {m->in_c, m->in_h, m->in_w};
  long mx = m->seq_len > 0 ? m->seq_len : shp_size(cur);
  if (m->seq_len == 0) s->in0 = (double *)calloc(shp_size(cur), sizeof(double));
  for (int l = 0; l < L; ++l) {
    const or_layer *ly = &m->layers[l];
    shp o = out_shape(ly, cur, m->seq_len);
    s->shape[l] = o;
    long n = shp_size(o);
    if (n > mx) mx = n;
    s->a[l] = (double *)calloc(n, sizeof(double));
    if (ly->kind == OR_DENSE || ly->kind == OR_CONV2D) s->z[l] = (double *)calloc(n, sizeof(double));
    if (ly->kind == OR_MAXPOOL2D) s->arg[l] = (int *)calloc(n, sizeof(int));
    if (ly->kind == OR_LSTM_LAST || ly->kind == OR_LSTM_SEQ) s->lstm[l] = (double *)calloc((long)cur.c * 6 * ly->d_out, sizeof(double));
    cur = o;
  }
  s->max_act = mx;
  s->d_a = (double *)calloc(mx, sizeof(double));
  s->d_b = (double *)calloc(mx, sizeof(double));
  return s;
}

static void scratch_free(scratch *s) {
  for (int l = 0; l < s->n_layers; ++l) { free(s->z[l]); free(s->a[l]); free(s->arg[l]); free(s->lstm[l]); }
  free(s->shape); free(s->z); free(s->a); free(s->arg); free(s->lstm); free(s->in0); free(s->d_a); free(s->d_b);
  free(s);
}

/* ---------------------------------------------------------------- forward */

/* Returns the example's loss: logsumexp(logits) - logits[y]. */
static double forward(const or_model *m, const double *theta, const void *x, int y, scratch *s) {
  const double *in = NULL;
  const int32_t *tok = NULL;
  shp cur = {m->in_c, m->in_h, m->in_w};
  if (m->seq_len > 0) tok = (const int32_t *)x;
  else {
    const float *xf = (const float *)x;
    for (int j = 0; j < shp_size(cur); ++j) s->in0[j] = (double)xf[j];
    in = s->in0;
  }
  const double *th = theta;
  s->margin = INFINITY;
  for (int l = 0; l < m->n_layers; ++l) {
    const or_layer *L = &m->layers[l];
    shp o = s->shape[l];
    double *a = s->a[l];
    switch (L->kind) {
    case OR_DENSE: {
      const double *W = th, *b = th + (long)L->d_in * L->d_out;
      for (int j = 0; j < L->d_out; ++j) {
        double acc = b[j];
        for (int k = 0; k < L->d_in; ++k) acc += in[k] * W[(long)k * L->d_out + j];
        s->z[l][j] = acc;
        a[j] = act_f(L->act, acc);
        if (L->act == OR_ACT_RELU && acc != 0 && fabs(acc) < s->margin) s->margin = fabs(acc);
      }
    } break;
    case OR_CONV2D: {
      const double *W = th, *b = th + (long)L->c_out * L->c_in * L->kh * L->kw;
      for (int d = 0; d < L->c_out; ++d)
        for (int oh = 0; oh < o.h; ++oh)
          for (int ow = 0; ow < o.w; ++ow) {
            double acc = b[d];
            for (int c = 0; c < L->c_in; ++c)
              for (int kh = 0; kh < L->kh; ++kh)
                for (int kw = 0; kw < L->kw; ++kw) {
                  int ih = oh * L->stride - L->pad + kh, iw = ow * L->stride - L->pad + kw;
                  if (ih < 0 || ih >= cur.h || iw < 0 || iw >= cur.w) continue;
                  acc += in[((long)c * cur.h + ih) * cur.w + iw] *
                         W[(((long)d * L->c_in + c) * L->kh + kh) * L->kw + kw];
                }
            long oi = ((long)d * o.h + oh) * o.w + ow;
            s->z[l][oi] = acc;
            a[oi] = act_f(L->act, acc);
            if (L->act == OR_ACT_RELU && acc != 0 && fabs(acc) < s->margin) s->margin = fabs(acc);
          }
    } break;
    case OR_MAXPOOL2D: {
      for (int c = 0; c < o.c; ++c)
        for (int oh = 0; oh < o.h; ++oh)
          for (int ow = 0; ow < o.w; ++ow) {
            int best = -1, nbest = 0;
            double bv = 0, second = -INFINITY;
            for (int kh = 0; kh < L->kh; ++kh)
              for (int kw = 0; kw < L->kw; ++kw) {
                int idx = (c * cur.h + oh * L->stride + kh) * cur.w + ow * L->stride + kw;
                double v = in[idx];
                if (best < 0 || v > bv) { if (best >= 0) second = bv; best = idx; bv = v; nbest = 1; }
                else { if (v == bv) ++nbest; if (v > second) second = v; }
              }
            long oi = ((long)c * o.h + oh) * o.w + ow;
            a[oi] = bv;
            s->arg[l][oi] = best;
            if (nbest > 1) s->ties++;
            if (bv > second && bv - second < s->margin) s->margin = bv - second; /* exact ties follow the first-maximum rule */
          }
    } break;
    case OR_EMBEDDING: {
      for (int t = 0; t < m->seq_len; ++t)
        for (int e = 0; e < L->dim; ++e) a[(long)t * L->dim + e] = th[(long)tok[t] * L->dim + e];
    } break;
    case OR_SEQ_MEAN: { /* the embedding network of Appendix B: mean of the T step vectors */
      int T = cur.c, D = cur.h;
      for (int e = 0; e < D; ++e) {
        double acc = 0;
        for (int t = 0; t < T; ++t) acc += in[(long)t * D + e];
        a[e] = acc / T;
      }
    } break;
    case OR_AVGPOOL2D: { /* Appendix B, CIFAR10 network: the mean of every window */
      for (int c = 0; c < o.c; ++c)
        for (int oh = 0; oh < o.h; ++oh)
          for (int ow = 0; ow < o.w; ++ow) {
            double acc = 0;
            for (int kh = 0; kh < L->kh; ++kh)
              for (int kw = 0; kw < L->kw; ++kw)
                acc += in[(c * cur.h + oh * L->stride + kh) * cur.w + ow * L->stride + kw];
            a[((long)c * o.h + oh) * o.w + ow] = acc / (L->kh * L->kw);
          }
    } break;
    case OR_LSTM_LAST:
    case OR_LSTM_SEQ: {
      int T = cur.c, D = L->d_in, H = L->d_out;
      const double *Wih = th, *Whh = th + (long)D * 4 * H, *b = Whh + (long)H * 4 * H;
      double *st = s->lstm[l];
      for (int t = 0; t < T; ++t) {
        double *gi = st + ((long)t * 6 + 0) * H, *gf = gi + H, *gg = gf + H, *go = gg + H, *c = go + H, *h = c + H;
        const double *hp = t ? st + ((long)(t - 1) * 6 + 5) * H : NULL;
        const double *cp = t ? st + ((long)(t - 1) * 6 + 4) * H : NULL;
        for (int j = 0; j < 4 * H; ++j) {
          double acc = b[j];
          for (int k = 0; k < D; ++k) acc += in[(long)t * D + k] * Wih[(long)k * 4 * H + j];
          if (hp) for (int k = 0; k < H; ++k) acc += hp[k] * Whh[(long)k * 4 * H + j];
          int q = j / H, r = j % H;
          if (q == 0) gi[r] = sigm(acc);
          else if (q == 1) gf[r] = sigm(acc);
          else if (q == 2) gg[r] = tanh(acc);
          else go[r] = sigm(acc);
        }
        for (int r = 0; r < H; ++r) {
          c[r] = gf[r] * (cp ? cp[r] : 0.0) + gi[r] * gg[r];
          h[r] = go[r] * tanh(c[r]);
        }
      }
      if (L->kind == OR_LSTM_SEQ) { /* Appendix B, LSTM network: the output is the whole sequence of h_t */
        for (int t = 0; t < T; ++t)
          for (int r = 0; r < H; ++r) a[(long)t * H + r] = st[((long)t * 6 + 5) * H + r];
      } else {
        for (int r = 0; r < H; ++r) a[r] = st[((long)(T - 1) * 6 + 5) * H + r];
      }
    } break;
    }
    th += layer_params(L);
    in = a;
    cur = o;
  }
  /* softmax cross-entropy of one example */
  int K = m->n_classes;
  double mx = in[0];
  for (int k = 1; k < K; ++k) if (in[k] > mx) mx = in[k];
  double se = 0;
  for (int k = 0; k < K; ++k) se += exp(in[k] - mx);
  return mx + log(se) - in[y];
}

/* ---------------------------------------------------------------- backward */

/* Writes the example's full flattened gradient into g[0:P] (overwritten). */
static void backward(const or_model *m, const double *theta, const void *x, int y, scratch *s, double *g) {
  long P = oracle_num_params(m);
  memset(g, 0, sizeof(double) * P);
  int Lc = m->n_layers;
  const int32_t *tok = m->seq_len > 0 ? (const int32_t *)x : NULL;
  /* d(loss)/d(logits) = softmax - onehot */
  double *dout = s->d_a, *din = s->d_b;
  {
    const double *zL = s->a[Lc - 1];
    int K = m->n_classes;
    double mx = zL[0];
    for (int k = 1; k < K; ++k) if (zL[k] > mx) mx = zL[k];
    double se = 0;
    for (int k = 0; k < K; ++k) se += exp(zL[k] - mx);
    for (int k = 0; k < K; ++k) dout[k] = exp(zL[k] - mx) / se - (k == y ? 1.0 : 0.0);
  }
  long off = P;
  for (int l = Lc - 1; l >= 0; --l) {
    const or_layer *L = &m->layers[l];
    off -= layer_params(L);
    const double *th = theta + off;
    double *gl = g + off;
    shp o = s->shape[l];
    shp ishp;
    const double *in;
    if (l > 0) { ishp = s->shape[l - 1]; in = s->a[l - 1]; }
    else { ishp.c = m->in_c; ishp.h = m->in_h; ishp.w = m->in_w; in = s->in0; }
    long n_in = (l > 0) ? shp_size(ishp) : (m->seq_len > 0 ? m->seq_len : shp_size(ishp));
    switch (L->kind) {
    case OR_DENSE: {
      const double *W = th;
      double *gW = gl, *gb = gl + (long)L->d_in * L->d_out;
      for (int k = 0; k < L->d_in; ++k) din[k] = 0;
      for (int j = 0; j < L->d_out; ++j) {
        double dz = dout[j] * act_df(L->act, s->z[l][j]);
        gb[j] = dz;
        for (int k = 0; k < L->d_in; ++k) {
          gW[(long)k * L->d_out + j] = in[k] * dz; /* outer product a (x) delta */
          din[k] += W[(long)k * L->d_out + j] * dz;
        }
      }
    } break;
    case OR_CONV2D: {
      const double *W = th;
      double *gW = gl, *gb = gl + (long)L->c_out * L->c_in * L->kh * L->kw;
      for (long j = 0; j < n_in; ++j) din[j] = 0;
      for (int d = 0; d < L->c_out; ++d)
        for (int oh = 0; oh < o.h; ++oh)
          for (int ow = 0; ow < o.w; ++ow) {
            long oi = ((long)d * o.h + oh) * o.w + ow;
            double dz = dout[oi] * act_df(L->act, s->z[l][oi]);
            gb[d] += dz;
            for (int c = 0; c < L->c_in; ++c)
              for (int kh = 0; kh < L->kh; ++kh)
                for (int kw = 0; kw < L->kw; ++kw) {
                  int ih = oh * L->stride - L->pad + kh, iw = ow * L->stride - L->pad + kw;
                  if (ih < 0 || ih >= ishp.h || iw < 0 || iw >= ishp.w) continue;
                  long wi = (((long)d * L->c_in + c) * L->kh + kh) * L->kw + kw;
                  long xi = ((long)c * ishp.h + ih) * ishp.w + iw;
                  gW[wi] += in[xi] * dz;
                  din[xi] += W[wi] * dz;
                }
          }
    } break;
    case OR_MAXPOOL2D: {
      for (long j = 0; j < n_in; ++j) din[j] = 0;
      for (long oi = 0; oi < shp_size(o); ++oi) din[s->arg[l][oi]] += dout[oi];
    } break;
    case OR_EMBEDDING: {
      for (int t = 0; t < m->seq_len; ++t)
        for (int e = 0; e < L->dim; ++e) gl[(long)tok[t] * L->dim + e] += dout[(long)t * L->dim + e];
    } break;
    case OR_SEQ_MEAN: {
      int T = ishp.c, D = ishp.h;
      for (int t = 0; t < T; ++t)
        for (int e = 0; e < D; ++e) din[(long)t * D + e] = dout[e] / T;
    } break;
    case OR_AVGPOOL2D: {
      for (long j = 0; j < n_in; ++j) din[j] = 0;
      for (int c = 0; c < o.c; ++c)
        for (int oh = 0; oh < o.h; ++oh)
          for (int ow = 0; ow < o.w; ++ow) {
            double share = dout[((long)c * o.h + oh) * o.w + ow] / (L->kh * L->kw);
            for (int kh = 0; kh < L->kh; ++kh)
              for (int kw = 0; kw < L->kw; ++kw)
                din[(c * ishp.h + oh * L->stride + kh) * ishp.w + ow * L->stride + kw] += share;
          }
    } break;
    case OR_LSTM_LAST:
    case OR_LSTM_SEQ: {
      int T = ishp.c, D = L->d_in, H = L->d_out;
      const int seq = L->kind == OR_LSTM_SEQ;
      const double *Wih = th, *Whh = th + (long)D * 4 * H;
      double *gWih = gl, *gWhh = gl + (long)D * 4 * H, *gb = gWhh + (long)H * 4 * H;
      const double *st = s->lstm[l];
      double *dh = (double *)calloc(H, sizeof(double)), *dc = (double *)calloc(H, sizeof(double));
      double *dg = (double *)calloc(4 * H, sizeof(double)), *dhp = (double *)calloc(H, sizeof(double));
      /* dh = dL/dh_t: what the later steps send back through W_hh, plus the loss's direct share of h_t
         (every step for the sequence output, the last step only otherwise) */
      if (!seq) for (int r = 0; r < H; ++r) dh[r] = dout[r];
      for (int t = T - 1; t >= 0; --t) {
        if (seq) for (int r = 0; r < H; ++r) dh[r] += dout[(long)t * H + r];
        const double *gi = st + ((long)t * 6 + 0) * H, *gf = gi + H, *gg = gf + H, *go = gg + H, *c = go + H;
        const double *hp = t ? st + ((long)(t - 1) * 6 + 5) * H : NULL;
        const double *cp = t ? st + ((long)(t - 1) * 6 + 4) * H : NULL;
        for (int r = 0; r < H; ++r) {
          double tc = tanh(c[r]);
          double dct = dc[r] + dh[r] * go[r] * (1.0 - tc * tc);
          dg[3 * H + r] = dh[r] * tc * go[r] * (1.0 - go[r]);                 /* o pre-activation */
          dg[0 * H + r] = dct * gg[r] * gi[r] * (1.0 - gi[r]);                /* i */
          dg[1 * H + r] = dct * (cp ? cp[r] : 0.0) * gf[r] * (1.0 - gf[r]);   /* f */
          dg[2 * H + r] = dct * gi[r] * (1.0 - gg[r] * gg[r]);                /* g */
          dc[r] = dct * gf[r];
        }
        for (int k = 0; k < H; ++k) dhp[k] = 0;
        for (int k = 0; k < D; ++k) din[(long)t * D + k] = 0;
        for (int j = 0; j < 4 * H; ++j) {
          gb[j] += dg[j];
          for (int k = 0; k < D; ++k) {
            gWih[(long)k * 4 * H + j] += in[(long)t * D + k] * dg[j];
            din[(long)t * D + k] += Wih[(long)k * 4 * H + j] * dg[j];
          }
          for (int k = 0; k < H; ++k) {
            if (hp) gWhh[(long)k * 4 * H + j] += hp[k] * dg[j];
            dhp[k] += Whh[(long)k * 4 * H + j] * dg[j];
          }
        }
        for (int k = 0; k < H; ++k) dh[k] = dhp[k];
      }
      free(dh); free(dc); free(dg); free(dhp);
    } break;
    }
    double *tmp = dout; dout = din; din = tmp;
  }
}

/* ---------------------------------------------------------------- exported: per-example pieces */

/* Loss of one example with fp64 parameters (used for finite differences). */
double oracle_example_loss(const or_model *m, const double *theta, const void *x, int y) {
  scratch *s = scratch_new(m);
  double l = forward(m, theta, x, y, s);
  scratch_free(s);
  return l;
}

/* Gradient of one example's loss; g has oracle_num_params doubles.  Returns the
 * loss; *ties (may be NULL) receives the number of tied pool windows. */
double oracle_example_grad(const or_model *m, const double *theta, const void *x, int y, double *g, long *ties) {
  scratch *s = scratch_new(m);
  double l = forward(m, theta, x, y, s);
  backward(m, theta, x, y, s, g);
  if (ties) *ties = s->ties;
  scratch_free(s);
  return l;
}

/* ---------------------------------------------------------------- exported: max-pool routing of near-tied windows
 *
 * A max-pool sends a window's gradient to its maximum (the first one in row-major order).  An fp32
 * implementation decides that maximum on fp32 activations; where the two largest values of a window differ
 * by less than the rounding error of the forward pass, either element is a valid choice of subgradient.
 * The two functions below let a test enumerate every such choice on the CPU and check an fp32 result
 * against the set of valid ones: the first lists, for one example, the window elements within tau of their
 * window's maximum; the second computes the example's gradient with chosen windows routed to a listed
 * element.  Forward values are never altered (the pool's output stays the fp64 maximum). */

/* Flat input index of window element (kh, kw) of pool output oi. */
static int pool_in_index(const or_layer *L, shp in, shp o, long oi, int kh, int kw) {
  int ow = (int)(oi % o.w), oh = (int)((oi / o.w) % o.h), c = (int)(oi / ((long)o.w * o.h));
  return (c * in.h + oh * L->stride + kh) * in.w + ow * L->stride + kw;
}

/* Lists up to cap entries (layer, out_idx, in_idx, gap): element in_idx of the window of output out_idx of
 * max-pool layer `layer` lies 0 < gap <= tau below that window's maximum.  Exact ties are not listed: they
 * follow the first-maximum rule on every implementation.
 * The ReLU has the same kind of decision: its subgradient is 1 for z > 0 and 0 otherwise, and an fp32 forward
 * pass may put a pre-activation with |z| below its rounding error on the other side of zero (the forward value
 * changes by nothing that matters, the backward factor by 1).  Such units of dense / convolution layers are
 * listed as (layer, unit index, -1, |z|) for 0 < |z| <= tau; z = 0 exactly is on the 0 side everywhere.
 * Returns the number of entries (which may exceed cap; only the first cap are written). */
long oracle_pool_near_ties(const or_model *m, const double *theta, const void *x, int y, double tau, long cap,
                           int *layer, int *out_idx, int *in_idx, double *gap) {
  scratch *s = scratch_new(m);
  forward(m, theta, x, y, s);
  long n = 0;
  for (int l = 0; l < m->n_layers; ++l) {
    const or_layer *L = &m->layers[l];
    if ((L->kind == OR_DENSE || L->kind == OR_CONV2D) && L->act == OR_ACT_RELU) {
      for (long oi = 0; oi < shp_size(s->shape[l]); ++oi) {
        double z = fabs(s->z[l][oi]);
        if (z > 0 && z <= tau) {
          if (n < cap) { layer[n] = l; out_idx[n] = (int)oi; in_idx[n] = -1; gap[n] = z; }
          ++n;
        }
      }
      continue;
    }
    if (L->kind != OR_MAXPOOL2D) continue;
    shp o = s->shape[l], in;
    const double *av;
    if (l > 0) { in = s->shape[l - 1]; av = s->a[l - 1]; }
    else { in.c = m->in_c; in.h = m->in_h; in.w = m->in_w; av = s->in0; }
    for (long oi = 0; oi < shp_size(o); ++oi) {
      double bv = s->a[l][oi];
      for (int kh = 0; kh < L->kh; ++kh)
        for (int kw = 0; kw < L->kw; ++kw) {
          int idx = pool_in_index(L, in, o, oi, kh, kw);
          double d = bv - av[idx];
          if (d > 0 && d <= tau) {
            if (n < cap) { layer[n] = l; out_idx[n] = (int)oi; in_idx[n] = idx; gap[n] = d; }
            ++n;
          }
        }
    }
  }
  scratch_free(s);
  return n;
}

/* Gradient of one example's loss with n_route decisions taken by hand: the gradient of output out_idx[r] of
 * max-pool layer layer[r] goes to input element in_idx[r], which must lie inside that window; or, with
 * in_idx[r] = -1, unit out_idx[r] of the ReLU dense / convolution layer layer[r] takes the subgradient of the
 * other side of zero.  Returns the loss, or NaN if a route names a layer of another kind, an output out of range
 * or an element outside the window. */
double oracle_example_grad_routed(const or_model *m, const double *theta, const void *x, int y, long n_route,
                                  const int *layer, const int *out_idx, const int *in_idx, double *g) {
  scratch *s = scratch_new(m);
  double loss = forward(m, theta, x, y, s);
  for (long r = 0; r < n_route; ++r) {
    int l = layer[r], ok = 0;
    if (in_idx[r] == -1) {
      if (l >= 0 && l < m->n_layers && (m->layers[l].kind == OR_DENSE || m->layers[l].kind == OR_CONV2D) &&
          m->layers[l].act == OR_ACT_RELU && out_idx[r] >= 0 && out_idx[r] < shp_size(s->shape[l])) {
        /* the backward pass reads the pre-activation only through the activation's derivative */
        double z = s->z[l][out_idx[r]];
        s->z[l][out_idx[r]] = z > 0 ? -1.0 : 1.0;
        continue;
      }
      scratch_free(s);
      return NAN;
    }
    if (l >= 0 && l < m->n_layers && m->layers[l].kind == OR_MAXPOOL2D && out_idx[r] >= 0 &&
        out_idx[r] < shp_size(s->shape[l])) {
      const or_layer *L = &m->layers[l];
      shp o = s->shape[l], in;
      if (l > 0) in = s->shape[l - 1];
      else { in.c = m->in_c; in.h = m->in_h; in.w = m->in_w; }
      for (int kh = 0; kh < L->kh; ++kh)
        for (int kw = 0; kw < L->kw; ++kw)
          if (pool_in_index(L, in, o, out_idx[r], kh, kw) == in_idx[r]) ok = 1;
    }
    if (!ok) { scratch_free(s); return NAN; }
    s->arg[l][out_idx[r]] = in_idx[r];
  }
  backward(m, theta, x, y, s, g);
  scratch_free(s);
  return loss;
}

/* ---------------------------------------------------------------- noise */

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* z[0:n] standard normals of the stream keyed by seed (coordinate j uses block j/4). */
void oracle_noise(uint64_t seed, long n, double *z) {
  const double two_pi = 6.283185307179586476925286766559;
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  for (long blk = 0; blk * 4 < n; ++blk) {
    uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), 0, 0}, r[4];
    oracle_philox4x32_10(ctr, key, r);
    double u[4], zz[4];
    for (int q = 0; q < 4; ++q) u[q] = ((double)(r[q] >> 9) + 0.5) * (1.0 / 8388608.0);
    double r0 = sqrt(-2.0 * log(u[0])), r1 = sqrt(-2.0 * log(u[2]));
    zz[0] = r0 * cos(two_pi * u[1]); zz[1] = r0 * sin(two_pi * u[1]);
    zz[2] = r1 * cos(two_pi * u[3]); zz[3] = r1 * sin(two_pi * u[3]);
    for (int q = 0; q < 4 && blk * 4 + q < n; ++q) z[blk * 4 + q] = zz[q];
  }
}

/* ---------------------------------------------------------------- the step */

/* params fp32[P]; x fp32[B, in_c*in_h*in_w] or int32[B, seq_len]; y int32[B] (all host).
 * out fp32[P] = sum_i clip(g_i) + sigma*C*z.  Optional outputs (may be NULL):
 *   norms[B]  unclipped ||g_i||;  clipped_sum[P] the fp64 sum before noise;  ties;
 *   pool_margin[B]  (also: smallest non-zero |z| over the example's ReLU pre-activations)
 *                   smallest non-zero gap between the maximum and the runner-up over the example's
 *   pool windows (+inf without pooling; exact ties go to the first maximum on every implementation): an fp32 implementation may route a window whose
 *   gap is at rounding level to the other element (see oracle_pool_near_ties);
 *   abs_sum[P]  sum_i |s_i g_i[j]|, the magnitude the terms of coordinate j had before they cancelled: rounding
 *   errors of any summation scale with it, so tests state their per-tensor tolerance in terms of it.
 * C = +inf disables clipping; sigma = 0 adds exactly nothing.  clip = 0 skips the
 * clipping branch altogether (the non-private summed gradient).  Returns 0. */
int oracle_dp_step(const or_model *m, const float *params, const void *x, const int32_t *y, int B, double C,
                   double sigma, uint64_t seed, int clip, float *out, double *norms, double *clipped_sum,
                   long *ties, double *pool_margin, double *abs_sum, int n_threads) {
  long P = oracle_num_params(m);
  double *theta = (double *)malloc(sizeof(double) * P);
  for (long j = 0; j < P; ++j) theta[j] = (double)params[j];
  long xstride = m->seq_len > 0 ? m->seq_len : (long)m->in_c * m->in_h * m->in_w;
  int nt = 1;
#ifdef _OPENMP
  nt = n_threads > 0 ? n_threads : omp_get_max_threads();
#endif
  if (nt > B) nt = B > 0 ? B : 1;
  double **acc = (double **)calloc(nt, sizeof(double *));
  double **mag = (double **)calloc(nt, sizeof(double *));
  long *tie_t = (long *)calloc(nt, sizeof(long));
#ifdef _OPENMP
#pragma omp parallel num_threads(nt)
#endif
  {
    int tid = 0;
#ifdef _OPENMP
    tid = omp_get_thread_num();
#endif
    double *a = (double *)calloc(P, sizeof(double));
    double *g = (double *)malloc(sizeof(double) * P);
    scratch *s = scratch_new(m);
    acc[tid] = a;
    double *ab = abs_sum ? (double *)calloc(P, sizeof(double)) : NULL;
    mag[tid] = ab;
    /* contiguous block of examples per thread */
    int lo = (int)((long)B * tid / nt), hi = (int)((long)B * (tid + 1) / nt);
    for (int i = lo; i < hi; ++i) {
      const void *xi = m->seq_len > 0 ? (const void *)((const int32_t *)x + i * xstride)
                                      : (const void *)((const float *)x + i * xstride);
      forward(m, theta, xi, y[i], s);
      backward(m, theta, xi, y[i], s, g);
      double n2 = 0;
      for (long j = 0; j < P; ++j) n2 += g[j] * g[j];
      double n = sqrt(n2);
      double sc = (clip && n > C) ? C / n : 1.0;
      if (norms) norms[i] = n;
      if (pool_margin) pool_margin[i] = s->margin;
      for (long j = 0; j < P; ++j) a[j] += sc * g[j];
      if (ab) for (long j = 0; j < P; ++j) ab[j] += fabs(sc * g[j]);
    }
    tie_t[tid] = s->ties;
    scratch_free(s);
    free(g);
  }
  for (int t = 1; t < nt; ++t) {
    for (long j = 0; j < P; ++j) acc[0][j] += acc[t][j];
    if (abs_sum) for (long j = 0; j < P; ++j) mag[0][j] += mag[t][j];
    tie_t[0] += tie_t[t];
  }
  if (abs_sum) memcpy(abs_sum, mag[0], sizeof(double) * P);
  if (ties) *ties = tie_t[0];
  if (clipped_sum) memcpy(clipped_sum, acc[0], sizeof(double) * P);
  if (sigma > 0) {
    double *z = (double *)malloc(sizeof(double) * (P + 4));
    oracle_noise(seed, P, z);
    for (long j = 0; j < P; ++j) out[j] = (float)(acc[0][j] + sigma * C * z[j]);
    free(z);
  } else {
    for (long j = 0; j < P; ++j) out[j] = (float)acc[0][j];
  }
  for (int t = 0; t < nt; ++t) { free(acc[t]); free(mag[t]); }
  free(acc); free(mag); free(tie_t); free(theta);
  return 0;
}

/* DPSGD item 4 after items 2-3 (Section 1): theta <- theta - (lr / B) * (clipped sum + sigma*C*z), the step taken
 * in double from the double-precision aggregate and rounded once to float.  theta_new may alias nothing. */
int oracle_sgd_step(const or_model *m, const float *params, const void *x, const int32_t *y, int B, double C,
                    double sigma, uint64_t seed, double lr, float *theta_new, int n_threads) {
  long P = oracle_num_params(m);
  if (B < 1) return -1;
  float *out = (float *)malloc(sizeof(float) * P);
  double *csum = (double *)malloc(sizeof(double) * P);
  double *z = (double *)malloc(sizeof(double) * P);
  int rc = (out && csum && z) ? 0 : -1;
  if (rc == 0) rc = oracle_dp_step(m, params, x, y, B, C, 0.0, seed, 1, out, NULL, csum, NULL, NULL, NULL, n_threads);
  if (rc == 0) {
    if (sigma > 0) oracle_noise(seed, P, z);
    for (long j = 0; j < P; ++j) {
      double agg = csum[j] + (sigma > 0 ? sigma * C * z[j] : 0.0);
      theta_new[j] = (float)((double)params[j] - lr / B * agg);
    }
  }
  free(out); free(csum); free(z);
  return rc;
}

/* DPSGD item 1 (Section 1): the minibatch.  The paper leaves the draw open; the reading taken is `batch` indices
 * drawn independently and uniformly from [0, n) (with replacement), index k from lane k%4 of the Philox block
 * with counter (k/4 lo, k/4 hi, 1, 0) -- third counter word 1, so the draw never shares a block with the noise
 * stream of the same seed (third word 0) -- mapped to the range by the multiply-shift (r * n) >> 32. */
void oracle_sample_indices(uint64_t seed, long n, int batch, int32_t *idx) {
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  for (int k = 0; k < batch; ++k) {
    uint64_t blk = (uint64_t)(k >> 2);
    uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), 1u, 0u}, r[4];
    oracle_philox4x32_10(ctr, key, r);
    idx[k] = (int32_t)(((uint64_t)r[k & 3] * (uint64_t)n) >> 32);
  }
}

/* `steps` iterations of the whole procedure (Section 1, items 1-4) on a dataset held in memory: step t draws its
 * minibatch and its noise from seed0 + t, takes the private step on the drawn examples and updates the parameters.
 * params_out receives the parameters after the last step (rounded to float after every step, as a caller that
 * chains oracle_sgd_step would hold them). */
int oracle_train(const or_model *m, const float *params, const void *data_x, const int32_t *data_y, long n, int steps,
                 int B, double C, double sigma, uint64_t seed0, double lr, float *params_out, int n_threads) {
  long P = oracle_num_params(m);
  long xstride = m->seq_len > 0 ? m->seq_len : (long)m->in_c * m->in_h * m->in_w;
  if (B < 1 || n < 1) return -1;
  float *cur = (float *)malloc(sizeof(float) * P), *next = (float *)malloc(sizeof(float) * P);
  int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * B), *yb = (int32_t *)malloc(sizeof(int32_t) * B);
  char *xb = (char *)malloc((size_t)B * xstride * 4);
  memcpy(cur, params, sizeof(float) * P);
  int rc = 0;
  for (int t = 0; t < steps && rc == 0; ++t) {
    oracle_sample_indices(seed0 + (uint64_t)t, n, B, idx);
    for (int k = 0; k < B; ++k) {
      memcpy(xb + (size_t)k * xstride * 4, (const char *)data_x + (size_t)idx[k] * xstride * 4, (size_t)xstride * 4);
      yb[k] = data_y[idx[k]];
    }
    rc = oracle_sgd_step(m, cur, xb, yb, B, C, sigma, seed0 + (uint64_t)t, lr, next, n_threads);
    float *tmp = cur; cur = next; next = tmp;
  }
  memcpy(params_out, cur, sizeof(float) * P);
  free(cur); free(next); free(idx); free(yb); free(xb);
  return rc;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// C-ABI library of the private gradient step (see include/dp_step.h).
// Plan at init (all shapes static, all workspace allocated once), then every
// dp_step only enqueues kernels on the context's stream.
#include "../../include/dp_step.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

#include "gemm_tile.h"
#include "conv_direct.h"
#include "conv_gram.h"
#include "ceilings.h"
#include "cnn_fused.h"
#include "conv_wino.h"
#include "conv_first.h"
#include "dense_fused.h"
#include "kernels_misc.h"
#include "kernels_seq.h"
#include "lstm_wgrad.h"
#include "operands.h"
#include "rows_gemm.h"

static thread_local char g_hip_err[256] = "";

#define HIP_TRY(expr)                                                                                \
  do {                                                                                               \
    hipError_t e_ = (expr);                                                                          \
    if (e_ != hipSuccess) {                                                                          \
      snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return DP_EHIP;                                                                                \
    }                                                                                                \
  } while (0)

// ---------------------------------------------------------------- epilogues / problems

template <class A_, class B_>
struct ProbBase {
  typedef A_ A;
  typedef B_ B;
  int M, N, K, k_chunk, tiles_n, tiles, splits, groups;
  A a;
  B b;
};

// out[m*ld + n] = act(acc + bias[n])                                  (dense forward, LSTM input projection)
template <class A_, class B_>
struct ProbBiasAct : ProbBase<A_, B_> {
  static constexpr bool kReduce = false;
  float *out; const float *bias; int ld, act;
  DEVI void store(int, int, int m, int n, float v) const { out[(long)m * ld + n] = act_apply(act, v + bias[n]); }
};

// out[z*zstride + m*ld + n] = acc                                     (batched plain product)
template <class A_, class B_>
struct ProbBatchOut : ProbBase<A_, B_> {
  static constexpr bool kReduce = false;
  float *out; long zstride; int ld;
  DEVI void store(int z, int, int m, int n, float v) const { out[z * zstride + (long)m * ld + n] = v; }
};

// out[m*ld + n] = acc * act'(a_prev[m*ld + n])                        (dense backward-data)
template <class A_, class B_>
struct ProbBwdAct : ProbBase<A_, B_> {
  static constexpr bool kReduce = false;
  float *out; const float *a_prev; int ld, act;
  DEVI void store(int, int, int m, int n, float v) const {
    long o = (long)m * ld + n;
    out[o] = act ? v * act_deriv_from_out(act, a_prev[o]) : v;
  }
};

// conv forward: m = output channel, n = pixel (b, p): out[b, m, p] = act(acc + bias[m])
template <class A_, class B_>
struct ProbConvFwd : ProbBase<A_, B_> {
  static constexpr bool kReduce = false;
  float *out; const float *bias; int D, P, act; FastDiv dP;
  DEVI void store(int, int, int m, int n, float v) const {
    int b = (int)dP.div(n), p = n - b * P;
    out[((long)b * D + m) * P + p] = act_apply(act, v + bias[m]);
  }
};

// conv backward-data: m = input channel, n = input pixel (b, ih*W+iw): out[b, m, hw] = acc * act'(a_prev)
template <class A_, class B_>
struct ProbConvBwd : ProbBase<A_, B_> {
  static constexpr bool kReduce = false;
  float *out; const float *a_prev; int C, HW, act; FastDiv dHW;
  DEVI void store(int, int, int m, int n, float v) const {
    int b = (int)dHW.div(n), r = n - b * HW;
    long o = ((long)b * C + m) * HW + r;
    out[o] = act ? v * act_deriv_from_out(act, a_prev[o]) : v;
  }
};

// split-K partial of a clipped sum: part[split*stride + m*ldm + n]; if bias_col >= 0 the column
// n == bias_col goes to bias_off + m instead (conv: bias gradient is the ones-tap column).
template <class A_, class B_>
struct ProbPartial : ProbBase<A_, B_> {
  static constexpr bool kReduce = false;
  float *part; long stride; int ldm, bias_col; long bias_off;
  DEVI void store(int, int split, int m, int n, float v) const {
    long o = (n == bias_col) ? bias_off + m : (long)m * ldm + n;
    part[split * stride + o] = v;
  }
};

// per-example weight-gradient tile, squared and summed: slot[(slot0 + tile)*slot_stride + z]
template <class A_, class B_>
struct ProbSqNorm : ProbBase<A_, B_> {
  static constexpr bool kReduce = true;
  float *slots; long slot_stride; int slot0;
  float *gstore; long gstride; // optional: example z's gradient is also written to gstore[z*gstride + m*N + n]
  DEVI float contrib(int z, int m, int n, float v) const {
    if (gstore) gstore[z * gstride + (long)m * this->N + n] = v;
    return v * v;
  }
  DEVI void store_tile(int z, int tile, float s) const { slots[(long)(slot0 + tile) * slot_stride + z] = s; }
};

// ---------------------------------------------------------------- context

struct Layer {
  dp_layer_desc d;
  int inC, inH, inW, outC, outH, outW; // chw view; vectors are C x 1 x 1; sequences: C = T, H = D
  long in_size, out_size;              // floats per example
  long p_off, p_count;
  long pstride = 0; // floats between split-K partial rows: p_count rounded up to 16 bytes
  float *a = nullptr; // output activations [maxB, out_size]
  float *g = nullptr; // gradient w.r.t. pre-activation (w.r.t. output where the layer has no activation)
  uint8_t *arg = nullptr;
  float *part = nullptr; // split-K partials of the clipped sum [max_split][p_count]
  float *fpart = nullptr; int fsplit = 1; // dense forward: split-K partials [fsplit][maxB*d_out] when the output is small
  int max_split = 0;
  int max_slots = 0;
  ConvGeom geom;
  // stride-1 3x3 convolutions: LDS-staged direct kernels (otherwise the generic contraction)
  bool dir_fwd = false, dir_bwd = false, dir_wg = false, wg_flat = false;
  bool first_fwd = false; // the network's first layer, at most 3 input channels: forward by conv_first_kernel
  bool first_wg = false;  // ... and its per-example weight gradient (norm pass) by conv_first_wgrad_kernel
  bool wg_ws = false; // weight gradient with specialised staging / multiplying waves (two LDS buffers)
  bool gram = false;  // per-example norm from the P x P Gram matrices (small planes)
  float *cols = nullptr; // strided convolutions, backward-data: [maxB][C*KH*KW][OH*OW] products W^T Delta
  float *gst = nullptr; // [maxB][gorder.n_w + D] per-example gradients written by the norm pass (large planes)
  GradOrder gorder{};
  int fwd_npw = 64, bwd_npw = 64, wg_db = 1;
  ConvTile t_fwd, t_bwd, t_wgn, t_wgc;
  float *wt_f = nullptr, *wt_b = nullptr; // re-laid weights for the direct kernels
  // forward / backward-data by the F(2x2, 3x3) minimal-filtering kernel: output-channel blocks per workgroup (0: not
  // used), transformed weights [16][cpad][mpad]
  int wino_f = 0, wino_b = 0;
  bool wino_wg = false; // batch sum of the weight gradient in the F(3x3, 2x2) form on 8x8 planes (any multiple of 64 output channels)
  bool u_f_planned = false; // pad-1 3x3 stride-1 layer with even planes: the minimal-filtering family applies
  bool wino_wgu = false;    // per-example and batch weight gradient in that form on 16- and 32-wide planes (32 / 64 output channels)
  bool wino_norm = false; // norm pass (with stored gradients) in the same form: 16- and 32-wide planes, 32 or 64 output channels
  float *u_f = nullptr, *u_b = nullptr;
  int uf_cpad = 0, uf_mpad = 0, ub_cpad = 0, ub_mpad = 0;
  std::vector<std::string> lab; // profiling labels "<kernel>#<layer index>" (stable after init)
  // embedding: counting-sort workspace of the clipped sum
  int *e_count = nullptr, *e_start = nullptr, *e_chunk0 = nullptr, *e_cursor = nullptr, *e_list = nullptr;
  // lstm
  bool lstm_wg = false; // per-example weight gradient by lstm_wgrad_kernel (16x16 MFMA blocks, one example per two workgroups)
  float *gates = nullptr, *cs = nullptr, *hs = nullptr;
  int T = 0, Din = 0, H = 0;
};

struct ProfRec { int label; hipEvent_t e0, e1; };

// label "<name>#<layer index>", created once per layer and name (pointer stays valid until free)
static const char *layer_label(Layer &l, int li, const char *name) {
  std::string want = std::string(name) + "#" + std::to_string(li);
  for (auto &s : l.lab)
    if (s == want) return s.c_str();
  return nullptr;
}
static const char *const kLayerLabels[] = {"dense_fwd", "dense_fwd_epilogue", "dense_norm", "dense_bwd_data", "dense_clipped_sum",
                                           "conv_weight_layout", "conv_fwd", "conv_wgrad_norm", "conv_bwd_data", "conv_clipped_sum",
                                           "maxpool_fwd", "maxpool_bwd", "lstm_xproj", "lstm_fwd", "lstm_bwd", "lstm_wgrad_norm",
                                           "lstm_dx", "lstm_clipped_sum", "emb_norm", "emb_gather", "emb_bucket", "emb_scatter", "fill_zero",
                                           "seq_mean_fwd", "seq_mean_bwd", "avgpool_fwd", "avgpool_bwd", "conv_weighted_sum", "lstm_weighted_sum"};

struct dp_ctx {
  dp_model_desc m;
  std::vector<Layer> L;
  int maxB = 0;
  long P = 0;
  hipStream_t stream = nullptr;
  std::vector<void *> allocs;
  size_t ws_bytes = 0;
  float *slots = nullptr; int max_slots = 0;
  float *norms = nullptr, *s = nullptr;
  float *ones = nullptr; // [maxB] of 1.0: the clip factors of a step that clips nothing
  int last_batch = -1;
  dp_plan_options opt{}; // route switches, read once at init
  int *bad = nullptr;    // dp_step_validate: number of out-of-range ids / labels
  uint32_t *xb = nullptr; int *yb = nullptr, *idx = nullptr; // dp_step_loop: the drawn minibatch (allocated on its first call)
  bool fused1 = false; // the model is one dense layer small enough for dense1_fused_kernel
  bool fusedcnn = false; float *cnn_part = nullptr; // the small MNIST-shaped CNN in one launch (cnn_small_fused_kernel)
  bool joint2 = false; // fused2 / head2 and both clipped sums in one dense_small_gemm_kernel launch
  bool fused2 = false; // two dense layers: everything between the hidden layer's forward product and the clipped sums in dense2_mid_kernel
  // The embedding layer's counting sort of the batch's tokens depends on the inputs alone: it runs on a stream of the
  // library's own (fork / join by events) beside the forward pass.
  hipStream_t side = nullptr; hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool head2 = false;  // a deeper network that ends in two dense layers: the same kernel up to both layers' norms and delta1
  // profiling
  bool prof = false;
  std::vector<const char *> labels; // string literals
  std::vector<int> label_launches;
  std::vector<float> label_ms;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  size_t pool_used = 0;
  int err = 0;
};

static int label_id(dp_ctx *c, const char *name) {
  for (size_t i = 0; i < c->labels.size(); ++i)
    if (strcmp(c->labels[i], name) == 0) return (int)i;
  c->labels.push_back(name);
  c->label_launches.push_back(0);
  c->label_ms.push_back(0.f);
  return (int)c->labels.size() - 1;
}

// Brackets a launch with events when profiling is on.
struct Launcher {
  dp_ctx *c;
  bool waste_aware() const { return c->opt.gemm_plain_tiles == 0; }
  template <class F>
  void operator()(const char *label, dim3, dim3, F &&f) const {
    if (c->prof && c->pool_used + 2 <= c->pool.size()) {
      ProfRec r;
      r.label = label_id(c, label);
      r.e0 = c->pool[c->pool_used++];
      r.e1 = c->pool[c->pool_used++];
      (void)hipEventRecord(r.e0, c->stream);
      f(c->stream);
      (void)hipEventRecord(r.e1, c->stream);
      c->recs.push_back(r);
    } else {
      f(c->stream);
    }
  }
};

template <class T>
static int dev_alloc(dp_ctx *c, T **p, size_t n) {
  void *q = nullptr;
  size_t bytes = (n ? n : 1) * sizeof(T);
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) {
    snprintf(g_hip_err, sizeof(g_hip_err), "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
    return DP_ENOMEM;
  }
  c->allocs.push_back(q);
  c->ws_bytes += bytes;
  *p = (T *)q;
  return DP_OK;
}

static ConvGeom make_geom(const Layer &l) {
  ConvGeom g;
  g.C = l.inC; g.H = l.inH; g.W = l.inW; g.D = l.outC; g.OH = l.outH; g.OW = l.outW;
  g.KH = l.d.kh; g.KW = l.d.kw; g.S = l.d.stride; g.PAD = l.d.pad;
  g.CKK = g.C * g.KH * g.KW; g.P = g.OH * g.OW;
  g.dP.init(g.P); g.dOW.init(g.OW); g.dKK.init(g.KH * g.KW); g.dKW.init(g.KW); g.dHW.init(g.H * g.W); g.dW.init(g.W);
  return g;
}


// ---------------------------------------------------------------- direct convolution planning

static bool make_conv_tile(ConvTile &t, int OH, int OW, int KH, int KW, int np_max, bool odd_plane, int nimg_cap) {
  if (OW > np_max || OW < 1) return false;
  if (OH * OW <= np_max) {
    t.NIMG = np_max / (OH * OW);
    if (t.NIMG > nimg_cap) t.NIMG = nimg_cap;
    t.TR = OH; t.row_tiles = 1;
  } else {
    t.NIMG = 1; t.TR = np_max / OW; t.row_tiles = ceil_div(OH, t.TR);
  }
  t.LDW = OW + KW - 1;
  t.IMGPL = (t.TR + KH - 1) * t.LDW;
  t.XPLANE = t.NIMG * t.IMGPL;
  if (odd_plane && (t.XPLANE & 1) == 0) t.XPLANE += 1;
  t.dOW.init(OW); t.dTROW.init(t.TR * OW); t.dLDW.init(t.LDW); t.dIMGPL.init(t.IMGPL);
  t.dXPLANE.init(t.XPLANE); t.dRT.init(t.row_tiles);
  return true;
}

static bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// Region of the 32 tiles of a minimal-filtering workgroup (tiles per row and per image are powers of two): whole
// tile rows of one image, or whole images.  Returns the staging items per thread for a chunk of 8 channels.
static int make_wino_region(ConvWinoRegion &rg, int H, int W) {
  const int TW = W / 2, TPI = (H / 2) * (W / 2);
  if (TW > 32) return 1 << 20;
  if (TPI >= 32) { rg.NIMG = 1; rg.ROWS = 2 * (32 / TW); } else { rg.NIMG = 32 / TPI; rg.ROWS = H; }
  rg.LDW = W + 2; rg.IMGPL = (rg.ROWS + 2) * rg.LDW; rg.RS = rg.NIMG * rg.IMGPL;
  rg.dRS.init(rg.RS); rg.dIMGPL.init(rg.IMGPL); rg.dLDW.init(rg.LDW);
  return ceil_div(WINO_CC * rg.RS, 256);
}

static void plan_direct_conv(Layer &l, int maxB, const dp_plan_options &opt) {
  const bool allow = opt.generic_conv == 0;
  const ConvGeom &g = l.geom;
  if (!allow || g.S != 1 || g.KH != 3 || g.KW != 3 || g.PAD > 2) return;
  if ((long)maxB * g.C * g.H * g.W >= (1l << 31) || (long)maxB * g.D * g.P >= (1l << 31)) return;
  // forward: output OH x OW
  {
    int npw = ((long)maxB * g.P / 256 >= 512) ? 64 : 32;
    if (make_conv_tile(l.t_fwd, g.OH, g.OW, 3, 3, 4 * npw, false, 1 << 20) &&
        l.t_fwd.XPLANE <= CONV_XPLANE_MAX) { l.dir_fwd = true; l.fwd_npw = npw; }
  }
  // backward-data: correlation of Delta (OH x OW) with flipped weights, output H x W, pad' = 2 - pad
  {
    int npw = ((long)maxB * g.H * g.W / 256 >= 512) ? 64 : 32;
    if (make_conv_tile(l.t_bwd, g.H, g.W, 3, 3, 4 * npw, false, 1 << 20) &&
        l.t_bwd.XPLANE <= CONV_XPLANE_MAX) { l.dir_bwd = true; l.bwd_npw = npw; }
  }
  // Minimal-filtering form for pad-1 planes whose tile grid is a power of two: 16 multiplies per 2x2 outputs and
  // channel instead of 36.  Measured against the direct kernel: ahead wherever a workgroup covers 64 output
  // channels; with 32 it is ahead only for short channel loops; the grid must still fill the chip.
  if (l.dir_fwd && l.dir_bwd && g.PAD == 1 && g.H == g.OH && g.W == g.OW && (g.H & 1) == 0 && (g.W & 1) == 0 &&
      is_pow2(g.W / 2) && is_pow2((g.H / 2) * (g.W / 2)) && !opt.no_minimal_filtering) {
    l.u_f_planned = true;
    const bool all = opt.minimal_filtering_all != 0; // tests: the kernel for every eligible shape
    ConvWinoRegion rg;
    const bool fits = make_wino_region(rg, g.H, g.W) <= 9; // staging items per thread the kernels are built for
    auto pick = [&](int Cin, int M) {
      int db = M > 32 ? 2 : 1;
      if (!fits) return 0;
      if (all) return db;
      if (Cin < 16) return 0;
      const long groups = ((long)maxB * (g.H / 2) * (g.W / 2) + 31) / 32;
      // 64 output channels per workgroup only where that still fills the chip; below about half a workgroup per CU
      // the direct kernel with its narrower tiles measured as fast or faster
      if (db == 2 && groups * ceil_div(M, 64) < 512) db = 1;
      if (groups * ceil_div(M, 32 * db) < 128) return 0;
      // 32 output channels per workgroup: the transform is amortised over half the multiplies, and the epilogue
      // over the channel loop only
      if (db == 1 && Cin < 32) return 0;
      return db;
    };
    // weight gradients in the same form with the roles exchanged (conv_wino_wgrad_unit_kernel): batch sums on 8x8 planes
    l.wino_wg = g.H == 8 && g.W == 8 && g.C % 32 == 0 && g.D % 64 == 0 && !opt.no_minimal_filtering_wgrad;
    // and per band of 16 tiles on 16- and 32-wide planes: whole blocks of 32 input channels, 32 or 64 output channels
    l.wino_wgu = g.C % 32 == 0 && (g.D == 32 || g.D == 64) &&
                 ((g.W == 32 && g.D == 32 && g.H % 2 == 0) || (g.W == 16 && g.H % 4 == 0)) &&
                 !opt.no_minimal_filtering_wgrad;
    l.wino_f = pick(g.C, g.D);
    l.wino_b = pick(g.D, g.C);
  }
  // per-example norm from Gram matrices: P^2 (9C + D) multiply-adds instead of 9 C D P, for the two plane sizes
  // the kernel is built for (pad 1, so the input plane equals the output plane)
  if (g.PAD == 1 && g.H == g.OH && g.W == g.OW && ((g.OH == 8 && g.OW == 8) || (g.OH == 4 && g.OW == 4)) &&
      (long)g.P * (g.CKK + g.D) < (long)g.D * g.CKK && !opt.no_gram)
    l.gram = true;
  // weight gradient
  const bool flat = g.C * 9 <= 32 && g.D <= 32;
  if ((g.C >= 16 || flat) && (g.OW & 3) == 0 && (g.W & 3) == 0) {
    int db = g.D <= 32 ? 1 : (g.D <= 64 ? 2 : 4);
    int pch_max = flat ? 256 : (db <= 2 ? 128 : 64);
    const int xch = flat ? g.C : 32;
    bool ok = make_conv_tile(l.t_wgn, g.OH, g.OW, 3, 3, pch_max, true, 1) &&
              make_conv_tile(l.t_wgc, g.OH, g.OW, 3, 3, pch_max, true, 1 << 20);
    if (ok) {
      long lds_n = (long)xch * l.t_wgn.XPLANE + 32l * db * ((l.t_wgn.NIMG * l.t_wgn.TR * g.OW) | 1);
      long lds_c = (long)xch * l.t_wgc.XPLANE + 32l * db * ((l.t_wgc.NIMG * l.t_wgc.TR * g.OW) | 1);
      bool fits = (lds_n + 64) * 4 <= 64 * 1024 && (lds_c + 64) * 4 <= 64 * 1024;
      // room in the staging area for the cross-wave sum of the waves that split the pixel pairs
      const long xs = flat ? 3l * 16 * 64 : (db == 1 ? 2l * 5 * 16 * 64 : 0);
      if (lds_n < xs || lds_c < xs) fits = false;
      for (const ConvTile *t : {&l.t_wgn, &l.t_wgc}) {
        const int pch = t->NIMG * t->TR * g.OW;
        if ((long)xch * t->NIMG * (t->TR + 2) * (g.W / 4) > CONV_WG_XV * 256) fits = false; // input items per thread
        if (32l * db * pch / 4 > ((db == 1 && !flat) ? 4 : 8) * 256) fits = false;          // Delta items per thread
        if ((pch & 3) != 0) fits = false;
      }
      if (fits) { l.dir_wg = true; l.wg_db = db; l.wg_flat = flat; }
      // specialised-wave variant: two staging buffers + the cross-wave area must fit one CU's LDS
      // (measured: pays where the single-buffer kernel runs one workgroup per CU, i.e. 128 output channels)
      if (fits && (db == 4 || opt.specialised_waves_all)) {
        const long ws = 2 * std::max(lds_n, lds_c) + xs + 64;
        // its bias sums are exchanged inside a wave: the threads of one Delta row must be a power of two of lanes
        const int pq_n = l.t_wgn.NIMG * l.t_wgn.TR * g.OW / 4, pq_c = l.t_wgc.NIMG * l.t_wgc.TR * g.OW / 4;
        const bool rows_ok = is_pow2(pq_n) && pq_n <= 64 && is_pow2(pq_c) && pq_c <= 64;
        l.wg_ws = ws * 4 + 2048 <= 160 * 1024 && rows_ok && !opt.no_specialised_waves;
      }
    }
  }
}

template <class LN>
static void launch_conv_s1(const LN &Ln, const char *label, const ConvS1Args &a, int npw) {
  int dt = a.M <= 32 ? 32 : (a.M <= 64 ? 64 : 128);
  const int cc = a.Cin <= 4 ? 4 : 8; // first layers: a chunk of four channels covers the whole input
  const int pix_blocks = a.t.NIMG > 1 ? ceil_div(a.B, a.t.NIMG) : a.B * a.t.row_tiles;
  // a small batch of small planes leaves CUs idle with wide output tiles: narrow them until the grid fills the chip
  const int min_blocks = Ln.c->opt.conv_min_blocks > 0 ? Ln.c->opt.conv_min_blocks : 512;
  while (dt > 32 && pix_blocks * ceil_div(a.M, dt) < min_blocks) dt >>= 1;
  dim3 grid(pix_blocks, ceil_div(a.M, dt)), block(256);
  size_t smem = sizeof(float) * ((size_t)cc * a.t.XPLANE + (size_t)cc * 9 * dt);
#define DP_CONV_CASE(dt_, npw_, cc_)                                                                 \
  if (dt == dt_ && npw == npw_ && cc == cc_) {                                                       \
    Ln(label, grid, block, [&](hipStream_t st) {                                                     \
      hipLaunchKernelGGL((conv_s1_kernel<3, 3, dt_, npw_, cc_>), grid, block, smem, st, a);          \
    });                                                                                              \
    return;                                                                                          \
  }
  DP_CONV_CASE(32, 64, 8) DP_CONV_CASE(64, 64, 8) DP_CONV_CASE(128, 64, 8)
  DP_CONV_CASE(32, 32, 8) DP_CONV_CASE(64, 32, 8) DP_CONV_CASE(128, 32, 8)
  DP_CONV_CASE(32, 64, 4) DP_CONV_CASE(64, 64, 4) DP_CONV_CASE(128, 64, 4)
  DP_CONV_CASE(32, 32, 4) DP_CONV_CASE(64, 32, 4) DP_CONV_CASE(128, 32, 4)
#undef DP_CONV_CASE
}

static int ilog2_exact(int v) { int s = 0; while ((1 << s) < v) ++s; return s; }

template <class LN>
static void launch_conv_wino(const LN &Ln, const char *label, ConvWinoArgs a, int db) {
  a.tw_shift = ilog2_exact(a.W / 2);
  a.tpi_shift = ilog2_exact((a.H / 2) * (a.W / 2));
  ConvWinoRegion rg;
  const int need = make_wino_region(rg, a.H, a.W);
  const int xi = need <= 6 ? 6 : (need <= 7 ? 7 : 9);
  const long tiles = (long)a.B * (a.H / 2) * (a.W / 2);
  dim3 grid((unsigned)((tiles + 31) / 32), a.Mpad / (32 * db)), block(256);
  // 32 input and at most 32 output channels: persistent workgroups that keep the transformed weights in registers
  // (wider layers run it once per block of 32 output channels: the transform is repeated per block, which costs less
  // than the per-group prologue of the kernels below at four chunks per group)
  if (a.Cin == 32 && a.Cpad == 32 && a.Mpad % 32 == 0 && a.Mpad <= 64 && !Ln.c->opt.no_resident_weights) {
    // what the kernel fixes at compile time for whole blocks of 32 output channels (every store unconditional)
    const int fast = a.M % 32 != 0 ? 0 : (a.bias != nullptr ? (a.pool == 1 ? 1 : (a.pool == 0 ? 3 : 0)) : (a.act != 0 ? 2 : 0));
#define DP_WINOR_CASE(G_, cond_)                                                                  \
  if (a.W == G_::W && (cond_)) {                                                                  \
    const int n_groups = a.B * (a.H / G_::ROWS);                                                  \
    const int per_wg = ceil_div(n_groups * (a.Mpad / 32), 512); /* two workgroups per CU, all resident */ \
    dim3 rgrid(ceil_div(n_groups, per_wg), a.Mpad / 32);                                          \
    Ln(label, rgrid, block, [&](hipStream_t st) {                                                 \
      if (fast == 1) hipLaunchKernelGGL((conv_wino_res_kernel<G_, 1>), rgrid, block, 0, st, a, n_groups, per_wg);      \
      else if (fast == 2) hipLaunchKernelGGL((conv_wino_res_kernel<G_, 2>), rgrid, block, 0, st, a, n_groups, per_wg); \
      else if (fast == 3) hipLaunchKernelGGL((conv_wino_res_kernel<G_, 3>), rgrid, block, 0, st, a, n_groups, per_wg); \
      else hipLaunchKernelGGL((conv_wino_res_kernel<G_, 0>), rgrid, block, 0, st, a, n_groups, per_wg);                \
    });                                                                                           \
    return;                                                                                       \
  }
    DP_WINOR_CASE(WinoG32, a.H % 4 == 0) DP_WINOR_CASE(WinoG16, a.H % 8 == 0)
#undef DP_WINOR_CASE
  }
  // 64 output channels per workgroup, whole chunks of input channels, one of the plane shapes the register-operand
  // kernel is built for
  if (db == 2 && a.Cin % WINO_CC == 0) {
#define DP_WINO3_CASE(G_, cond_)                                                                  \
  if (a.W == G_::W && (cond_)) {                                                                  \
    Ln(label, grid, block, [&](hipStream_t st) {                                                  \
      hipLaunchKernelGGL((conv_wino_reg_kernel<2, G_>), grid, block, 0, st, a);                   \
    });                                                                                           \
    return;                                                                                       \
  }
    DP_WINO3_CASE(WinoG32, a.H % 4 == 0) DP_WINO3_CASE(WinoG16, a.H % 8 == 0) DP_WINO3_CASE(WinoG8, a.H == 8)
#undef DP_WINO3_CASE
  }
  const size_t smem = sizeof(float) * (2 * 16 * WINO_CC * 32 + 2 * WINO_CC * (size_t)rg.RS);
#define DP_WINO_CASE(db_, xi_)                                                                    \
  if (db == db_ && xi == xi_) {                                                                   \
    Ln(label, grid, block, [&](hipStream_t st) {                                                  \
      hipLaunchKernelGGL((conv_wino_kernel<db_, xi_>), grid, block, smem, st, a, rg);             \
    });                                                                                           \
    return;                                                                                       \
  }
  DP_WINO_CASE(1, 6) DP_WINO_CASE(1, 7) DP_WINO_CASE(1, 9) DP_WINO_CASE(2, 6) DP_WINO_CASE(2, 7) DP_WINO_CASE(2, 9)
#undef DP_WINO_CASE
}

static size_t conv_wgrad_ws_smem(const ConvWgArgs &a, int db, bool flat) {
  const size_t buf = (size_t)(flat ? a.C : 32) * a.t.XPLANE + 32 * (size_t)db * a.LDP;
  const size_t xs = flat ? 3 * 16 * 64 : (db == 1 ? 2 * 5 * 16 * 64 : 0);
  return sizeof(float) * (2 * buf + xs + 64); // + 64: look-ahead reads of skipped steps past the last staged row
}

// the specialised-wave kernels use more than the default 64 KB of dynamic LDS
static bool conv_wgrad_ws_enable() {
  bool ok = true;
#define DP_WS_ATTR(db_, flat_, clip_)                                                                          \
  ok = ok && hipFuncSetAttribute((const void *)conv_s1_wgrad_ws_kernel<3, 3, db_, flat_, clip_>,               \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 2048) == hipSuccess;
  DP_WS_ATTR(1, false, false) DP_WS_ATTR(1, false, true) DP_WS_ATTR(2, false, false) DP_WS_ATTR(2, false, true)
  DP_WS_ATTR(1, true, false) DP_WS_ATTR(1, true, true) DP_WS_ATTR(4, false, false) DP_WS_ATTR(4, false, true)
#undef DP_WS_ATTR
  return ok;
}

template <class LN>
static void launch_conv_wgrad(const LN &Ln, const char *label, const ConvWgArgs &a, int db, bool flat, bool ws, int groups) {
  dim3 grid(flat ? 1 : ceil_div(a.C, 32), groups), block(ws ? 512 : 256);
  // + 64 floats: the K loop's look-ahead reads of skipped steps may run past the last staged row
  size_t smem = ws ? conv_wgrad_ws_smem(a, db, flat)
                   : sizeof(float) * ((size_t)(flat ? a.C : 32) * a.t.XPLANE + 32 * (size_t)db * a.LDP + 64);
#define DP_WG_CASE(db_, flat_)                                                                       \
  if (!ws && db == db_ && flat == flat_) {                                                           \
    Ln(label, grid, block, [&](hipStream_t st) {                                                     \
      if (a.mode == 0)                                                                               \
        hipLaunchKernelGGL((conv_s1_wgrad_kernel<3, 3, db_, flat_, false>), grid, block, smem, st, a); \
      else                                                                                           \
        hipLaunchKernelGGL((conv_s1_wgrad_kernel<3, 3, db_, flat_, true>), grid, block, smem, st, a);  \
    });                                                                                              \
    return;                                                                                          \
  }
  DP_WG_CASE(1, false) DP_WG_CASE(2, false) DP_WG_CASE(4, false) DP_WG_CASE(1, true)
#undef DP_WG_CASE
#define DP_WS_CASE(db_, flat_)                                                                       \
  if (ws && db == db_ && flat == flat_) {                                                            \
    Ln(label, grid, block, [&](hipStream_t st) {                                                     \
      if (a.mode == 0)                                                                               \
        hipLaunchKernelGGL((conv_s1_wgrad_ws_kernel<3, 3, db_, flat_, false>), grid, block, smem, st, a); \
      else                                                                                           \
        hipLaunchKernelGGL((conv_s1_wgrad_ws_kernel<3, 3, db_, flat_, true>), grid, block, smem, st, a);  \
    });                                                                                              \
    return;                                                                                          \
  }
  DP_WS_CASE(1, false) DP_WS_CASE(2, false) DP_WS_CASE(4, false) DP_WS_CASE(1, true)
#undef DP_WS_CASE
}

// Arguments for the slice of at most 128 output channels that starts at channel d0 (layers with more output
// channels take one launch per slice: Delta and the clipped-mode output are offset to the slice).
#define DP_WG_DSLICE 128
static ConvWgArgs make_wg_args(const Layer &l, const float *x, int B, const ConvTile &t, int d0) {
  const ConvGeom &g = l.geom;
  ConvWgArgs a{};
  a.x = x; a.delta = l.g + (long)d0 * g.P; a.B = B; a.C = g.C; a.H = g.H; a.W = g.W; a.OH = g.OH; a.OW = g.OW; a.pad = g.PAD;
  a.D = std::min(DP_WG_DSLICE, g.D - d0); a.Dstride = g.D;
  a.bias_off = (long)g.D * g.CKK + d0 - (long)d0 * g.CKK; // relative to the slice's own output base
  a.t = t;
  a.PCH = t.NIMG * t.TR * g.OW; a.LDP = a.PCH | 1;
  a.WQ = g.W / 4; a.ROWS = t.TR + 2;
  a.dWQ.init(a.WQ); a.dROWS.init(a.ROWS); a.dNIMG.init(t.NIMG); a.dPQ.init(a.PCH / 4);
  return a;
}

// split-K partials: at most 1024 splits and 16 M floats per parameter tensor
#define DP_MAX_SPLIT 1024
#define DP_MAX_PART_FLOATS (16l << 20)

// ---------------------------------------------------------------- init / free

extern "C" int dp_step_init(const dp_model_desc *model, int max_batch, void *hip_stream, dp_ctx **out) {
  return dp_step_init_ex(model, max_batch, hip_stream, nullptr, out);
}

extern "C" int dp_step_init_ex(const dp_model_desc *model, int max_batch, void *hip_stream, const dp_plan_options *options,
                               dp_ctx **out) {
  if (!model || !out || max_batch < 1 || model->n_layers < 1 || !model->layers) return DP_EINVAL;
  dp_ctx *c = new (std::nothrow) dp_ctx();
  if (!c) return DP_ENOMEM;
  if (options) c->opt = *options;
  c->m = *model;
  c->m.layers = nullptr;
  c->maxB = max_batch;
  c->stream = (hipStream_t)hip_stream;
  int rc = DP_OK;
  int curC = model->in_c, curH = model->in_h, curW = model->in_w;
  bool is_tok = model->seq_len > 0, is_seq = false;
  long off = 0;
  int total_slots = 0;
  for (int i = 0; i < model->n_layers && rc == DP_OK; ++i) {
    Layer l;
    l.d = model->layers[i];
    l.inC = curC; l.inH = curH; l.inW = curW;
    l.p_off = off;
    l.p_count = 0;
    switch (l.d.kind) {
    case DP_DENSE:
      if (is_tok || is_seq || l.d.in_features != curC * curH * curW || l.d.out_features < 1) { rc = DP_EINVAL; break; }
      l.outC = l.d.out_features; l.outH = l.outW = 1;
      l.p_count = (long)l.d.in_features * l.d.out_features + l.d.out_features;
      l.max_slots = 1;
      break;
    case DP_CONV2D:
      if (is_tok || is_seq || l.d.in_ch != curC || l.d.kh < 1 || l.d.kw < 1 || l.d.stride < 1 || l.d.pad < 0) { rc = DP_EINVAL; break; }
      l.outC = l.d.out_ch;
      l.outH = (curH + 2 * l.d.pad - l.d.kh) / l.d.stride + 1;
      l.outW = (curW + 2 * l.d.pad - l.d.kw) / l.d.stride + 1;
      if (l.outH < 1 || l.outW < 1) { rc = DP_EINVAL; break; }
      l.p_count = (long)l.d.out_ch * l.d.in_ch * l.d.kh * l.d.kw + l.d.out_ch;
      l.max_slots = ceil_div(l.d.out_ch, 32) * ceil_div(l.d.in_ch * l.d.kh * l.d.kw + 1, 32);
      break;
    case DP_MAXPOOL2D:
    case DP_AVGPOOL2D:
      if (is_tok || is_seq || i == 0 || l.d.kh < 1 || l.d.kw < 1 || l.d.stride < 1 || l.d.kh * l.d.kw > 255) { rc = DP_EINVAL; break; }
      if (model->layers[i - 1].kind != DP_CONV2D) { rc = DP_EUNSUPPORTED; break; }
      l.outC = curC;
      l.outH = (curH - l.d.kh) / l.d.stride + 1;
      l.outW = (curW - l.d.kw) / l.d.stride + 1;
      if (l.outH < 1 || l.outW < 1) { rc = DP_EINVAL; break; }
      break;
    case DP_EMBEDDING:
      if (!is_tok || i != 0 || l.d.vocab < 1 || l.d.vocab > (1 << 21) || l.d.embed_dim < 1 || model->seq_len > EMB_TMAX) { rc = DP_EINVAL; break; }
      l.inC = model->seq_len; l.inH = l.inW = 1;
      l.outC = model->seq_len; l.outH = l.d.embed_dim; l.outW = 1;
      l.p_count = (long)l.d.vocab * l.d.embed_dim;
      l.max_slots = 1;
      is_tok = false; is_seq = true;
      break;
    case DP_LSTM_LAST:
    case DP_LSTM_SEQ:
      if (!is_seq || l.d.hidden < 1 || l.d.in_features != curH) { rc = DP_EINVAL; break; }
      if (l.d.hidden > 128 || i == 0 || model->layers[i - 1].kind != DP_EMBEDDING) { rc = DP_EUNSUPPORTED; break; }
      l.T = curC; l.Din = curH; l.H = l.d.hidden;
      l.lstm_wg = lstm_wgrad_fits(l.Din, l.H, l.T) && !c->opt.no_lstm_wgrad;
      l.p_count = (long)l.Din * 4 * l.H + (long)l.H * 4 * l.H + 4 * l.H;
      l.max_slots = ceil_div(l.Din + l.H + 1, 32) * ceil_div(4 * l.H, 32);
      if (l.lstm_wg) l.max_slots = std::max(l.max_slots, LWG_SLOTS);
      if (l.d.kind == DP_LSTM_SEQ) {
        if (i + 1 >= model->n_layers || model->layers[i + 1].kind != DP_SEQ_MEAN) { rc = DP_EUNSUPPORTED; break; }
        l.outC = l.T; l.outH = l.H; l.outW = 1; // stays a sequence
      } else {
        l.outC = l.H; l.outH = l.outW = 1;
        is_seq = false;
      }
      break;
    case DP_SEQ_MEAN:
      if (!is_seq) { rc = DP_EINVAL; break; }
      if (i == 0 || (model->layers[i - 1].kind != DP_EMBEDDING && model->layers[i - 1].kind != DP_LSTM_SEQ)) { rc = DP_EUNSUPPORTED; break; }
      l.T = curC; l.Din = curH;
      l.outC = curH; l.outH = l.outW = 1;
      is_seq = false;
      break;
    default: rc = DP_EINVAL;
    }
    if (rc != DP_OK) break;
    l.in_size = (long)l.inC * l.inH * l.inW;
    l.out_size = (long)l.outC * l.outH * l.outW;
    if (l.d.kind == DP_CONV2D) {
      l.geom = make_geom(l);
      plan_direct_conv(l, max_batch, c->opt);
      const ConvGeom &g = l.geom;
      l.first_fwd = c->L.empty() && !l.wino_f && !c->opt.generic_conv && !c->opt.no_first_layer_kernel &&
                    conv_first_fits(g.C, g.H, g.W, g.D, g.KH, g.KW, g.S, g.PAD) && (long)max_batch * g.D * g.H * g.W < (1l << 31);
      // (the stored row keeps the accumulator order of the flattened direct kernel, which stays the fallback)
      l.first_wg = c->L.empty() && l.dir_wg && l.wg_flat && !c->opt.generic_conv && !c->opt.no_first_layer_kernel &&
                   conv_first_wgrad_fits(g.C, g.H, g.W, g.D, g.KH, g.KW, g.S, g.PAD);
      if (l.first_wg) l.max_slots = std::max(l.max_slots, 4); // its norm comes as one partial per wave
    }
    off += l.p_count;
    total_slots += l.max_slots;
    curC = l.outC; curH = l.outH; curW = l.outW;
    c->L.push_back(l);
  }
  if (rc == DP_OK) {
    const Layer &last = c->L.back();
    const bool logits_ok = (last.d.kind == DP_DENSE && last.d.act == DP_ACT_NONE) || last.d.kind == DP_AVGPOOL2D;
    if (is_tok || is_seq || last.out_size != model->n_classes || !logits_ok) rc = DP_EINVAL;
    int nparam = 0;
    for (auto &l : c->L) nparam += l.p_count > 0;
    if (nparam > DP_MAX_SEG) rc = DP_EUNSUPPORTED;
  }
  if (rc != DP_OK) { delete c; return rc; }
  {
    bool any = false;
    for (auto &l : c->L) any = any || l.lstm_wg;
    if (any && hipFuncSetAttribute((const void *)lstm_wgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)lstm_wgrad_lds_bytes()) != hipSuccess) {
      (void)hipGetLastError();
      for (auto &l : c->L) l.lstm_wg = false;
    }
  }
  {
    bool any_ws = false;
    for (auto &l : c->L) any_ws = any_ws || l.wg_ws;
    if (any_ws && !conv_wgrad_ws_enable()) { // large dynamic LDS refused: keep the single-buffer kernels
      (void)hipGetLastError();
      for (auto &l : c->L) l.wg_ws = false;
    }
  }
  c->P = off;
  c->max_slots = total_slots;
  c->fused1 = c->L.size() == 1 && c->L[0].d.kind == DP_DENSE && dense1_fits(c->L[0].d.in_features, c->L[0].d.out_features) &&
              !c->opt.no_fused_dense;
  {
    // the network cnn_small_fused_kernel is written for, layer by layer
    auto conv_is = [&](const Layer &l, int ci, int co, int k, int st, int pad) {
      return l.d.kind == DP_CONV2D && l.d.in_ch == ci && l.d.out_ch == co && l.d.kh == k && l.d.kw == k && l.d.stride == st && l.d.pad == pad;
    };
    auto pool_is = [&](const Layer &l) { return l.d.kind == DP_MAXPOOL2D && l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 1; };
    c->fusedcnn = c->L.size() == 6 && model->in_c == 1 && model->in_h == 28 && model->in_w == 28 && model->n_classes == 10 &&
                  conv_is(c->L[0], 1, 16, 8, 2, 3) && pool_is(c->L[1]) && conv_is(c->L[2], 16, 32, 4, 2, 0) && pool_is(c->L[3]) &&
                  c->L[4].d.kind == DP_DENSE && c->L[4].d.in_features == 512 && c->L[4].d.out_features == 32 &&
                  c->L[5].d.kind == DP_DENSE && c->L[5].d.in_features == 32 && c->L[5].d.out_features == 10 &&
                  c->L[5].d.act == DP_ACT_NONE && off == cnnf::NPARAM && !c->opt.no_fused_cnn;
    if (c->fusedcnn && hipFuncSetAttribute((const void *)cnn_small_fused_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)cnnf::LDS_BYTES) != hipSuccess) {
      (void)hipGetLastError();
      c->fusedcnn = false;
    }
  }
  {
    const size_t n = c->L.size();
    c->head2 = n >= 3 && c->L[n - 2].d.kind == DP_DENSE && c->L[n - 1].d.kind == DP_DENSE &&
               dense1_fits(c->L[n - 1].d.in_features, c->L[n - 1].d.out_features) && !c->fusedcnn && !c->opt.no_fused_dense;
  }
  c->fused2 = c->L.size() == 2 && c->L[0].d.kind == DP_DENSE && c->L[1].d.kind == DP_DENSE &&
              dense1_fits(c->L[1].d.in_features, c->L[1].d.out_features) && !c->opt.no_fused_dense;
  if ((c->fused2 || c->head2) && !c->opt.no_small_gemm && !dense_small_gemm_prepare()) { // its LDS size refused: the tiled contraction
    (void)hipGetLastError();
    c->opt.no_small_gemm = 1;
  }
  // both clipped sums of the two-layer network in one launch of that kernel (widths in whole groups of four floats)
  c->joint2 = c->fused2 && !c->opt.no_small_gemm && c->L[0].d.in_features % 4 == 0 && c->L[0].d.out_features % 4 == 0;
  if (c->head2 && !c->opt.no_small_gemm) { // the same for the two dense layers that close a deeper network
    const dp_layer_desc &h = c->L[c->L.size() - 2].d;
    c->joint2 = h.in_features % 4 == 0 && h.out_features % 4 == 0;
  }
  if (rc == DP_OK && !c->L.empty() && c->L[0].d.kind == DP_EMBEDDING && !c->opt.no_side_stream) {
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      if (c->side) { (void)hipStreamDestroy(c->side); c->side = nullptr; } // (the step then keeps everything on one stream)
    }
  }
  for (size_t i = 0; i < c->L.size(); ++i) {
    c->L[i].lab.reserve(sizeof(kLayerLabels) / sizeof(kLayerLabels[0]));
    for (const char *nm : kLayerLabels) c->L[i].lab.push_back(std::string(nm) + "#" + std::to_string(i));
  }
  const long mb = max_batch;
  for (auto &l : c->L) {
    if (rc != DP_OK) break;
    const bool emb = l.d.kind == DP_EMBEDDING;
    rc = dev_alloc(c, &l.a, mb * l.out_size); // embedding: the gathered rows x[B, T, D]
    if (rc == DP_OK) rc = dev_alloc(c, &l.g, mb * std::max<long>(l.out_size, &l == &c->L.back() ? 16 : 0)); // (the loss gradient: rows of up to 16 floats)
    if (rc == DP_OK && l.d.kind == DP_MAXPOOL2D) rc = dev_alloc(c, &l.arg, mb * l.out_size);
    if (rc == DP_OK && l.p_count > 0) {
      l.max_split = 1;
      if (!emb) {
        long ms = DP_MAX_PART_FLOATS / l.p_count;
        l.max_split = (int)(ms < 8 ? 8 : (ms > DP_MAX_SPLIT ? DP_MAX_SPLIT : ms));
      }
      l.pstride = (l.p_count + 3) & ~3l;
      rc = dev_alloc(c, &l.part, (size_t)l.max_split * l.pstride);
    }
    if (rc == DP_OK && l.d.kind == DP_DENSE) {
      // a small output with a long K would leave most CUs idle and expose every load's latency: split K
      GemmShape sh = pick_tile(max_batch, l.d.out_features, 1, c->opt.gemm_plain_tiles == 0);
      long tiles = (long)sh.tiles_m * sh.tiles_n;
      int by_k = l.d.in_features / 64;
      if (tiles < 512 && by_k >= 2) {
        long want = (1024 + tiles - 1) / tiles;
        l.fsplit = (int)(want < by_k ? want : by_k);
        if (l.fsplit > 64) l.fsplit = 64;
        rc = dev_alloc(c, &l.fpart, (size_t)l.fsplit * mb * l.out_size);
      }
    }
    if (rc == DP_OK && (l.dir_fwd || l.dir_bwd)) {
      // rows rounded up to whole chunks plus one spare chunk, and 128 spare floats: the kernels load weight
      // tiles without range tests and read this zero padding instead
      const size_t rf = (size_t)(ceil_div(l.geom.C, CONV_CC) + 1) * CONV_CC * 9, rb = (size_t)(ceil_div(l.geom.D, CONV_CC) + 1) * CONV_CC * 9;
      const size_t nf = rf * ((l.geom.D + 3) & ~3) + 128, nb = rb * ((l.geom.C + 3) & ~3) + 128;
      rc = dev_alloc(c, &l.wt_f, nf);
      if (rc == DP_OK) rc = dev_alloc(c, &l.wt_b, nb);
      if (rc == DP_OK && (hipMemsetAsync(l.wt_f, 0, nf * sizeof(float), c->stream) != hipSuccess ||
                          hipMemsetAsync(l.wt_b, 0, nb * sizeof(float), c->stream) != hipSuccess)) rc = DP_EHIP;
    }
    if (rc == DP_OK && l.wino_f) {
      l.uf_cpad = ceil_div(l.geom.C, WINO_CC) * WINO_CC; l.uf_mpad = ceil_div(l.geom.D, 32 * l.wino_f) * 32 * l.wino_f;
      const size_t n = (size_t)16 * l.uf_cpad * l.uf_mpad;
      rc = dev_alloc(c, &l.u_f, n);
      if (rc == DP_OK && hipMemsetAsync(l.u_f, 0, n * sizeof(float), c->stream) != hipSuccess) rc = DP_EHIP;
    }
    if (rc == DP_OK && l.wino_b && &l != &c->L.front()) {
      l.ub_cpad = ceil_div(l.geom.D, WINO_CC) * WINO_CC; l.ub_mpad = ceil_div(l.geom.C, 32 * l.wino_b) * 32 * l.wino_b;
      const size_t n = (size_t)16 * l.ub_cpad * l.ub_mpad;
      rc = dev_alloc(c, &l.u_b, n);
      if (rc == DP_OK && hipMemsetAsync(l.u_b, 0, n * sizeof(float), c->stream) != hipSuccess) rc = DP_EHIP;
    }
    // Strided convolutions (no direct kernel): backward-data as a plain per-example product into columns followed
    // by a gather over the windows, instead of a contraction whose Delta operand is gathered element by element
    // with most of the strided taps empty
    if (rc == DP_OK && l.d.kind == DP_CONV2D && !l.dir_bwd && l.geom.S > 1 && &l != &c->L.front() &&
        (size_t)mb * l.geom.CKK * l.geom.P <= ((size_t)1 << 28) && !c->opt.no_columns)
      rc = dev_alloc(c, &l.cols, (size_t)mb * l.geom.CKK * l.geom.P);
    // Large planes: the norm pass writes each example's gradient (8 bytes of traffic per coordinate, written and
    // read once) and the clipped sum becomes a weighted sum of those rows; repeating the contraction instead costs
    // 2 P flops per coordinate, which is more from P = 256 pixels on.
    if (rc == DP_OK && l.d.kind == DP_CONV2D && l.dir_wg && !l.gram && !l.wg_ws && l.geom.D <= DP_WG_DSLICE &&
        l.geom.P >= 256 && (size_t)mb * l.p_count <= ((size_t)1 << 30) && !c->opt.no_stored_gradients) {
      // the order in which conv_s1_wgrad_kernel<3, 3, wg_db, wg_flat, false> holds the gradient in its accumulators
      GradOrder &o = l.gorder;
      const ConvGeom &g = l.geom;
      // per-example contraction in the F(3x3, 2x2) form (conv_wino_wgrad_norm_kernel): whole blocks of 32 input
      // channels, 32 or 64 output channels, planes whose bands of 16 tiles the kernel is built for; its rows are in
      // the parameter layout
      l.wino_norm = l.wino_wgu;
      if (l.wino_norm) {
        o = GradOrder{};
        o.C = g.C; o.D = g.D; o.KK = 9; o.flat = 2;
        o.n_total = l.p_count;
      } else {
      o.C = l.geom.C; o.D = l.geom.D; o.KK = 9; o.flat = l.wg_flat ? 1 : 0;
      o.WN = l.wg_flat ? 1 : 2;                       // wg_db is 1 or 2 here
      o.NW = l.wg_flat ? 1 : (l.wg_db == 1 ? 2 : 4);
      o.NBW = l.wg_flat ? 1 : 5;
      const long cblocks = l.wg_flat ? 1 : ceil_div(l.geom.C, 32);
      o.n_w = cblocks * o.NW * o.NBW * 1024;
      o.n_total = o.n_w + o.D;
      }
      rc = dev_alloc(c, &l.gst, (size_t)mb * o.n_total);
    }
    // the same route for convolutions on the generic contraction (other strides / filter sizes): its per-example
    // tile is [D][C*KK + 1], the last column being the bias gradient
    if (rc == DP_OK && l.d.kind == DP_CONV2D && !l.dir_wg && !l.gram && l.geom.P >= 128 &&
        (size_t)mb * l.p_count <= ((size_t)1 << 30) && !c->opt.no_stored_gradients) {
      GradOrder &o = l.gorder;
      o = GradOrder{};
      o.C = l.geom.C; o.D = l.geom.D; o.KK = l.geom.KH * l.geom.KW; o.flat = 3;
      o.n_total = (long)o.D * (o.C * o.KK + 1);
      rc = dev_alloc(c, &l.gst, (size_t)mb * o.n_total);
    }
    if (rc == DP_OK && emb) {
      const size_t V = l.d.vocab;
      rc = dev_alloc(c, &l.e_count, V + 1);
      if (rc == DP_OK) rc = dev_alloc(c, &l.e_start, V + 1);
      if (rc == DP_OK) rc = dev_alloc(c, &l.e_chunk0, V + 1);
      if (rc == DP_OK) rc = dev_alloc(c, &l.e_cursor, V + 1);
      if (rc == DP_OK) rc = dev_alloc(c, &l.e_list, (size_t)mb * l.outC);
    }
    if (rc == DP_OK && (l.d.kind == DP_LSTM_LAST || l.d.kind == DP_LSTM_SEQ)) {
      rc = dev_alloc(c, &l.gates, mb * l.T * 4 * l.H);
      if (rc == DP_OK) rc = dev_alloc(c, &l.cs, mb * l.T * l.H);
      if (l.d.kind == DP_LSTM_SEQ) l.hs = l.a; // the hidden states are the layer's output
      else if (rc == DP_OK) rc = dev_alloc(c, &l.hs, mb * l.T * l.H);
      // long sequences: the norm contraction writes each example's gradient ([Din + H + 1][4H], which is the layer's
      // parameter layout) and the clipped sum is a weighted sum of those rows: 8 bytes of traffic per coordinate
      // against the 2 T flops of contracting it again
      if (rc == DP_OK && l.T >= 128 && (size_t)mb * l.p_count <= ((size_t)1 << 30) && !c->opt.no_stored_gradients) {
        l.gorder = GradOrder{};
        l.gorder.flat = 2; l.gorder.n_total = l.p_count;
        rc = dev_alloc(c, &l.gst, (size_t)mb * l.p_count);
      }
    }
  }
  if (rc == DP_OK) rc = dev_alloc(c, &c->slots, (size_t)c->max_slots * mb);
  if (rc == DP_OK) rc = dev_alloc(c, &c->norms, mb);
  if (rc == DP_OK) rc = dev_alloc(c, &c->s, mb);
  if (rc == DP_OK) rc = dev_alloc(c, &c->ones, mb);
  if (rc == DP_OK) rc = dev_alloc(c, &c->bad, 1);
  if (rc == DP_OK && c->fusedcnn) rc = dev_alloc(c, &c->cnn_part, (size_t)256 * ((cnnf::NPARAM + 3) & ~3));
  if (rc == DP_OK) {
    std::vector<float> one(mb, 1.f);
    if (hipMemcpy(c->ones, one.data(), sizeof(float) * mb, hipMemcpyHostToDevice) != hipSuccess) rc = DP_EHIP;
  }
  // the zero fills above were enqueued on the context's stream (which need not be ordered against the null
  // stream): they are complete before the first step can be enqueued
  if (rc == DP_OK && hipStreamSynchronize(c->stream) != hipSuccess) rc = DP_EHIP;
  if (rc != DP_OK) { dp_step_free(c); return rc; }
  *out = c;
  return DP_OK;
}

extern "C" void dp_step_free(dp_ctx *c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  for (void *p : c->allocs) (void)hipFree(p);
  for (hipEvent_t e : c->pool) (void)hipEventDestroy(e);
  delete c;
}

extern "C" size_t dp_step_num_params(const dp_ctx *c) { return c ? (size_t)c->P : 0; }
extern "C" size_t dp_step_workspace_bytes(const dp_ctx *c) { return c ? c->ws_bytes : 0; }

extern "C" const char *dp_step_strerror(int code) {
  switch (code) {
  case DP_OK: return "ok";
  case DP_EINVAL: return "invalid argument";
  case DP_ENOMEM: return g_hip_err[0] ? g_hip_err : "out of device memory";
  case DP_EHIP: return g_hip_err[0] ? g_hip_err : "HIP runtime error";
  case DP_EUNSUPPORTED: return "layer sequence or size not supported by the kernels";
  case DP_ETOOBIG: return "sizes beyond the limits of the allocation-free entry point (in_features <= 1023, n_classes <= 15, "
                          "in_features * (n_classes rounded up to 4, 10 or 15, + 4) <= 14800, batch <= 65536)";
  default: return "unknown status";
  }
}

// ---------------------------------------------------------------- the step

static inline dim3 grid1d(long n, int block) { return dim3((unsigned)((n + block - 1) / block)); }

template <int HP>
static void launch_lstm_fwd(const Launcher &Ln, Layer &l, const float *Whh, int B, const char *label) {
  dim3 grid(B), block(LSTM_THREADS);
  Ln(label, grid, block, [&](hipStream_t st) {
    hipLaunchKernelGGL(lstm_fwd_kernel<HP>, grid, block, 0, st, l.gates, Whh, l.hs, l.cs,
                       l.d.kind == DP_LSTM_SEQ ? (float *)nullptr : l.a, B, l.T, l.H);
  });
}
template <int HP>
static void launch_lstm_bwd(const Launcher &Ln, Layer &l, const float *Whh, int B, const char *label) {
  dim3 grid(B), block(LSTM_THREADS);
  Ln(label, grid, block, [&](hipStream_t st) {
    if (l.d.kind == DP_LSTM_SEQ)
      hipLaunchKernelGGL((lstm_bwd_kernel<HP, true>), grid, block, 0, st, l.gates, (const float *)l.cs, Whh, (const float *)l.g, B, l.T, l.H);
    else
      hipLaunchKernelGGL((lstm_bwd_kernel<HP, false>), grid, block, 0, st, l.gates, (const float *)l.cs, Whh, (const float *)l.g, B, l.T, l.H);
  });
}
#define LSTM_DISPATCH(fn, H, ...)                 \
  do {                                            \
    if ((H) <= 4) fn<4>(__VA_ARGS__);             \
    else if ((H) <= 8) fn<8>(__VA_ARGS__);        \
    else if ((H) <= 16) fn<16>(__VA_ARGS__);      \
    else if ((H) <= 32) fn<32>(__VA_ARGS__);      \
    else if ((H) <= 64) fn<64>(__VA_ARGS__);      \
    else if ((H) <= 100) fn<100>(__VA_ARGS__);    \
    else fn<128>(__VA_ARGS__);                    \
  } while (0)

#define LL(name) layer_label(l, i, name)
// runs body(tag) with tag = std::true_type when the operands can be staged as float4, else std::false_type
template <class F>
static inline void vec_dispatch(bool cond, F &&body) {
  if (cond) body(std::true_type{});
  else body(std::false_type{});
}
static int run_step(dp_ctx *c, const float *params, const void *x, const int32_t *y, int B, bool priv, float C,
                    float sigma, uint64_t seed, float *out, float *theta_update = nullptr, float update_step = 0.f) {
  Launcher Ln{c};
  const int nL = (int)c->L.size();
  const long slot_stride = c->maxB;
  int slot_next = 0;
  FinalizeArgs fa;
  fa.nseg = 0;

  // the network ends in a dense layer of at most 64 classes: its bias, the loss gradient and its norm share a launch
  const bool fused_head = c->L[nL - 1].d.kind == DP_DENSE && c->L[nL - 1].d.out_features <= 64;
  int head_ns = 0; // forward split-K partials of the last layer still to be summed (0: its output is complete)
  if (B > 0 && c->fusedcnn && aligned16(params)) {
    // the small CNN: forward, backward, every example's gradient, norm, clip factor and the partial clipped sums in
    // one launch; a workgroup walks through its examples
    CnnFusedArgs a{};
    a.params = params; a.x = (const float *)x; a.y = (const int *)y; a.part = c->cnn_part; a.pstride = (cnnf::NPARAM + 3) & ~3;
    a.norms = priv ? c->norms : nullptr; a.s = priv ? c->s : nullptr; a.B = B;
    a.act1 = c->L[0].d.act; a.act2 = c->L[2].d.act; a.act3 = c->L[4].d.act; a.C = C; a.priv = priv ? 1 : 0;
    const int tiles = std::min(B, 256);
    Ln("cnn_small_fused", dim3(tiles), dim3(cnnf::THREADS), [&](hipStream_t st) {
      hipLaunchKernelGGL(cnn_small_fused_kernel, dim3(tiles), dim3(cnnf::THREADS), cnnf::LDS_BYTES, st, a);
    });
    for (auto &l : c->L) {
      if (l.p_count == 0) continue;
      FinalizeSeg &sg = fa.seg[fa.nseg++];
      sg.p_off = l.p_off; sg.n = l.p_count; sg.part = c->cnn_part + l.p_off; sg.stride = a.pstride; sg.nsplit = tiles;
    }
  } else if (B > 0 && c->fused1) {
    // softmax regression: logits, loss gradient, norm, clip factor and the clipped partial sums in one launch
    Layer &l = c->L[0];
    Dense1Args a{};
    a.x = (const float *)x; a.W = params; a.bias = params + (long)l.d.in_features * l.d.out_features; a.y = (const int *)y;
    a.part = l.part; a.norms = priv ? c->norms : nullptr; a.s = priv ? c->s : nullptr; a.delta = nullptr;
    a.B = B; a.d_in = l.d.in_features; a.N = l.d.out_features; a.C = C; a.priv = priv ? 1 : 0;
    int tiles = 0;
    Ln("dense1_fused", dim3(1), dim3(256), [&](hipStream_t st) {
      tiles = launch_dense1_fused(st, a, std::min<long>(DENSE1_MAX_TILES, (long)l.max_split));
    });
    FinalizeSeg &sg = fa.seg[fa.nseg++];
    sg.p_off = 0; sg.n = l.p_count; sg.part = l.part; sg.stride = dense1_part_stride(a.d_in, a.N); sg.nsplit = tiles;
  } else if (B > 0) {
    // The embedding layer's token lists for its clipped sum (a counting sort of the batch by token id) and its zeroed
    // partial: inputs of emb_reduce_kernel that depend on x alone.
    auto emb_prepare = [&](Layer &l, int i, auto &&launch) {
      const long rows = (long)B * l.outC;
      const int V = l.d.vocab;
      (void)i;
        {
          dim3 grid = grid1d(l.p_count + V + 1, 256), block(256);
          launch(LL("fill_zero"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(fill_zero_kernel, grid, block, 0, st, l.part, l.p_count, (float *)l.e_count, (long)(V + 1));
          });
        }
        if (V <= EMB_LDS_V && rows <= EMB_ONE_MAX_ROWS && !c->opt.no_single_bucket) {
          launch(LL("emb_bucket"), dim3(1), dim3(1024), [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_bucket_one_kernel, dim3(1), dim3(1024), sizeof(int) * V, st, (const int *)x, l.e_start,
                               l.e_chunk0, l.e_list, (int)rows, V);
          });
        } else {
          dim3 grid = grid1d(rows, 1024), block(1024);
          const size_t smem = V <= EMB_LDS_V ? sizeof(int) * V : 0;
          launch(LL("emb_bucket"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_count_kernel, grid, block, smem, st, (const int *)x, l.e_count, rows, V);
          });
          launch(LL("emb_bucket"), dim3(1), dim3(1024), [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_scan_kernel, dim3(1), dim3(1024), 0, st, (const int *)l.e_count, l.e_start,
                               l.e_chunk0, l.e_cursor, V);
          });
          launch(LL("emb_bucket"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_fill_kernel, grid, block, smem, st, (const int *)x, (const int *)l.e_start,
                               l.e_cursor, l.e_list, rows, V);
          });
        }
    };
    bool emb_early = false;
    // The token lists are built on the library's second stream from the start of the step (measured: forked here the
    // embedding network's step is 12 us shorter; forked at the start of the backward pass it is not, and the LSTM
    // network gains the same 15 us either way -- the sort's launches slow the launches they run beside, and each event
    // wait costs the waiting stream about 6 us).
    if (c->side && !c->prof && c->L[0].d.kind == DP_EMBEDDING && c->L[0].p_count > 0) {
      auto on_side = [&](const char *, dim3, dim3, auto &&f) { f(c->side); };
      (void)hipEventRecord(c->ev_fork, c->stream);
      (void)hipStreamWaitEvent(c->side, c->ev_fork, 0);
      emb_prepare(c->L[0], 0, on_side);
      (void)hipEventRecord(c->ev_join, c->side);
      emb_early = true;
    }
    // ------------------------------------------------------------ re-laid weights of the direct convolutions and
    // transformed weights of the minimal-filtering kernels: one launch for both (two where a table overflows)
    {
      ConvLayoutArgs la{};
      WinoLayoutArgs wa{};
      int big_l = 0, big_w = 0;
      auto flush = [&]() {
        if (la.n == 0 && wa.n == 0) return;
        const int biggest = std::max(big_l, big_w);
        dim3 grid((unsigned)std::min(64, ceil_div(biggest, 256)), la.n + wa.n), block(256);
        Ln("conv_weight_layout", grid, block, [&](hipStream_t st) {
          hipLaunchKernelGGL(conv_weights_kernel, grid, block, 0, st, params, la, wa);
        });
        la.n = 0; wa.n = 0; big_l = 0; big_w = 0;
      };
      for (int i = 0; i < nL; ++i) {
        Layer &l = c->L[i];
        if (l.d.kind != DP_CONV2D) continue;
        const ConvGeom &g = l.geom;
        if (l.dir_fwd || l.dir_bwd) {
          // only the layouts a direct kernel of this step reads (the minimal-filtering kernels have their own)
          float *need_f = (l.dir_fwd && !l.u_f && !l.first_fwd) ? l.wt_f : nullptr;
          float *need_b = (l.dir_bwd && !l.u_b && i > 0) ? l.wt_b : nullptr;
          if (need_f || need_b) {
            auto &e = la.l[la.n++];
            e.w_off = l.p_off; e.wt_f = need_f; e.wt_b = need_b; e.D = g.D; e.C = g.C;
            e.Dp = (g.D + 3) & ~3; e.Cp = (g.C + 3) & ~3;
            big_l = std::max(big_l, g.D * g.CKK);
          }
        }
        if (l.u_f || l.u_b) {
          auto &e = wa.l[wa.n++];
          e.w_off = l.p_off; e.uf = l.u_f; e.ub = l.u_b; e.D = g.D; e.C = g.C;
          e.Cfp = l.uf_cpad; e.Dfp = l.uf_mpad; e.Dbp = l.ub_cpad; e.Cbp = l.ub_mpad;
          big_w = std::max(big_w, g.D * g.C);
        }
        if (la.n == CONV_LAYOUT_MAX || wa.n == 16) flush();
      }
      flush();
    }
    // ------------------------------------------------------------ forward
    const float *in = (const float *)x;
    int fused_pool = -1;
    const bool no_pool_fusion = c->opt.no_pool_fusion != 0;
    const bool f2 = c->fused2, h2 = c->head2;
    int mid_ns = 0, mid_tiles = 0;
    SmallGemmArgs joint_g[2] = {};
    bool joint = false;
    for (int i = 0; i < nL; ++i) {
      if ((f2 && i == 1) || (h2 && i == nL - 1)) break; // the logits are computed by the kernel that follows the hidden layer
      Layer &l = c->L[i];
      const float *W = params + l.p_off;
      switch (l.d.kind) {
      case DP_DENSE: {
        if ((f2 || (h2 && i == nL - 2)) && !c->opt.no_small_gemm) {
          // the hidden layer's forward product, complete (bias and activation applied): K split inside the workgroup
          SmallGemmArgs g{};
          g.A = in; g.a_sr = l.d.in_features; g.a_sk = 1;
          g.B = W; g.b_sr = 1; g.b_sk = l.d.out_features;
          g.bias = W + (long)l.d.in_features * l.d.out_features; g.act = l.d.act;
          g.C = l.a; g.c_sm = l.d.out_features; g.c_sn = 1; g.C_ones = nullptr;
          g.M = B; g.N = l.d.out_features; g.K = l.d.in_features; g.a_ones = 0;
          if (dense_small_gemm_fits(g)) {
            Ln(LL("dense_fwd"), dim3(1), dim3(256), [&](hipStream_t st) { launch_dense_small_gemm(st, g); });
            break;
          }
        }
        if (l.fsplit > 1) {
          const long stride = (long)c->maxB * l.out_size;
          int ns = 1;
          auto run = [&](auto vt) {
            constexpr bool V = decltype(vt)::value;
            typedef ProbPartial<OpRowMajor<V>, OpKMajor<V, false>> Pb;
            Pb p{};
            p.M = B; p.N = l.d.out_features; p.K = l.d.in_features;
            p.a.set(in, l.d.in_features);
            p.b.set(W, l.d.out_features);
            p.part = l.fpart; p.stride = stride; p.ldm = l.d.out_features; p.bias_col = -1; p.bias_off = 0;
            ns = launch_gemm_split(p, l.fsplit, Ln, LL("dense_fwd"));
          };
          vec_dispatch(OpRowMajor<true>::can_vec(in, l.d.in_features, 0, l.d.in_features) &&
                              OpKMajor<true, false>::can_vec(W, l.d.out_features, 0, l.d.out_features), run);
          if (i == nL - 1 && fused_head) { head_ns = ns; break; } // bias + loss gradient + norm in one launch below
          if (f2 || (h2 && i == nL - 2)) { mid_ns = ns; break; }  // bias + activation where the partials are consumed
          const long total = (long)B * l.out_size;
          dim3 grid = grid1d(total, 256), block(256);
          const float *bias = W + (long)l.d.in_features * l.d.out_features;
          Ln(LL("dense_fwd_epilogue"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(bias_act_reduce_kernel, grid, block, 0, st, (const float *)l.fpart, ns, stride, bias,
                               l.d.act, l.a, total, l.d.out_features);
          });
          break;
        }
        auto run = [&](auto vt) {
          constexpr bool V = decltype(vt)::value;
          typedef ProbBiasAct<OpRowMajor<V>, OpKMajor<V, false>> Pb;
          Pb p{};
          p.M = B; p.N = l.d.out_features; p.K = l.d.in_features;
          p.a.set(in, l.d.in_features);
          p.b.set(W, l.d.out_features);
          p.out = l.a; p.bias = W + (long)l.d.in_features * l.d.out_features; p.ld = l.d.out_features; p.act = l.d.act;
          launch_gemm(p, 1, Ln, LL("dense_fwd"));
        };
        vec_dispatch(OpRowMajor<true>::can_vec(in, l.d.in_features, 0, l.d.in_features) &&
                            OpKMajor<true, false>::can_vec(W, l.d.out_features, 0, l.d.out_features), run);
      } break;
      case DP_CONV2D: {
        if (l.u_f) {
          const ConvGeom &g = l.geom;
          ConvWinoArgs a{};
          a.x = in; a.u = l.u_f; a.bias = W + (long)g.D * g.CKK; a.a_prev = nullptr; a.out = l.a;
          a.B = B; a.Cin = g.C; a.Cpad = l.uf_cpad; a.H = g.H; a.W = g.W; a.M = g.D; a.Mpad = l.uf_mpad; a.act = l.d.act;
          // a 2x2 / stride-2 pool right after the layer: one tile of the kernel is one pool window
          if (i + 1 < nL && (c->L[i + 1].d.kind == DP_MAXPOOL2D || c->L[i + 1].d.kind == DP_AVGPOOL2D) &&
              c->L[i + 1].d.kh == 2 && c->L[i + 1].d.kw == 2 && c->L[i + 1].d.stride == 2 && !no_pool_fusion) {
            a.pool = c->L[i + 1].d.kind == DP_MAXPOOL2D ? 1 : 2;
            a.pool_out = c->L[i + 1].a; a.pool_arg = c->L[i + 1].arg;
            fused_pool = i + 1;
          }
          launch_conv_wino(Ln, LL("conv_fwd"), a, l.wino_f);
          break;
        }
        if (l.first_fwd) {
          // an RGB first layer: persistent workgroups, weights in registers, the next tile's loads under the current stores
          const ConvGeom &g = l.geom;
          ConvFirstArgs a{};
          a.x = in; a.w = W; a.bias = W + (long)g.D * g.CKK; a.out = l.a;
          a.B = B; a.Cin = g.C; a.H = g.H; a.M = g.D; a.act = l.d.act;
          a.n_tiles = B * (g.H / CF_TR);
          a.tiles_per_wg = ceil_div(a.n_tiles, 1024);
          dim3 grid(ceil_div(a.n_tiles, a.tiles_per_wg)), block(256);
          Ln(LL("conv_fwd"), grid, block, [&](hipStream_t st) {
#define DP_CF_CASE(full_, act_)                                                                                   \
  if ((g.D == 32) == full_ && a.act == act_) hipLaunchKernelGGL((conv_first_kernel<full_, act_>), grid, block, 0, st, a);
            DP_CF_CASE(true, DP_ACT_NONE) DP_CF_CASE(true, DP_ACT_RELU) DP_CF_CASE(true, DP_ACT_TANH)
            DP_CF_CASE(false, DP_ACT_NONE) DP_CF_CASE(false, DP_ACT_RELU) DP_CF_CASE(false, DP_ACT_TANH)
#undef DP_CF_CASE
          });
          break;
        }
        if (l.dir_fwd) {
          const ConvGeom &g = l.geom;
          ConvS1Args a{};
          a.x = in; a.wt = l.wt_f; a.bias = W + (long)g.D * g.CKK; a.a_prev = nullptr; a.out = l.a;
          a.B = B; a.Cin = g.C; a.H = g.H; a.W = g.W; a.M = g.D; a.Mpad = (g.D + 3) & ~3; a.OH = g.OH; a.OW = g.OW; a.pad = g.PAD;
          a.act = l.d.act; a.t = l.t_fwd;
          launch_conv_s1(Ln, LL("conv_fwd"), a, l.fwd_npw);
          break;
        }
        const ConvGeom &g = l.geom;
        auto run = [&](auto vt) {
          constexpr bool V = decltype(vt)::value;
          typedef ProbConvFwd<OpRowMajor<V>, OpConvPatch<true>> Pb;
          Pb p{};
          p.M = g.D; p.N = B * g.P; p.K = g.CKK;
          p.a.set(W, g.CKK);
          p.b.x = in; p.b.g = g; p.b.has_ones = 0; p.b.by_z = 0;
          p.out = l.a; p.bias = W + (long)g.D * g.CKK; p.D = g.D; p.P = g.P; p.act = l.d.act; p.dP = g.dP;
          launch_gemm(p, 1, Ln, LL("conv_fwd"));
        };
        vec_dispatch(OpRowMajor<true>::can_vec(W, g.CKK, 0, g.CKK), run);
      } break;
      case DP_MAXPOOL2D: {
        if (i == fused_pool) break; // taken in the epilogue of the convolution before it
        long total = (long)B * l.out_size;
        dim3 grid = grid1d(total, 256), block(256);
        const bool p22 = l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 2 && (l.inH & 1) == 0 && (l.inW & 1) == 0;
        if (p22) {
          Ln(LL("maxpool_fwd"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(maxpool2x2_fwd_kernel, grid, block, 0, st, in, l.a, l.arg, total, l.outW, l.inW);
          });
        } else
        Ln(LL("maxpool_fwd"), grid, block, [&](hipStream_t st) {
          Split3 dv; dv.dX.init(l.outW); dv.dY.init(l.outH);
          if (l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 1)
            hipLaunchKernelGGL((maxpool_fwd_kernel<2, 1>), grid, block, 0, st, in, l.a, l.arg, total, l.inH, l.inW, l.outH,
                               l.outW, l.d.kh, l.d.kw, l.d.stride, dv);
          else
            hipLaunchKernelGGL((maxpool_fwd_kernel<0, 0>), grid, block, 0, st, in, l.a, l.arg, total, l.inH, l.inW, l.outH,
                               l.outW, l.d.kh, l.d.kw, l.d.stride, dv);
        });
      } break;
      case DP_EMBEDDING: {
        const long n = (long)B * l.out_size;
        if ((l.d.embed_dim & 3) == 0 && aligned16(W) && aligned16(l.a)) {
          dim3 grid = grid1d(n / 4, 256), block(256);
          Ln(LL("emb_gather"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_gather4_kernel, grid, block, 0, st, (const int *)x, (const float4 *)W, (float4 *)l.a,
                               (long)B * l.outC, l.d.embed_dim / 4);
          });
        } else {
          dim3 grid = grid1d(n, 256), block(256);
          Ln(LL("emb_gather"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_gather_kernel, grid, block, 0, st, (const int *)x, W, l.a, (long)B * l.outC,
                               l.d.embed_dim);
          });
        }
      } break;
      case DP_SEQ_MEAN: {
        dim3 grid(B), block(256);
        Ln(LL("seq_mean_fwd"), grid, block, [&](hipStream_t st) {
          hipLaunchKernelGGL(seq_mean_fwd_kernel, grid, block, 0, st, in, l.a, l.T, l.Din);
        });
      } break;
      case DP_AVGPOOL2D: {
        if (i == fused_pool) break; // taken in the epilogue of the convolution before it
        long total = (long)B * l.out_size;
        dim3 grid = grid1d(total, 256), block(256);
        const bool p22 = l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 2 && (l.inH & 1) == 0 && (l.inW & 1) == 0;
        if (p22) {
          Ln(LL("avgpool_fwd"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(avgpool2x2_fwd_kernel, grid, block, 0, st, in, l.a, total, l.outW, l.inW);
          });
        } else
        Ln(LL("avgpool_fwd"), grid, block, [&](hipStream_t st) {
          Split3 dv; dv.dX.init(l.outW); dv.dY.init(l.outH);
          hipLaunchKernelGGL(avgpool_fwd_kernel, grid, block, 0, st, in, l.a, total, l.inH, l.inW, l.outH, l.outW,
                             l.d.kh, l.d.kw, l.d.stride, dv);
        });
      } break;
      case DP_LSTM_LAST:
      case DP_LSTM_SEQ: {
        const int G = 4 * l.H;
        if (rows_gemm_fits(l.Din, G, 4, 1) && aligned16(in) && !c->opt.no_rows_gemm) {
          // gates = x W_ih + b with W_ih held in registers by persistent workgroups
          RowsGemmArgs a{};
          a.A = in; a.W = W; a.w_sk = G; a.w_sn = 1; a.bias = W + (long)l.Din * G + (long)l.H * G; a.C = l.gates;
          a.M = (long)B * l.T; a.K = l.Din; a.N = G;
          const long tiles = (a.M + 31) / 32;
          dim3 grid((unsigned)std::min<long>(tiles, 256)), block(RG_THREADS);
          Ln(LL("lstm_xproj"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL((rows_gemm_kernel<4, 1, 2>), grid, block, rows_gemm_lds_bytes(2), st, a);
          });
        } else {
        auto run = [&](auto vt) {
          constexpr bool V = decltype(vt)::value;
          typedef ProbBiasAct<OpRowMajor<V>, OpKMajor<V, false>> Pb;
          Pb p{};
          p.M = B * l.T; p.N = G; p.K = l.Din;
          p.a.set(in, l.Din);
          p.b.set(W, G);
          p.out = l.gates; p.bias = W + (long)l.Din * G + (long)l.H * G; p.ld = G; p.act = DP_ACT_NONE;
          launch_gemm(p, 1, Ln, LL("lstm_xproj"));
        };
        vec_dispatch(OpRowMajor<true>::can_vec(in, l.Din, 0, l.Din) && OpKMajor<true, false>::can_vec(W, G, 0, G), run);
        }
        const float *Whh = W + (long)l.Din * G;
        LSTM_DISPATCH(launch_lstm_fwd, l.H, Ln, l, Whh, B, LL("lstm_fwd"));
      } break;
      }
      in = l.a;
    }
    if (f2) {
      // two dense layers: logits, loss gradient, both layers' norms, the clip factor, s * delta of the hidden layer and
      // the partial clipped sums of the logit layer, all per example, in one launch
      Layer &l0 = c->L[0], &l1 = c->L[1];
      Dense2Args a{};
      a.x = (const float *)x; a.hpart = mid_ns > 0 ? l0.fpart : l0.a; a.hstride = (long)c->maxB * l0.out_size; a.ns = mid_ns;
      a.b1 = params + l0.p_off + (long)l0.d.in_features * l0.d.out_features;
      a.W2 = params + l1.p_off; a.b2 = a.W2 + (long)l1.d.in_features * l1.d.out_features; a.y = (const int *)y;
      a.sdelta1 = l0.g; a.part2 = l1.part; a.norms = priv ? c->norms : nullptr; a.s = priv ? c->s : nullptr;
      a.B = B; a.d_in = l0.d.in_features; a.H = l1.d.in_features; a.N = l1.d.out_features; a.act = l0.d.act;
      a.C = C; a.priv = priv ? 1 : 0;
      if (c->joint2 && mid_ns == 0) {
        // X^T (s Delta1) and a1^T (s Delta2), each with the column sums of its s Delta (the row of ones): complete in
        // one partial row, K (= the batch) split inside the workgroup
        SmallGemmArgs &g0 = joint_g[0], &g1 = joint_g[1];
        g0.A = (const float *)x; g0.a_sr = 1; g0.a_sk = l0.d.in_features; g0.a_ones = 1;
        g0.B = l0.g; g0.b_sr = 1; g0.b_sk = l0.d.out_features;
        g0.C = l0.part; g0.c_sm = l0.d.out_features; g0.c_sn = 1; g0.C_ones = l0.part + (long)l0.d.in_features * l0.d.out_features;
        g0.M = l0.d.in_features; g0.N = l0.d.out_features; g0.K = B; g0.act = DP_ACT_NONE;
        g1.A = l0.a; g1.a_sr = 1; g1.a_sk = l1.d.in_features; g1.a_ones = 1;
        g1.B = l1.g; g1.b_sr = 1; g1.b_sk = 16;
        g1.C = l1.part; g1.c_sm = l1.d.out_features; g1.c_sn = 1; g1.C_ones = l1.part + (long)l1.d.in_features * l1.d.out_features;
        g1.M = l1.d.in_features; g1.N = l1.d.out_features; g1.K = B; g1.act = DP_ACT_NONE;
        joint = dense_small_gemm_fits(g0) && dense_small_gemm_fits(g1);
        if (joint) { a.head = 2; a.delta2_out = l1.g; a.part2 = nullptr; }
      }
      Ln("dense2_mid", dim3(1), dim3(256), [&](hipStream_t st) {
        mid_tiles = launch_dense2_mid(st, a, std::min(DENSE1_MAX_TILES, l1.max_split));
      });
    }
    if (h2) {
      // a deeper network that ends in two dense layers: logits, loss gradient, both layers' norms and the hidden layer's
      // backprop, per example, in one launch (the clip factors need the other layers' norms and come later)
      Layer &l0 = c->L[nL - 2], &l1 = c->L[nL - 1];
      Dense2Args a{};
      a.x = nL > 2 ? (const float *)c->L[nL - 3].a : (const float *)x;
      a.hpart = mid_ns > 0 ? l0.fpart : l0.a; a.hstride = (long)c->maxB * l0.out_size; a.ns = mid_ns;
      a.b1 = params + l0.p_off + (long)l0.d.in_features * l0.d.out_features;
      a.W2 = params + l1.p_off; a.b2 = a.W2 + (long)l1.d.in_features * l1.d.out_features; a.y = (const int *)y;
      a.sdelta1 = l0.g; a.part2 = nullptr; a.norms = nullptr; a.s = nullptr;
      a.B = B; a.d_in = l0.d.in_features; a.H = l1.d.in_features; a.N = l1.d.out_features; a.act = l0.d.act;
      a.C = C; a.priv = priv ? 1 : 0;
      a.head = 1; a.a1_out = mid_ns > 0 ? l0.a : nullptr; a.delta2_out = l1.g; a.d2_ld = a.N;
      if (c->joint2 && mid_ns == 0) {
        // both layers' clipped sums in one launch later on (delta1, delta2 scaled by the clip factors as they are staged)
        SmallGemmArgs &g0 = joint_g[0], &g1 = joint_g[1];
        g0.A = a.x; g0.a_sr = 1; g0.a_sk = l0.d.in_features; g0.a_ones = 1;
        g0.B = l0.g; g0.b_sr = 1; g0.b_sk = l0.d.out_features;
        g0.C = l0.part; g0.c_sm = l0.d.out_features; g0.c_sn = 1; g0.C_ones = l0.part + (long)l0.d.in_features * l0.d.out_features;
        g0.M = l0.d.in_features; g0.N = l0.d.out_features; g0.K = B; g0.act = DP_ACT_NONE;
        g1.A = l0.a; g1.a_sr = 1; g1.a_sk = l1.d.in_features; g1.a_ones = 1;
        g1.B = l1.g; g1.b_sr = 1; g1.b_sk = 16;
        g1.C = l1.part; g1.c_sm = l1.d.out_features; g1.c_sn = 1; g1.C_ones = l1.part + (long)l1.d.in_features * l1.d.out_features;
        g1.M = l1.d.in_features; g1.N = l1.d.out_features; g1.K = B; g1.act = DP_ACT_NONE;
        joint = dense_small_gemm_fits(g0) && dense_small_gemm_fits(g1);
        if (joint) a.d2_ld = 16;
      }
      if (priv) {
        a.slot2 = c->slots + (long)slot_next * slot_stride;
        a.slot1 = c->slots + (long)(slot_next + 1) * slot_stride;
        slot_next += 2;
      }
      Ln("dense2_head", dim3(1), dim3(256), [&](hipStream_t st) { (void)launch_dense2_mid(st, a, DENSE1_MAX_TILES); });
    }
    // ------------------------------------------------------------ loss gradient
    if (f2 || h2) {
    } else if (fused_head) {
      // the last dense layer's bias, the loss gradient and that layer's norm (the first slot of the backward
      // pass) in one launch, one wave per example
      Layer &l = c->L[nL - 1];
      const float *Wl = params + l.p_off;
      const float *lin = nL > 1 ? c->L[nL - 2].a : (const float *)x;
      float *slot = priv ? c->slots + (long)slot_next * slot_stride : nullptr;
      if (priv) slot_next += 1;
      const bool single_layer = priv && nL == 1; // this slot is the whole norm: the clip factors come along
      dim3 grid = grid1d((long)B * 64, 256), block(256);
      Ln("logits_loss_norm", grid, block, [&](hipStream_t st) {
        hipLaunchKernelGGL(logits_loss_norm_kernel, grid, block, 0, st,
                           head_ns > 0 ? (const float *)l.fpart : (const float *)nullptr, head_ns,
                           (long)c->maxB * l.out_size, Wl + (long)l.d.in_features * l.d.out_features, (const int *)y, lin,
                           l.d.in_features, l.a, l.g, slot, single_layer ? c->norms : (float *)nullptr,
                           single_layer ? c->s : (float *)nullptr, C, B, l.d.out_features);
      });
    } else {
      Layer &l = c->L[nL - 1];
      dim3 grid = grid1d(B, 128), block(128);
      Ln("softmax_xent_grad", grid, block, [&](hipStream_t st) {
        hipLaunchKernelGGL(softmax_xent_grad_kernel, grid, block, 0, st, (const float *)l.a, (const int *)y, l.g, B,
                           c->m.n_classes);
      });
    }
    // ------------------------------------------------------------ backward: data gradients and per-example norms
    for (int i = f2 ? -1 : (h2 ? nL - 2 : nL - 1); i >= 0; --i) {
      Layer &l = c->L[i];
      const float *W = params + l.p_off;
      const float *lin = i > 0 ? c->L[i - 1].a : (const float *)x;
      Layer *prev = i > 0 ? &c->L[i - 1] : nullptr;
      const int prev_act = (prev && (prev->d.kind == DP_DENSE || prev->d.kind == DP_CONV2D)) ? prev->d.act : DP_ACT_NONE;
      switch (l.d.kind) {
      case DP_DENSE: {
        if (priv && !(i == nL - 1 && fused_head) && !(h2 && i == nL - 2)) {
          dim3 grid = grid1d((long)B * 64, 256), block(256);
          float *slot = c->slots + (long)slot_next * slot_stride;
          slot_next += 1;
          Ln(LL("dense_norm"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(dense_norm_kernel, grid, block, 0, st, lin, l.d.in_features, (const float *)l.g,
                               l.d.out_features, slot, B);
          });
        }
        if (prev) {
          auto run = [&](auto vt) {
            constexpr bool V = decltype(vt)::value;
            typedef ProbBwdAct<OpRowMajor<V>, OpRowMajor<V>> Pb;
            Pb p{};
            p.M = B; p.N = l.d.in_features; p.K = l.d.out_features;
            p.a.set(l.g, l.d.out_features);
            p.b.set(W, l.d.out_features);
            p.out = prev->g; p.a_prev = prev->a; p.ld = l.d.in_features; p.act = prev_act;
            launch_gemm(p, 1, Ln, LL("dense_bwd_data"));
          };
          vec_dispatch(OpRowMajor<true>::can_vec(l.g, l.d.out_features, 0, l.d.out_features) &&
                              OpRowMajor<true>::can_vec(W, l.d.out_features, 0, l.d.out_features), run);
        }
      } break;
      case DP_CONV2D: {
        const ConvGeom &g = l.geom;
        if (priv && l.gram && aligned16(lin)) {
          ConvGramArgs ga{lin, l.g, c->slots + (long)slot_next * slot_stride, B, g.C, g.D};
          slot_next += 1;
          dim3 block(256);
          if (g.OH == 8) {
            dim3 grid(ceil_div(B, ConvGramGeom<8, 8>::NIMG));
            Ln(LL("conv_wgrad_norm"), grid, block, [&](hipStream_t st) {
              hipLaunchKernelGGL((conv_gram_norm_kernel<8, 8>), grid, block, 0, st, ga);
            });
          } else {
            dim3 grid(ceil_div(B, ConvGramGeom<4, 4>::NIMG));
            Ln(LL("conv_wgrad_norm"), grid, block, [&](hipStream_t st) {
              hipLaunchKernelGGL((conv_gram_norm_kernel<4, 4>), grid, block, 0, st, ga);
            });
          }
        } else if (priv && l.wino_norm && l.gst && aligned16(lin)) {
          const int cblocks = g.C / 32;
          ConvWinoWgUnitArgs a{};
          a.x = lin; a.dy = l.g; a.slots = c->slots; a.gstore = l.gst; a.slot_stride = slot_stride;
          a.gstride = l.gorder.n_total; a.slot0 = slot_next;
          a.B = B; a.C = g.C; a.D = g.D; a.H = g.H;
          a.ex_per_block = std::max(1, (int)((long)B * cblocks / 2048));
          slot_next += cblocks;
          dim3 grid(cblocks, ceil_div(B, a.ex_per_block)), block(256);
          Ln(LL("conv_wgrad_norm"), grid, block, [&](hipStream_t st) {
            if (g.W == 32) hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<32, 1, 1, true>), grid, block, 0, st, a);
            else if (g.D == 32) hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<16, 2, 1, true>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<16, 2, 2, true>), grid, block, 0, st, a);
          });
        } else if (priv && l.first_wg && aligned16(lin) && aligned16(l.g)) {
          ConvFirstWgArgs a{};
          a.x = lin; a.dy = l.g; a.slots = c->slots + (long)slot_next * slot_stride; a.slot_stride = slot_stride;
          a.gstore = l.gst; a.gstride = l.gorder.n_total; a.gbias_off = l.gorder.n_w;
          a.B = B; a.Cin = g.C; a.H = g.H; a.D = g.D;
          a.ex_per_wg = ceil_div(B, 512); // two workgroups per CU (one example per workgroup measured 56 us against 45)
          slot_next += 4;                 // one partial per wave
          dim3 grid(ceil_div(B, a.ex_per_wg)), block(256);
          Ln(LL("conv_wgrad_norm"), grid, block, [&](hipStream_t st) {
#define DP_CFW_CASE(full_, store_, h_)                                                                             \
  if ((g.D == 32) == full_ && (l.gst != nullptr) == store_ && g.H == h_)                                           \
    hipLaunchKernelGGL((conv_first_wgrad_kernel<full_, store_, h_>), grid, block, 0, st, a);
            DP_CFW_CASE(true, true, 32) DP_CFW_CASE(true, false, 32) DP_CFW_CASE(false, true, 32) DP_CFW_CASE(false, false, 32)
            DP_CFW_CASE(true, true, 16) DP_CFW_CASE(true, false, 16) DP_CFW_CASE(false, true, 16) DP_CFW_CASE(false, false, 16)
#undef DP_CFW_CASE
          });
        } else if (priv && l.dir_wg && aligned16(lin)) {
          // one round of resident workgroups, each walking through its run of examples: the next
          // example's tiles are fetched while the current one is multiplied and reduced
          const int cblocks = l.wg_flat ? 1 : ceil_div(g.C, 32);
          const int resident = 256 * (l.wg_ws ? 1 : (l.wg_db <= 2 ? 2 : 1));
          const int epb = ceil_div(B, std::max(1, resident / cblocks)); // per slice (measured: better than sharing one round)
          for (int d0 = 0; d0 < g.D; d0 += DP_WG_DSLICE) {
            ConvWgArgs a = make_wg_args(l, lin, B, l.t_wgn, d0);
            a.scale = c->ones; a.out = c->slots; a.mode = 0; a.ex_per_block = epb;
            a.slot_stride = slot_stride; a.slot0 = slot_next;
            a.gstore = l.gst; a.gstride = l.gorder.n_total; a.gbias_off = l.gorder.n_w;
            slot_next += cblocks;
            launch_conv_wgrad(Ln, LL("conv_wgrad_norm"), a, l.wg_db, l.wg_flat, l.wg_ws, ceil_div(B, epb));
          }
        } else if (priv) {
          auto run = [&](auto vt) {
            constexpr bool V = decltype(vt)::value;
            typedef ProbSqNorm<OpRowMajor<V>, OpConvPatch<false>> Pb;
            Pb p{};
            p.M = g.D; p.N = g.CKK + 1; p.K = g.P;
            p.a.set(l.g, g.P, (long)g.D * g.P);
            p.b.x = lin; p.b.g = g; p.b.has_ones = 1; p.b.by_z = 1;
            p.slots = c->slots; p.slot_stride = slot_stride; p.slot0 = slot_next;
            if (!l.dir_wg) { p.gstore = l.gst; p.gstride = l.gorder.n_total; } // ([D][CKK + 1] rows)
            GemmShape s = launch_gemm(p, B, Ln, LL("conv_wgrad_norm"));
            slot_next += s.tiles_m * s.tiles_n;
          };
          vec_dispatch(OpRowMajor<true>::can_vec(l.g, g.P, (long)g.D * g.P, g.P), run);
        }
        if (prev && l.u_b) {
          ConvWinoArgs a{};
          a.x = l.g; a.u = l.u_b; a.bias = nullptr; a.a_prev = prev->a; a.out = prev->g;
          a.B = B; a.Cin = g.D; a.Cpad = l.ub_cpad; a.H = g.H; a.W = g.W; a.M = g.C; a.Mpad = l.ub_mpad; a.act = prev_act;
          launch_conv_wino(Ln, LL("conv_bwd_data"), a, l.wino_b);
        } else if (prev && l.dir_bwd) {
          ConvS1Args a{};
          a.x = l.g; a.wt = l.wt_b; a.bias = nullptr; a.a_prev = prev->a; a.out = prev->g;
          a.B = B; a.Cin = g.D; a.H = g.OH; a.W = g.OW; a.M = g.C; a.Mpad = (g.C + 3) & ~3; a.OH = g.H; a.OW = g.W; a.pad = 2 - g.PAD;
          a.act = prev_act; a.t = l.t_bwd;
          launch_conv_s1(Ln, LL("conv_bwd_data"), a, l.bwd_npw);
        } else if (prev && l.cols) {
          {
            typedef ProbBatchOut<OpKMajor<false, false>, OpKMajor<false, false>> Pb;
            Pb p{};
            p.M = g.CKK; p.N = g.P; p.K = g.D;
            p.a.set(W, g.CKK);                       // (ckk, d) = W[d*CKK + ckk]
            p.b.set(l.g, g.P, (long)g.D * g.P);      // (p, d) of example z = Delta[z][d][p]
            p.out = l.cols; p.zstride = (long)g.CKK * g.P; p.ld = g.P;
            launch_gemm(p, B, Ln, LL("conv_bwd_data"));
          }
          const long total = (long)B * l.in_size;
          dim3 grid = grid1d(total, 256), block(256);
          Col2imDiv dv;
          dv.dW.init(g.W); dv.dH.init(g.H); dv.dC.init(g.C); dv.dS.init(g.S);
          Ln(LL("conv_bwd_data"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(conv_col2im_kernel, grid, block, 0, st, (const float *)l.cols, (const float *)prev->a,
                               prev->g, total, g.C, g.H, g.W, g.OH, g.OW, g.KH, g.KW, g.S, g.PAD, prev_act, dv);
          });
        } else if (prev) {
          typedef ProbConvBwd<OpConvWeightT, OpConvDeltaGather> Pb;
          Pb p{};
          p.M = g.C; p.N = B * g.H * g.W; p.K = g.D * g.KH * g.KW;
          p.a.w = W; p.a.g = g;
          p.b.delta = l.g; p.b.g = g; p.b.dS.init(g.S);
          p.out = prev->g; p.a_prev = prev->a; p.C = g.C; p.HW = g.H * g.W; p.act = prev_act; p.dHW = g.dHW;
          launch_gemm(p, 1, Ln, LL("conv_bwd_data"));
        }
      } break;
      case DP_MAXPOOL2D: {
        long total = (long)B * l.in_size;
        dim3 grid = grid1d(total, 256), block(256);
        const bool p22 = l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 2 && (l.inH & 1) == 0 && (l.inW & 1) == 0;
        if (p22) {
          const long nwin = (long)B * l.out_size;
          // (the pooled plane l.a stands in for the activation plane: the derivative is taken at the window's maximum)
          if ((l.outW & 1) == 0 && (l.inW & 3) == 0 && aligned16(prev->g) && aligned16(l.g) && aligned16(l.a)) {
            dim3 g2 = grid1d(nwin / 2, 256);
            Ln(LL("maxpool_bwd"), g2, block, [&](hipStream_t st) {
              hipLaunchKernelGGL(maxpool2x2_bwd2_kernel, g2, block, 0, st, (const float *)l.g, (const uint8_t *)l.arg,
                                 (const float *)l.a, prev->g, nwin / 2, l.outW / 2, l.inW, prev_act);
            });
          } else {
            dim3 g2 = grid1d(nwin, 256);
            Ln(LL("maxpool_bwd"), g2, block, [&](hipStream_t st) {
              hipLaunchKernelGGL(maxpool2x2_bwd_kernel, g2, block, 0, st, (const float *)l.g, (const uint8_t *)l.arg,
                                 (const float *)l.a, prev->g, nwin, l.outW, l.inW, prev_act);
            });
          }
        } else
        Ln(LL("maxpool_bwd"), grid, block, [&](hipStream_t st) {
          Split3 dv; dv.dX.init(l.inW); dv.dY.init(l.inH);
          FastDiv dS; dS.init(l.d.stride);
          if (l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 1)
            hipLaunchKernelGGL((maxpool_bwd_kernel<2, 1>), grid, block, 0, st, (const float *)l.g, (const uint8_t *)l.arg,
                               (const float *)prev->a, prev->g, total, l.inH, l.inW, l.outH, l.outW, l.d.kh, l.d.kw,
                               l.d.stride, prev_act, dv, dS);
          else
            hipLaunchKernelGGL((maxpool_bwd_kernel<0, 0>), grid, block, 0, st, (const float *)l.g, (const uint8_t *)l.arg,
                               (const float *)prev->a, prev->g, total, l.inH, l.inW, l.outH, l.outW, l.d.kh, l.d.kw,
                               l.d.stride, prev_act, dv, dS);
        });
      } break;
      case DP_AVGPOOL2D: {
        long total = (long)B * l.in_size;
        dim3 grid = grid1d(total, 256), block(256);
        const bool p22 = l.d.kh == 2 && l.d.kw == 2 && l.d.stride == 2 && (l.inH & 1) == 0 && (l.inW & 1) == 0;
        if (p22) {
          const long nwin = (long)B * l.out_size;
          dim3 g2 = grid1d(nwin, 256);
          Ln(LL("avgpool_bwd"), g2, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(avgpool2x2_bwd_kernel, g2, block, 0, st, (const float *)l.g, (const float *)prev->a,
                               prev->g, nwin, l.outW, l.inW, prev_act);
          });
        } else
        Ln(LL("avgpool_bwd"), grid, block, [&](hipStream_t st) {
          Split3 dv; dv.dX.init(l.inW); dv.dY.init(l.inH);
          FastDiv dS; dS.init(l.d.stride);
          hipLaunchKernelGGL(avgpool_bwd_kernel, grid, block, 0, st, (const float *)l.g, (const float *)prev->a,
                             prev->g, total, l.inH, l.inW, l.outH, l.outW, l.d.kh, l.d.kw, l.d.stride, prev_act, dv, dS);
        });
      } break;
      case DP_LSTM_LAST:
      case DP_LSTM_SEQ: {
        const int G = 4 * l.H;
        const float *Whh = W + (long)l.Din * G;
        LSTM_DISPATCH(launch_lstm_bwd, l.H, Ln, l, Whh, B, LL("lstm_bwd"));
        if (priv && l.lstm_wg && aligned16(lin) && aligned16(l.hs) && aligned16(l.gates)) {
          LstmWgArgs a{};
          a.x = lin; a.hs = l.hs; a.dg = l.gates; a.slots = c->slots; a.slot_stride = slot_stride; a.slot0 = slot_next;
          a.gstore = l.gst; a.gstride = l.p_count; a.B = B; a.T = l.T; a.Din = l.Din; a.H = l.H;
          const int halves = G > LWG_NH * 16 ? 2 : 1;
          slot_next += halves * 8; // one partial per wave
          // persistent workgroups, one per CU (their LDS leaves room for no second one): 128 x 2 halves
          dim3 grid(std::min(B, 256 / halves), halves), block(LWG_THREADS);
          Ln(LL("lstm_wgrad_norm"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(lstm_wgrad_kernel, grid, block, lstm_wgrad_lds_bytes(), st, a);
          });
        } else if (priv) {
          auto run = [&](auto vt) {
            constexpr bool V = decltype(vt)::value;
            typedef ProbSqNorm<OpLstmIn<V>, OpKMajor<V, false>> Pb;
            Pb p{};
            p.M = l.Din + l.H + 1; p.N = G; p.K = l.T;
            p.a.set(lin, l.hs, c->ones, l.Din, l.H, l.T, 1);
            p.b.set(l.gates, G, (long)l.T * G); p.b.by_z = 1;
            p.slots = c->slots; p.slot_stride = slot_stride; p.slot0 = slot_next;
            p.gstore = l.gst; p.gstride = l.p_count;
            GemmShape s = launch_gemm(p, B, Ln, LL("lstm_wgrad_norm"));
            slot_next += s.tiles_m * s.tiles_n;
          };
          vec_dispatch(OpLstmIn<true>::can_vec(lin, l.hs, l.Din, l.H) &&
                              OpKMajor<true, false>::can_vec(l.gates, G, (long)l.T * G, G), run);
        }
        // (measured on the 512 x 256-step configuration: 148 us this way against 133 us on the generic contraction --
        // one column block per wave leaves one LDS read per multiply and one wave of eight idle -- so the route stays
        // off; the kernel is kept for the projection, where it is 119 against 178 us)
        if (false && rows_gemm_fits(G, l.Din, 1, 4) && aligned16(l.gates) && !c->opt.no_rows_gemm) {
          // dx = dgates W_ih^T with W_ih^T held in registers by persistent workgroups
          RowsGemmArgs a{};
          a.A = l.gates; a.W = W; a.w_sk = 1; a.w_sn = G; a.bias = nullptr; a.C = prev->g;
          a.M = (long)B * l.T; a.K = G; a.N = l.Din;
          const long tiles = (a.M + 63) / 64;
          dim3 grid((unsigned)std::min<long>(tiles, 256)), block(RG_THREADS);
          Ln(LL("lstm_dx"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL((rows_gemm_kernel<1, 4, 4>), grid, block, rows_gemm_lds_bytes(4), st, a);
          });
        } else { // dx = dgates W_ih^T: gradient w.r.t. the embedding outputs
          auto run = [&](auto vt) {
            constexpr bool V = decltype(vt)::value;
            typedef ProbBwdAct<OpRowMajor<V>, OpRowMajor<V>> Pb;
            Pb p{};
            p.M = B * l.T; p.N = l.Din; p.K = G;
            p.a.set(l.gates, G);
            p.b.set(W, G);
            p.out = prev->g; p.a_prev = nullptr; p.ld = l.Din; p.act = DP_ACT_NONE;
            launch_gemm(p, 1, Ln, LL("lstm_dx"));
          };
          vec_dispatch(OpRowMajor<true>::can_vec(l.gates, G, 0, G) && OpRowMajor<true>::can_vec(W, G, 0, G), run);
        }
      } break;
      case DP_SEQ_MEAN: {
        const long n = (long)B * l.in_size;
        dim3 grid = grid1d(n, 256), block(256);
        Ln(LL("seq_mean_bwd"), grid, block, [&](hipStream_t st) {
          hipLaunchKernelGGL(seq_mean_bwd_kernel, grid, block, 0, st, (const float *)l.g, prev->g, n, l.T, l.Din);
        });
      } break;
      case DP_EMBEDDING: {
        if (priv) {
          dim3 grid(B), block(256);
          float *slot = c->slots + (long)slot_next * slot_stride;
          slot_next += 1;
          Ln(LL("emb_norm"), grid, block, [&](hipStream_t st) { // keys per thread: sequence length rounded up to 256, 512 or 1024
            if (l.outC <= 256)
              hipLaunchKernelGGL(emb_norm_kernel<1>, grid, block, 0, st, (const int *)x, (const float *)l.g, slot, l.outC, l.d.embed_dim);
            else if (l.outC <= 512)
              hipLaunchKernelGGL(emb_norm_kernel<2>, grid, block, 0, st, (const int *)x, (const float *)l.g, slot, l.outC, l.d.embed_dim);
            else
              hipLaunchKernelGGL(emb_norm_kernel<4>, grid, block, 0, st, (const int *)x, (const float *)l.g, slot, l.outC, l.d.embed_dim);
          });
        }
      } break;
      }
    }
    // ------------------------------------------------------------ clip factors
    if (priv && !(fused_head && nL == 1) && !f2) {
      dim3 grid = grid1d(B, 128), block(128);
      const int ns = slot_next;
      Ln("clip_factor", grid, block, [&](hipStream_t st) {
        hipLaunchKernelGGL(clip_factor_kernel, grid, block, 0, st, (const float *)c->slots, ns, slot_stride, C,
                           c->norms, c->s, B);
      });
    }
    // (two fused dense layers: the hidden layer's delta already carries the clip factors)
    const float *sc = (priv && !f2) ? c->s : c->ones;
    // ------------------------------------------------------------ clipped sums (split-K partials)
    for (int i = 0; i < nL; ++i) {
      Layer &l = c->L[i];
      if (l.p_count == 0) continue;
      const float *lin = i > 0 ? c->L[i - 1].a : (const float *)x;
      int nsplit = 1;
      switch (l.d.kind) {
      case DP_DENSE: {
        if (joint && i >= nL - 2) {
          if (i == nL - 2) {
            if (h2) joint_g[0].k_scale = joint_g[1].k_scale = sc; // (the head kernel could not scale: the clip factors came later)
            Ln(LL("dense_clipped_sum"), dim3(1), dim3(256), [&](hipStream_t st) { launch_dense_small_gemm(st, joint_g[0], &joint_g[1]); });
          }
          nsplit = 1;
          break;
        }
        if (f2 && i == 1) { nsplit = mid_tiles; break; } // its partials were written by dense2_mid_kernel
        if (f2 && !c->opt.no_small_gemm) {
          // X^T (s Delta) and the column sums of s Delta, complete in one partial row: K (= the batch) split inside
          // the workgroup
          SmallGemmArgs g{};
          g.A = lin; g.a_sr = 1; g.a_sk = l.d.in_features; g.a_ones = 1;
          g.B = l.g; g.b_sr = 1; g.b_sk = l.d.out_features;
          g.bias = nullptr; g.act = DP_ACT_NONE;
          g.C = l.part; g.c_sm = l.d.out_features; g.c_sn = 1; g.C_ones = l.part + (long)l.d.in_features * l.d.out_features;
          g.M = l.d.in_features; g.N = l.d.out_features; g.K = B;
          if (dense_small_gemm_fits(g)) {
            Ln(LL("dense_clipped_sum"), dim3(1), dim3(256), [&](hipStream_t st) { launch_dense_small_gemm(st, g); });
            nsplit = 1;
            break;
          }
        }
        auto run = [&](auto vt) {
          constexpr bool V = decltype(vt)::value;
          typedef ProbPartial<OpKMajor<V, true>, OpKMajor<V, false>> Pb;
          Pb p{};
          p.M = l.d.in_features + 1; p.N = l.d.out_features; p.K = B;
          p.a.set(lin, l.d.in_features); p.a.scale = sc; p.a.ones_row = 1;
          p.b.set(l.g, l.d.out_features);
          p.part = l.part; p.stride = l.pstride; p.ldm = l.d.out_features; p.bias_col = -1; p.bias_off = 0;
          nsplit = launch_gemm_split(p, l.max_split, Ln, LL("dense_clipped_sum"));
        };
        vec_dispatch(OpKMajor<true, true>::can_vec(lin, l.d.in_features, 0, l.d.in_features) &&
                            OpKMajor<true, false>::can_vec(l.g, l.d.out_features, 0, l.d.out_features), run);
      } break;
      case DP_CONV2D: {
        const ConvGeom &g = l.geom;
        if (priv && l.gst && (!l.dir_wg || aligned16(lin))) {
          // the norm pass of this step stored every example's gradient: weighted sum of the rows
          const long gstride = l.gorder.n_total;
          int want = (int)std::min<long>(l.max_split, std::max<long>(1, 4096 / ceil_div(gstride, 256)));
          const int eps = std::max(4, ceil_div(B, want));
          nsplit = ceil_div(B, eps);
          dim3 grid((unsigned)ceil_div(gstride, 256), nsplit), block(256);
          Ln(LL("conv_weighted_sum"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(weighted_sum_kernel, grid, block, 0, st, (const float *)l.gst, gstride, sc, l.part,
                               l.pstride, l.gorder, B, eps);
          });
          break;
        }
        if ((l.wino_wgu || l.wino_wg) && aligned16(lin) && aligned16(l.g)) {
          // batch sum in the F(3x3, 2x2) form: blocks of 32 input x 32 or 64 output channels, splits over examples
          const int db = (g.D % 64 == 0) ? 2 : 1;
          const int tiles = (g.C / 32) * (g.D / (32 * db));
          int want = std::max(1, std::min(l.max_split, 512 / tiles));
          const int eps = ceil_div(B, want);
          nsplit = ceil_div(B, eps);
          ConvWinoWgUnitArgs a{};
          a.x = lin; a.dy = l.g; a.scale = sc; a.part = l.part; a.part_stride = l.pstride;
          a.B = B; a.C = g.C; a.D = g.D; a.H = g.H; a.ex_per_block = eps;
          dim3 grid(g.C / 32, nsplit, g.D / (32 * db)), block(256);
          Ln(LL("conv_clipped_sum"), grid, block, [&](hipStream_t st) {
            if (g.W == 8) hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<8, 4, 2, false>), grid, block, 0, st, a);
            else if (g.W == 32) hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<32, 1, 1, false>), grid, block, 0, st, a);
            else if (db == 1) hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<16, 2, 1, false>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((conv_wino_wgrad_unit_kernel<16, 2, 2, false>), grid, block, 0, st, a);
          });
          break;
        }
        if (l.dir_wg && aligned16(lin)) {
          const int cblocks = l.wg_flat ? 1 : ceil_div(g.C, 32);
          // one full round of resident workgroups (256 CUs x workgroups per CU) avoids a ragged tail
          const int occ = l.wg_ws ? 1 : (l.wg_db == 1 ? 3 : (l.wg_db == 2 ? 2 : 1));
          int want = (256 * occ) / cblocks;
          if (want < 1) want = 1;
          if (want > l.max_split) want = l.max_split;
          int epb = ceil_div(B, want);
          epb = ceil_div(epb, l.t_wgc.NIMG) * l.t_wgc.NIMG;
          nsplit = ceil_div(B, epb);
          for (int d0 = 0; d0 < g.D; d0 += DP_WG_DSLICE) {
            ConvWgArgs a = make_wg_args(l, lin, B, l.t_wgc, d0);
            a.scale = sc; a.out = l.part + (long)d0 * g.CKK; a.mode = 1; a.ex_per_block = epb; a.part_stride = l.pstride;
            launch_conv_wgrad(Ln, LL("conv_clipped_sum"), a, l.wg_db, l.wg_flat, l.wg_ws, nsplit);
          }
          break;
        }
        typedef ProbPartial<OpChanPix, OpConvPatch<false>> Pb;
        Pb p{};
        p.M = g.D; p.N = g.CKK + 1; p.K = B * g.P;
        p.a.t = l.g; p.a.scale = sc; p.a.D = g.D; p.a.P = g.P; p.a.by_z = 0; p.a.dP = g.dP;
        p.b.x = lin; p.b.g = g; p.b.has_ones = 1; p.b.by_z = 0;
        p.part = l.part; p.stride = l.pstride; p.ldm = g.CKK; p.bias_col = g.CKK; p.bias_off = (long)g.D * g.CKK;
        nsplit = launch_gemm_split(p, l.max_split, Ln, LL("conv_clipped_sum"));
      } break;
      case DP_LSTM_LAST:
      case DP_LSTM_SEQ: {
        const int G = 4 * l.H;
        if (priv && l.gst) { // the norm pass of this step stored every example's gradient
          int want = (int)std::min<long>(l.max_split, std::max<long>(1, 4096 / ceil_div(l.p_count, 256)));
          const int eps = std::max(4, ceil_div(B, want));
          nsplit = ceil_div(B, eps);
          dim3 grid((unsigned)ceil_div(l.p_count, 256), nsplit), block(256);
          Ln(LL("lstm_weighted_sum"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(weighted_sum_kernel, grid, block, 0, st, (const float *)l.gst, l.p_count, sc, l.part,
                               l.pstride, l.gorder, B, eps);
          });
          break;
        }
        auto run = [&](auto vt) {
          constexpr bool V = decltype(vt)::value;
          typedef ProbPartial<OpLstmIn<V>, OpKMajor<V, false>> Pb;
          Pb p{};
          p.M = l.Din + l.H + 1; p.N = G; p.K = B * l.T;
          p.a.set(lin, l.hs, sc, l.Din, l.H, l.T, 0);
          p.b.set(l.gates, G);
          p.part = l.part; p.stride = l.pstride; p.ldm = G; p.bias_col = -1; p.bias_off = 0;
          nsplit = launch_gemm_split(p, l.max_split, Ln, LL("lstm_clipped_sum"));
        };
        vec_dispatch(OpLstmIn<true>::can_vec(lin, l.hs, l.Din, l.H) && OpKMajor<true, false>::can_vec(l.gates, G, 0, G), run);
      } break;
      case DP_EMBEDDING: {
        const long rows = (long)B * l.outC;
        const int V = l.d.vocab;
        if (emb_early) (void)hipStreamWaitEvent(c->stream, c->ev_join, 0); // the token lists were built beside the forward pass
        else emb_prepare(l, i, Ln);
        {
          // every token has at most ceil(count/EMB_CH) chunks: rows/EMB_CH + V bounds their number
          dim3 grid((unsigned)(rows / EMB_CH + V + 1)), block(256);
          Ln(LL("emb_scatter"), grid, block, [&](hipStream_t st) {
            hipLaunchKernelGGL(emb_reduce_kernel, grid, block, 0, st, (const int *)l.e_start,
                               (const int *)l.e_chunk0, (const int *)l.e_list, (const float *)l.g, sc, l.part, V,
                               l.outC, l.d.embed_dim);
          });
        }
        nsplit = 1;
      } break;
      default: break;
      }
      FinalizeSeg &sg = fa.seg[fa.nseg++];
      sg.p_off = l.p_off; sg.n = l.p_count; sg.part = l.part; sg.stride = l.pstride; sg.nsplit = nsplit;
    }
  } else {
    for (auto &l : c->L) {
      if (l.p_count == 0) continue;
      FinalizeSeg &sg = fa.seg[fa.nseg++];
      sg.p_off = l.p_off; sg.n = l.p_count; sg.part = l.part; sg.stride = l.pstride; sg.nsplit = 0;
    }
  }
  // ------------------------------------------------------------ final write with fused noise
  {
    const float noise_std = (priv && sigma > 0.f) ? sigma * C : 0.f;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    Ln("finalize_noise", dim3(1), dim3(256), [&](hipStream_t st) {
      launch_finalize(st, fa, out, c->P, noise_std, k0, k1, theta_update, update_step);
    });
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    snprintf(g_hip_err, sizeof(g_hip_err), "kernel launch: %s", hipGetErrorString(e));
    return DP_EHIP;
  }
  if (priv) c->last_batch = B;
  return DP_OK;
}

extern "C" int dp_step(dp_ctx *c, const float *params, const void *x, const int32_t *y, int batch, float C, float sigma,
                       uint64_t seed, float *out_grad) {
  if (!c || !params || !out_grad || batch < 0 || batch > c->maxB) return DP_EINVAL;
  if (batch > 0 && (!x || !y)) return DP_EINVAL;
  if (!(C > 0.f) || !(sigma >= 0.f) || std::isnan(C) || std::isinf(sigma)) return DP_EINVAL;
  if (std::isinf(C) && sigma > 0.f) return DP_EINVAL;
  return run_step(c, params, x, y, batch, true, C, sigma, seed, out_grad);
}

extern "C" int dp_step_sgd(dp_ctx *c, float *params, const void *x, const int32_t *y, int batch, float C, float sigma,
                           uint64_t seed, float lr, float *out_grad) {
  if (!c || !params || batch < 1 || batch > c->maxB || !x || !y) return DP_EINVAL;
  if (!(C > 0.f) || !(sigma >= 0.f) || std::isnan(C) || std::isinf(sigma) || std::isnan(lr) || std::isinf(lr)) return DP_EINVAL;
  if (std::isinf(C) && sigma > 0.f) return DP_EINVAL;
  // every kernel of the step reads params before the final write, which is the last launch on the stream
  return run_step(c, params, x, y, batch, true, C, sigma, seed, out_grad, params, lr / (float)batch);
}

extern "C" int dp_step_nonprivate(dp_ctx *c, const float *params, const void *x, const int32_t *y, int batch,
                                  float *out_grad) {
  if (!c || !params || !out_grad || batch < 0 || batch > c->maxB) return DP_EINVAL;
  if (batch > 0 && (!x || !y)) return DP_EINVAL;
  return run_step(c, params, x, y, batch, false, INFINITY, 0.f, 0, out_grad);
}

// counts labels outside [0, n_classes) and token ids outside [0, vocab)
__global__ void validate_kernel(const int *__restrict__ y, int B, int n_classes, const int *__restrict__ tok, long n_tok,
                                int vocab, int *__restrict__ bad) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  int mine = 0;
  if (i < B) mine += (unsigned)y[i] >= (unsigned)n_classes;
  if (i < n_tok) mine += (unsigned)tok[i] >= (unsigned)vocab;
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
  if ((threadIdx.x & 63) == 0 && mine) atomicAdd(bad, mine);
}
__global__ void zero_int_kernel(int *p) { *p = 0; }

extern "C" int dp_step_validate(dp_ctx *c, const void *x, const int32_t *y, int batch, int *n_bad) {
  if (!c || !n_bad || batch < 0 || batch > c->maxB) return DP_EINVAL;
  *n_bad = 0;
  if (batch == 0) return DP_OK;
  if (!x || !y) return DP_EINVAL;
  const bool tok = c->m.seq_len > 0;
  const long n_tok = tok ? (long)batch * c->m.seq_len : 0;
  const long n = std::max<long>(batch, n_tok);
  hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, c->stream, c->bad);
  hipLaunchKernelGGL(validate_kernel, grid1d(n, 256), dim3(256), 0, c->stream, (const int *)y, batch, c->m.n_classes,
                     tok ? (const int *)x : (const int *)nullptr, n_tok, tok ? c->L[0].d.vocab : 1, c->bad);
  HIP_TRY(hipMemcpyAsync(n_bad, c->bad, sizeof(int), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  return DP_OK;
}

extern "C" int dp_step_last_norms(dp_ctx *c, float *norms_out) {
  if (!c || !norms_out || c->last_batch < 0) return DP_EINVAL;
  if (c->last_batch == 0) return DP_OK;
  HIP_TRY(hipMemcpyAsync(norms_out, c->norms, sizeof(float) * c->last_batch, hipMemcpyDeviceToDevice, c->stream));
  return DP_OK;
}

// ---------------------------------------------------------------- minibatch draw and the training loop

// DPSGD item 1: index k of the minibatch = (word k%4 of the Philox block with counter (k/4, 0, 1, 0)) * n >> 32 --
// uniform over [0, n), with replacement; the third counter word keeps these blocks apart from the noise stream's.
__global__ void sample_indices_kernel(uint32_t k0, uint32_t k1, long n, int batch, int *__restrict__ idx) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= batch) return;
  uint32_t r[4];
  philox4x32_10((uint32_t)(k >> 2), 0u, 1u, 0u, k0, k1, r);
  idx[k] = (int)(((uint64_t)r[k & 3] * (uint64_t)n) >> 32);
}

// one workgroup per drawn example: its input row (fp32 features or int32 token ids: 4-byte words) and its label
__global__ void gather_rows_kernel(const uint32_t *__restrict__ data_x, const int *__restrict__ data_y,
                                   const int *__restrict__ idx, long row_words, uint32_t *__restrict__ xb,
                                   int *__restrict__ yb) {
  const long src = (long)idx[blockIdx.x] * row_words, dst = (long)blockIdx.x * row_words;
  for (long i = threadIdx.x; i < row_words; i += blockDim.x) xb[dst + i] = data_x[src + i];
  if (threadIdx.x == 0) yb[blockIdx.x] = data_y[idx[blockIdx.x]];
}

extern "C" int dp_step_sample_indices(uint64_t seed, int64_t n_examples, int batch, int32_t *indices, void *hip_stream) {
  if (!indices || batch < 0 || n_examples < 1 || n_examples > 0x7fffffffl) return DP_EINVAL;
  if (batch == 0) return DP_OK;
  hipLaunchKernelGGL(sample_indices_kernel, grid1d(batch, 256), dim3(256), 0, (hipStream_t)hip_stream, (uint32_t)seed,
                     (uint32_t)(seed >> 32), (long)n_examples, batch, (int *)indices);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    snprintf(g_hip_err, sizeof(g_hip_err), "kernel launch: %s", hipGetErrorString(e));
    return DP_EHIP;
  }
  return DP_OK;
}

extern "C" int dp_step_loop(dp_ctx *c, float *params, const void *data_x, const int32_t *data_y, int64_t n_examples,
                            int steps, int batch, float C, float sigma, uint64_t seed0, float lr) {
  if (!c || !params || !data_x || !data_y || steps < 0 || batch < 1 || batch > c->maxB || n_examples < 1 ||
      n_examples > 0x7fffffffl)
    return DP_EINVAL;
  if (!(C > 0.f) || !(sigma >= 0.f) || std::isnan(C) || std::isinf(sigma) || std::isnan(lr) || std::isinf(lr)) return DP_EINVAL;
  if (std::isinf(C) && sigma > 0.f) return DP_EINVAL;
  const long row_words = c->m.seq_len > 0 ? c->m.seq_len : (long)c->m.in_c * c->m.in_h * c->m.in_w;
  if (!c->xb) { // first call on this context: room for one drawn minibatch
    int rc = dev_alloc(c, &c->xb, (size_t)c->maxB * row_words);
    if (rc == DP_OK) rc = dev_alloc(c, &c->yb, c->maxB);
    if (rc == DP_OK) rc = dev_alloc(c, &c->idx, c->maxB);
    if (rc != DP_OK) { c->xb = nullptr; return rc; }
  }
  Launcher Ln{c};
  for (int t = 0; t < steps; ++t) {
    const uint64_t seed = seed0 + (uint64_t)t;
    Ln("sample_minibatch", dim3(1), dim3(256), [&](hipStream_t st) {
      hipLaunchKernelGGL(sample_indices_kernel, grid1d(batch, 256), dim3(256), 0, st, (uint32_t)seed, (uint32_t)(seed >> 32),
                         (long)n_examples, batch, c->idx);
      hipLaunchKernelGGL(gather_rows_kernel, dim3(batch), dim3(256), 0, st, (const uint32_t *)data_x, (const int *)data_y,
                         (const int *)c->idx, row_words, c->xb, c->yb);
    });
    int rc = run_step(c, params, c->xb, c->yb, batch, true, C, sigma, seed, nullptr, params, lr / (float)batch);
    if (rc != DP_OK) return rc;
  }
  return DP_OK;
}

// ---------------------------------------------------------------- plan description and measured ceilings

extern "C" int dp_step_describe_plan(const dp_ctx *c, char *buf, size_t cap) {
  if (!c || !buf || cap == 0) return DP_EINVAL;
  std::string o;
  for (size_t i = 0; i < c->L.size(); ++i) {
    const Layer &l = c->L[i];
    if (l.p_count == 0) continue;
    std::string fwd = "-", bwd = "-", norm = "-", sum = "-";
    switch (l.d.kind) {
    case DP_DENSE:
      fwd = c->fused1 ? "fused" : "generic"; bwd = i > 0 ? "generic" : "-";
      norm = c->fused1 ? "fused" : "identity"; sum = c->fused1 ? "fused" : "generic";
      if (c->fused2) { norm = "fused"; if (i == 1) { fwd = bwd = "fused"; sum = c->joint2 ? "joint" : "fused"; } }
      if (c->head2 && i + 2 >= c->L.size()) { norm = "head"; if (i + 1 == c->L.size()) { fwd = bwd = "head"; if (c->joint2) sum = "joint"; } }
      if (c->fusedcnn) fwd = bwd = norm = sum = "fused-net";
      break;
    case DP_CONV2D:
      fwd = l.u_f ? (l.wino_f == 2 ? "mf64" : "mf32") : (l.first_fwd ? "first" : (l.dir_fwd ? "direct" : "generic"));
      if (l.u_f && i + 1 < c->L.size() && !c->opt.no_pool_fusion) { // the pool after the layer is taken in its epilogue
        const dp_layer_desc &n = c->L[i + 1].d;
        if ((n.kind == DP_MAXPOOL2D || n.kind == DP_AVGPOOL2D) && n.kh == 2 && n.kw == 2 && n.stride == 2)
          fwd += n.kind == DP_MAXPOOL2D ? "+maxpool" : "+avgpool";
      }
      bwd = i == 0 ? "-" : (l.u_b ? (l.wino_b == 2 ? "mf64" : "mf32") : (l.dir_bwd ? "direct" : (l.cols ? "columns" : "generic")));
      norm = l.gram ? "gram" : ((l.wino_norm && l.gst) ? "mf+store" : (l.dir_wg ? (l.gst ? "direct+store" : (l.wg_ws ? "ws" : "direct"))
                                                                                : (l.gst ? "generic+store" : "generic")));
      sum = l.gst ? "weighted" : ((l.wino_wgu || l.wino_wg) ? "mf" : (l.dir_wg ? (l.wg_ws ? "ws" : "direct") : "generic"));
      if (c->fusedcnn) fwd = bwd = norm = sum = "fused-net";
      break;
    case DP_EMBEDDING: fwd = "gather"; norm = "sorted-segments"; sum = "scatter"; break;
    case DP_LSTM_LAST:
    case DP_LSTM_SEQ: fwd = "recurrence"; bwd = "recurrence"; norm = l.gst ? "generic+store" : "generic"; sum = l.gst ? "weighted" : "generic"; break;
    default: break;
    }
    o += std::to_string(i) + ":fwd=" + fwd + ",bwd=" + bwd + ",norm=" + norm + ",sum=" + sum + ";";
  }
  if (o.size() + 1 > cap) return DP_EINVAL;
  memcpy(buf, o.c_str(), o.size() + 1);
  return DP_OK;
}

extern "C" int dp_step_ceiling(int what, void *hip_stream, double *value) {
  if (!value || what < 0 || what > 2) return DP_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  HIP_TRY(hipEventCreate(&e0));
  HIP_TRY(hipEventCreate(&e1));
  float ms = 0.f;
  int rc = DP_OK;
  auto fail = [&](hipError_t e, const char *what_) {
    snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what_, hipGetErrorString(e));
    rc = DP_EHIP;
  };
  if (what == 0) { // copy of 256 MiB: bytes read + bytes written per second
    const size_t bytes = (size_t)256 << 20;
    void *a = nullptr, *b = nullptr;
    hipError_t e = hipMalloc(&a, bytes);
    if (e == hipSuccess) e = hipMalloc(&b, bytes);
    if (e == hipSuccess) e = hipMemsetAsync(a, 0, bytes, st);
    if (e != hipSuccess) { fail(e, "hipMalloc"); }
    else {
      double best = 1e30;
      for (int rep = 0; rep < 6 && rc == DP_OK; ++rep) {
        (void)hipEventRecord(e0, st);
        hipLaunchKernelGGL(ceiling_copy_kernel, dim3(256 * 16), dim3(256), 0, st, (const float4 *)a, (float4 *)b, (long)(bytes / 16));
        (void)hipEventRecord(e1, st);
        e = hipEventSynchronize(e1);
        if (e != hipSuccess) { fail(e, "copy"); break; }
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (rep > 0 && ms < best) best = ms;
      }
      *value = 2.0 * (double)bytes / (best * 1e-3) / 1e9; // GB/s
    }
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
  } else if (what == 1) { // fp32 MFMA: 2048 workgroups x 4 waves x iters x 4 tiles x 4096 flops
    const int blocks = 2048, iters = 20000;
    void *o = nullptr;
    hipError_t e = hipMalloc(&o, (size_t)blocks * 256 * 4);
    if (e != hipSuccess) { fail(e, "hipMalloc"); }
    else {
      hipLaunchKernelGGL(ceiling_mfma_kernel, dim3(blocks), dim3(256), 0, st, (float *)o, 100, 1.f, 2.f);
      (void)hipEventRecord(e0, st);
      hipLaunchKernelGGL(ceiling_mfma_kernel, dim3(blocks), dim3(256), 0, st, (float *)o, iters, 1.f, 2.f);
      (void)hipEventRecord(e1, st);
      e = hipEventSynchronize(e1);
      if (e != hipSuccess) fail(e, "mfma loop");
      else {
        (void)hipEventElapsedTime(&ms, e0, e1);
        *value = (double)blocks * 4 * iters * 4 * 4096.0 / (ms * 1e-3) / 1e12; // TFLOP/s
      }
      (void)hipFree(o);
    }
  } else { // microseconds per launch of an empty kernel, 1000 launches back to back
    const int n = 1000;
    for (int i = 0; i < 50; ++i) hipLaunchKernelGGL(ceiling_empty_kernel, dim3(1), dim3(64), 0, st);
    (void)hipEventRecord(e0, st);
    for (int i = 0; i < n; ++i) hipLaunchKernelGGL(ceiling_empty_kernel, dim3(1), dim3(64), 0, st);
    (void)hipEventRecord(e1, st);
    hipError_t e = hipEventSynchronize(e1);
    if (e != hipSuccess) fail(e, "empty launches");
    else {
      (void)hipEventElapsedTime(&ms, e0, e1);
      *value = ms * 1e3 / n;
    }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}

// ---------------------------------------------------------------- profiling

static int drain_profile(dp_ctx *c) {
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (auto &r : c->recs) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, r.e0, r.e1));
    c->label_launches[r.label] += 1;
    c->label_ms[r.label] += ms;
  }
  c->recs.clear();
  c->pool_used = 0;
  return DP_OK;
}

extern "C" int dp_step_profile(dp_ctx *c, int enable) {
  if (!c) return DP_EINVAL;
  if (enable && c->pool.empty()) {
    c->pool.resize(16384);
    for (auto &e : c->pool) HIP_TRY(hipEventCreate(&e));
  }
  if (!enable && c->prof) {
    int rc = drain_profile(c);
    if (rc != DP_OK) return rc;
  }
  c->prof = enable != 0;
  return DP_OK;
}

extern "C" int dp_step_profile_read(dp_ctx *c, int cap, const char **labels, int *launches, float *total_ms, int reset) {
  if (!c || cap < 0) return DP_EINVAL;
  int rc = drain_profile(c);
  if (rc != DP_OK) return rc;
  int n = (int)c->labels.size();
  for (int i = 0; i < n && i < cap; ++i) {
    if (labels) labels[i] = c->labels[i];
    if (launches) launches[i] = c->label_launches[i];
    if (total_ms) total_ms[i] = c->label_ms[i];
  }
  if (reset)
    for (int i = 0; i < n; ++i) { c->label_launches[i] = 0; c->label_ms[i] = 0.f; }
  return n;
}

// ---------------------------------------------------------------- allocation-free entry point

// Scratch of dp_step_dense1_static: the partial clipped sums [tiles][P] and the clip factors [batch].  Every GPU
// the library is loaded on holds its own copy of this array until the process ends; host code reaches it only
// through the per-device address that hipGetSymbolAddress returns (the array's name is not a device address).
#define DP_STATIC_FLOATS (2l << 20) // 8 MiB
#define DP_STATIC_MAX_BATCH 65536
#define DP_STATIC_MAX_DEVICES 64
static __device__ __align__(256) float dp_static_scratch[DP_STATIC_FLOATS];
static std::mutex g_static_mu;
static float *g_static_ptr[DP_STATIC_MAX_DEVICES] = {};

static int static_scratch_ptr(float **out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= DP_STATIC_MAX_DEVICES) return DP_EINVAL;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (g_static_ptr[dev] == nullptr) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(dp_static_scratch)));
    if (p == nullptr) return DP_EHIP;
    g_static_ptr[dev] = (float *)p;
  }
  *out = g_static_ptr[dev];
  return DP_OK;
}

extern "C" int dp_step_dense1_static(const float *params, const float *x, const int32_t *y, int batch, int in_features,
                                     int n_classes, float C, float sigma, uint64_t seed, float *out_grad,
                                     float *norms_out, void *hip_stream) {
  if (!params || !out_grad || batch < 0 || in_features < 1 || n_classes < 1) return DP_EINVAL;
  if (batch > 0 && (!x || !y)) return DP_EINVAL;
  if (!(C > 0.f) || !(sigma >= 0.f) || std::isnan(C) || std::isinf(sigma)) return DP_EINVAL;
  if (std::isinf(C) && sigma > 0.f) return DP_EINVAL;
  if (!dense1_fits(in_features, n_classes) || batch > DP_STATIC_MAX_BATCH) return DP_ETOOBIG;
  const long P = (long)(in_features + 1) * n_classes;
  const long max_tiles = (DP_STATIC_FLOATS - DP_STATIC_MAX_BATCH) / dense1_part_stride(in_features, n_classes); // the clip factors take the last 65,536 floats
  if (max_tiles < 1) return DP_ETOOBIG;
  float *scratch = nullptr;
  int rc = static_scratch_ptr(&scratch);
  if (rc != DP_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  FinalizeArgs fa;
  fa.nseg = 1;
  FinalizeSeg &sg = fa.seg[0];
  const long pstride = dense1_part_stride(in_features, n_classes);
  sg.p_off = 0; sg.n = P; sg.part = scratch; sg.stride = pstride; sg.nsplit = 0;
  if (batch > 0) {
    Dense1Args a{};
    a.x = x; a.W = params; a.bias = params + (long)in_features * n_classes; a.y = (const int *)y;
    a.part = scratch; a.norms = norms_out; a.s = scratch + (DP_STATIC_FLOATS - DP_STATIC_MAX_BATCH); a.delta = nullptr;
    a.B = batch; a.d_in = in_features; a.N = n_classes; a.C = C; a.priv = 1;
    sg.nsplit = launch_dense1_fused(st, a, (int)std::min<long>(DENSE1_MAX_TILES, max_tiles));
  }
  const float noise_std = sigma > 0.f ? sigma * C : 0.f;
  launch_finalize(st, fa, out_grad, P, noise_std, (uint32_t)seed, (uint32_t)(seed >> 32), (float *)nullptr, 0.f);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    snprintf(g_hip_err, sizeof(g_hip_err), "kernel launch: %s", hipGetErrorString(e));
    return DP_EHIP;
  }
  return DP_OK;
}

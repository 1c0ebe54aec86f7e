// Tiled fp32 MFMA contraction for gfx950, parameterised by operand and epilogue functors.
//
// C[z](m, n) = sum_k A[z](m, k) * B[z](k, n),   k in the block's split-K range.
//
// Every contraction of the private step is an instance: dense / conv forward,
// backward-data, the per-example weight-gradient tiles whose squares are reduced
// to a norm, and the clipped sum A^T diag(s) Delta (DPSGD item 3, Section 1).
// An operand is not a matrix in memory but a functor: it names an element by a
// "fixed-dimension" context (row m of A / column n of B) and a "k" context, so
// im2col patches, gathered embedding rows, [x; h; 1] LSTM inputs and the clip
// factor s_i are applied while the tile is staged into LDS and never written out.
//
// Tile: BM x BN x 32, WM x WN wavefronts of 64 lanes; each wave owns a
// (BM/WM) x (BN/WN) sub-tile made of 32x32 blocks of v_mfma_f32_32x32x2_f32.
// LDS holds A and B tiles k-major (tile[k][row]) so the MFMA operand read
// (32 consecutive rows for one k) is conflict-free; rows are padded by 2 words
// so the transposing store of k-contiguous operands is conflict-free as well.
// Global loads for tile t+1 are issued into registers before the MFMAs of tile t.
#pragma once
#include <algorithm>
#include <cstdlib>
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DEVI __device__ __forceinline__

typedef float f32x16 __attribute__((ext_vector_type(16)));

// n / d for n < 2^31 by multiply-shift (d fixed on the host).
struct FastDiv {
  uint32_t d, mul, sh;
  void init(uint32_t d_) {
    d = d_ ? d_ : 1;
    sh = 0;
    while ((1ull << sh) < d) ++sh;
    mul = (uint32_t)((((1ull << 32) * ((1ull << sh) - d)) / d) + 1);
  }
  DEVI uint32_t div(uint32_t n) const { return (__umulhi(n, mul) + n) >> sh; }
};

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = 32, WM = WM_, WN = WN_;
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int TM = BM / WM, TN = BN / WN; // wave sub-tile
  static constexpr int MB = TM / 32, NB = TN / 32; // 32x32 MFMA blocks per wave
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert(THREADS % BK == 0 && THREADS % BM == 0 && THREADS % BN == 0, "loader mapping");
  static_assert((BM * BK) % THREADS == 0 && (BN * BK) % THREADS == 0, "loader mapping");
};

DEVI float4 f4zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }

// Stages one operand tile (ROWS x BK) from its functor into registers, then into LDS
// laid out k-major: tile[k*LD + row].  A functor splits an element access in three:
//   post(fc, kc)        what to do with the value (validity, scale, constant), from the contexts alone
//   raw(fc, kc, post)   the load itself, unconditional, from a safe address when the element is invalid
//   finish(raw, post)   the element value
// fetch() only issues raw loads; finish() runs in stash(), after the MFMAs of the previous
// tile, so nothing touches a loaded register (and forces a wait) while the loads are in flight.  Four variants: lanes walk k or the fixed
// dimension (whichever is contiguous in memory), one float or one float4 per item.
enum { LOAD_SCALAR_K = 0, LOAD_SCALAR_F = 1, LOAD_VEC_K = 2, LOAD_VEC_F = 3 };
template <class Op>
struct LoaderKind {
  static constexpr int value = Op::kVec ? (Op::kLanesAlongK ? LOAD_VEC_K : LOAD_VEC_F)
                                        : (Op::kLanesAlongK ? LOAD_SCALAR_K : LOAD_SCALAR_F);
};
template <class Op, int ROWS, int THREADS, int BK, int KIND = LoaderKind<Op>::value>
struct TileLoader;

// lanes run along k: a thread owns one k of the tile and CNT fixed rows
template <class Op, int ROWS, int THREADS, int BK>
struct TileLoader<Op, ROWS, THREADS, BK, LOAD_SCALAR_K> {
  static constexpr int LD = ROWS + 2;
  static constexpr int CNT = ROWS * BK / THREADS, RSTEP = THREADS / BK;
  typename Op::FC fc[CNT];
  typename Op::Post post[CNT];
  float r[CNT];
  int kk, r0;
  DEVI void init(const Op &op, int z, int row0, int nrows) {
    kk = threadIdx.x % BK;
    r0 = threadIdx.x / BK;
#pragma unroll
    for (int j = 0; j < CNT; ++j) fc[j] = op.fctx(z, row0 + r0 + j * RSTEP, nrows);
  }
  DEVI void fetch(const Op &op, int z, int k0, int kend) {
    typename Op::KC kc = op.kctx(z, k0 + kk, kend);
#pragma unroll
    for (int j = 0; j < CNT; ++j) { post[j] = op.post(fc[j], kc); r[j] = op.raw(fc[j], kc, post[j]); }
  }
  DEVI void stash(const Op &op, float *tile) const {
#pragma unroll
    for (int j = 0; j < CNT; ++j) tile[kk * LD + r0 + j * RSTEP] = op.finish(r[j], post[j]);
  }
};

// lanes run along the fixed dimension: a thread owns one row and CNT k's of the tile
template <class Op, int ROWS, int THREADS, int BK>
struct TileLoader<Op, ROWS, THREADS, BK, LOAD_SCALAR_F> {
  static constexpr int LD = ROWS + 2;
  static constexpr int CNT = ROWS * BK / THREADS, KSTEP = THREADS / ROWS;
  typename Op::FC fc;
  typename Op::Post post[CNT];
  float r[CNT];
  int rr, kq;
  DEVI void init(const Op &op, int z, int row0, int nrows) {
    rr = threadIdx.x % ROWS;
    kq = threadIdx.x / ROWS;
    fc = op.fctx(z, row0 + rr, nrows);
  }
  DEVI void fetch(const Op &op, int z, int k0, int kend) {
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
      typename Op::KC kc = op.kctx(z, k0 + kq + j * KSTEP, kend);
      post[j] = op.post(fc, kc);
      r[j] = op.raw(fc, kc, post[j]);
    }
  }
  DEVI void stash(const Op &op, float *tile) const {
#pragma unroll
    for (int j = 0; j < CNT; ++j) tile[(kq + j * KSTEP) * LD + rr] = op.finish(r[j], post[j]);
  }
};

// float4 along k (k-contiguous operand): a thread owns one group of 4 k's and CNT rows;
// the store into the k-major tile transposes (4 scalar LDS writes per item)
template <class Op, int ROWS, int THREADS, int BK>
struct TileLoader<Op, ROWS, THREADS, BK, LOAD_VEC_K> {
  static constexpr int LD = ROWS + 2;
  static constexpr int KG = BK / 4, RSTEP = THREADS / KG, CNT = ROWS / RSTEP;
  static_assert(ROWS % RSTEP == 0 && CNT >= 1, "vec-k loader mapping");
  typename Op::FC fc[CNT];
  typename Op::Post4 post[CNT];
  float4 r[CNT];
  int kg, r0;
  DEVI void init(const Op &op, int z, int row0, int nrows) {
    kg = threadIdx.x % KG;
    r0 = threadIdx.x / KG;
#pragma unroll
    for (int j = 0; j < CNT; ++j) fc[j] = op.fctx(z, row0 + r0 + j * RSTEP, nrows);
  }
  DEVI void fetch(const Op &op, int z, int k0, int kend) {
    typename Op::KC4 kc = op.kctx4(z, k0 + 4 * kg, kend);
#pragma unroll
    for (int j = 0; j < CNT; ++j) { post[j] = op.post4(fc[j], kc); r[j] = op.raw4(fc[j], kc, post[j]); }
  }
  DEVI void stash(const Op &op, float *tile) const {
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
      const float4 v = op.finish4(r[j], post[j]);
      float *d = tile + (4 * kg) * LD + r0 + j * RSTEP;
      d[0] = v.x; d[LD] = v.y; d[2 * LD] = v.z; d[3 * LD] = v.w;
    }
  }
};

// float4 along the fixed dimension (f-contiguous operand): a thread owns one group of
// 4 rows and CNT k's; one 16-byte LDS write per item
template <class Op, int ROWS, int THREADS, int BK>
struct TileLoader<Op, ROWS, THREADS, BK, LOAD_VEC_F> {
  static constexpr int LD = ROWS + 4;
  static constexpr int FG = ROWS / 4, KSTEP = THREADS / FG, CNT = BK / KSTEP;
  static_assert(THREADS % FG == 0 && BK % KSTEP == 0 && CNT >= 1, "vec-f loader mapping");
  typename Op::FC4 fc;
  typename Op::Post4 post[CNT];
  float4 r[CNT];
  int fg, kq;
  DEVI void init(const Op &op, int z, int row0, int nrows) {
    fg = threadIdx.x % FG;
    kq = threadIdx.x / FG;
    fc = op.fctx4(z, row0 + 4 * fg, nrows);
  }
  DEVI void fetch(const Op &op, int z, int k0, int kend) {
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
      typename Op::KC kc = op.kctx(z, k0 + kq + j * KSTEP, kend);
      post[j] = op.post4(fc, kc);
      r[j] = op.raw4(fc, kc, post[j]);
    }
  }
  DEVI void stash(const Op &op, float *tile) const {
#pragma unroll
    for (int j = 0; j < CNT; ++j)
      *reinterpret_cast<float4 *>(tile + (kq + j * KSTEP) * LD + 4 * fg) = op.finish4(r[j], post[j]);
  }
};

// Problem P provides:
//   int M, N, K, k_chunk (multiple of 32), tiles_n, tiles, splits, groups (set by the launcher);
//   A a; B b;               operand functors (kLanesAlongK, kVec; FC/KC contexts, load or load4)
//   static constexpr bool kReduce;
//   kReduce == false:  void store(int z, int split, int m, int n, float acc) const;
//   kReduce == true:   float contrib(int z, int m, int n, float acc) const;
//                      void store_tile(int z, int tile, float sum) const;
// TAIL: the K range of a block may end inside a tile (K or the split length is no multiple of 32); the last tile then
// multiplies only the k pairs that hold data.  (A separate instantiation: the extra branch costs the full-tile loop
// of the other one some of its scheduling.)
template <class Cfg, class P, bool TAIL = false>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_tile_kernel(const P p) {
  typedef TileLoader<typename P::A, Cfg::BM, Cfg::THREADS, Cfg::BK> LoadA;
  typedef TileLoader<typename P::B, Cfg::BN, Cfg::THREADS, Cfg::BK> LoadB;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, LDA = LoadA::LD, LDB = LoadB::LD;
  __shared__ __attribute__((aligned(16))) float As[BK * LDA];
  __shared__ __attribute__((aligned(16))) float Bs[BK * LDB];
  __shared__ float red[Cfg::WM * Cfg::WN];

  // XCD-aware placement.  Workgroups go round-robin to the 8 XCDs (each with its own L2) in
  // order of their linear id, so id % 8 names the XCD.  All tiles of one (batch item, K split)
  // read the same operand data: they are given to ONE XCD, back to back, so that data comes
  // from HBM once and from that L2 afterwards.  With fewer than 8 such groups the tiles of a
  // group are cut into 8 contiguous bands instead (neighbouring tiles share an operand).
  int z, split, tile;
  {
    const int L = blockIdx.x, xcd = L & 7, j = L >> 3;
    const int ngroups = p.groups;
    if (ngroups >= 8) {
      const int q = j / p.tiles;
      const int g = q * 8 + xcd;
      tile = j - q * p.tiles;
      if (g >= ngroups) return;
      z = g / p.splits; split = g - z * p.splits;
    } else {
      const int band = (p.tiles + 7) >> 3;
      const int g = j / band;
      tile = xcd * band + (j - g * band);
      if (g >= ngroups || tile >= p.tiles) return;
      z = g / p.splits; split = g - z * p.splits;
    }
  }
  const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int kbeg = split * p.k_chunk;
  const int kend = min(p.K, kbeg + p.k_chunk);

  LoadA la;
  LoadB lb;
  la.init(p.a, z, m0, p.M);
  lb.init(p.b, z, n0, p.N);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / Cfg::WN, wn = wave - wm * Cfg::WN;
  const int li = lane & 31, lk = lane >> 5;

  f32x16 acc[Cfg::MB][Cfg::NB];
#pragma unroll
  for (int i = 0; i < Cfg::MB; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (kbeg < kend) {
    la.fetch(p.a, z, kbeg, kend);
    lb.fetch(p.b, z, kbeg, kend);
  }
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    la.stash(p.a, As);
    lb.stash(p.b, Bs);
    __syncthreads();
    if (k0 + BK < kend) {
      la.fetch(p.a, z, k0 + BK, kend);
      lb.fetch(p.b, z, k0 + BK, kend);
    }
    auto kstep = [&](int ks) {
      float av[Cfg::MB], bv[Cfg::NB];
#pragma unroll
      for (int i = 0; i < Cfg::MB; ++i) av[i] = As[(ks + lk) * LDA + wm * Cfg::TM + i * 32 + li];
#pragma unroll
      for (int j = 0; j < Cfg::NB; ++j) bv[j] = Bs[(ks + lk) * LDB + wn * Cfg::TN + j * 32 + li];
#pragma unroll
      for (int i = 0; i < Cfg::MB; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
    };
    if (!TAIL || k0 + BK <= kend) {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 2) kstep(ks);
    } else {
      // the last, partial tile of K: only the k pairs that hold data (the rest of the tile is zeros), so a K of
      // 100 costs 3 1/8 tiles of multiplies, not 4
      const int kl = kend - k0;
      for (int ks = 0; ks < kl; ks += 2) kstep(ks);
    }
    __syncthreads();
  }

  // accumulator layout of the 32x32 block: lane holds column (lane % 32) and
  // rows 8*(r/4) + 4*(lane/32) + r%4 for r = 0..15
  float part = 0.f;
#pragma unroll
  for (int i = 0; i < Cfg::MB; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::NB; ++j) {
      const int n = n0 + wn * Cfg::TN + j * 32 + li;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * Cfg::TM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        if (m < p.M && n < p.N) {
          if constexpr (P::kReduce) part += p.contrib(z, m, n, acc[i][j][r]);
          else p.store(z, split, m, n, acc[i][j][r]);
        }
      }
    }
  if constexpr (P::kReduce) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
    if (lane == 0) red[wave] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
      float s = 0.f;
      for (int w = 0; w < Cfg::WM * Cfg::WN; ++w) s += red[w];
      p.store_tile(z, split * p.tiles + tile, s);
    }
  }
}

struct GemmShape {
  int bm, bn, tiles_m, tiles_n;
};

static inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

// Picks the tile for an M x N output: the largest that does not waste more than
// it must, shrinking while the launch would leave most of the 256 CUs idle.
static inline GemmShape pick_tile(int M, int N, long other_blocks, bool waste_aware = true) {
  int bm = M <= 32 ? 32 : (M <= 64 ? 64 : 128);
  int bn = N <= 32 ? 32 : (N <= 64 ? 64 : 128);
  auto blocks = [&](int a, int b) { return (long)ceil_div(M, a) * ceil_div(N, b) * other_blocks; };
  // allowed shapes: 32x32 64x64 128x128 32x128 128x32 64x128 128x64
  if (bm == 32 && bn == 64) bn = N <= 48 ? 32 : 128;
  if (bm == 64 && bn == 32) bm = M <= 48 ? 32 : 128;
  if (bm == 128 && bn == 128) {
    // a 64-wide side where it cuts the padded area by more than the smaller tile costs (measured: about 10 %)
    if (waste_aware) {
      auto padded = [&](int a, int b) { return (double)ceil_div(M, a) * a * ceil_div(N, b) * b; };
      const double full = padded(128, 128);
      if (padded(128, 64) < 0.9 * full) bn = 64;
      else if (padded(64, 128) < 0.9 * full) bm = 64;
    }
  }
  while (blocks(bm, bn) < 512) {
    if (bm == 128 && bn == 128) { bm = bn = 64; }
    else if (bm == 64 && bn == 64) { bm = bn = 32; }
    else if (bm == 128 && bn == 64) { bm = 64; }
    else if (bm == 64 && bn == 128) { bn = 64; }
    else break;
  }
  GemmShape s = {bm, bn, ceil_div(M, bm), ceil_div(N, bn)};
  return s;
}

// Launches the instantiation that matches the tile shape.  L is a callable
// (label, grid, block, launch-on-stream) supplied by the step so that timing
// events can bracket the launch.
template <class P, class Launcher>
static inline void launch_gemm_shape(P p, GemmShape s, int batch, int splits, Launcher &&L, const char *label) {
  p.tiles_n = s.tiles_n;
  p.tiles = s.tiles_m * s.tiles_n;
  p.splits = splits;
  p.groups = splits * batch;
  // ngroups >= 8: ceil(groups/8) rounds of 8 groups x tiles; else groups x 8 bands of ceil(tiles/8)
  const long nblk = p.groups >= 8 ? (long)ceil_div(p.groups, 8) * 8 * p.tiles
                                  : (long)p.groups * 8 * ceil_div(p.tiles, 8);
  dim3 grid((unsigned)nblk);
  const bool tail = (p.K % 32) != 0; // (k_chunk is a multiple of 32: only the end of K can fall inside a tile)
#define DP_GEMM_CASE(bm_, bn_, wm_, wn_)                                                    \
  if (s.bm == bm_ && s.bn == bn_) {                                                         \
    typedef TileCfg<bm_, bn_, wm_, wn_> Cfg;                                                \
    L(label, grid, dim3(Cfg::THREADS), [&](hipStream_t st) {                                \
      if (tail) hipLaunchKernelGGL((gemm_tile_kernel<Cfg, P, true>), grid, dim3(Cfg::THREADS), 0, st, p);  \
      else hipLaunchKernelGGL((gemm_tile_kernel<Cfg, P, false>), grid, dim3(Cfg::THREADS), 0, st, p);      \
    });                                                                                     \
    return;                                                                                 \
  }
  DP_GEMM_CASE(128, 128, 2, 2)
  DP_GEMM_CASE(64, 64, 2, 2)
  DP_GEMM_CASE(32, 32, 1, 1)
  DP_GEMM_CASE(32, 128, 1, 4)
  DP_GEMM_CASE(128, 32, 4, 1)
  DP_GEMM_CASE(64, 128, 2, 2)
  DP_GEMM_CASE(128, 64, 2, 2)
#undef DP_GEMM_CASE
}

// one K range per block, `batch` independent problems
template <class P, class Launcher>
static inline GemmShape launch_gemm(P p, int batch, Launcher &&L, const char *label) {
  GemmShape s = pick_tile(p.M, p.N, batch, L.waste_aware());
  p.k_chunk = (p.K + 31) / 32 * 32;
  launch_gemm_shape(p, s, batch, 1, L, label);
  return s;
}

// split-K: aims for ~1024 workgroups with at least 64 of K per split; returns the split count
template <class P, class Launcher>
static inline int launch_gemm_split(P p, int max_split, Launcher &&L, const char *label) {
  long by_k = p.K / 64;
  if (by_k < 1) by_k = 1;
  if (by_k > max_split) by_k = max_split;
  GemmShape s = pick_tile(p.M, p.N, by_k, L.waste_aware());
  long tiles = (long)s.tiles_m * s.tiles_n;
  // a handful of tiles: the launch is one serial chain of loads per workgroup, so the shortest chunks the kernel
  // takes (32) halve its duration
  if (tiles <= 4 && p.K / 32 > by_k) by_k = std::min<long>(p.K / 32, max_split);
  long want = (1024 + tiles - 1) / tiles;
  int nsplit = (int)(want < by_k ? want : by_k);
  p.k_chunk = ceil_div(ceil_div(p.K, nsplit), 32) * 32;
  nsplit = ceil_div(p.K, p.k_chunk);
  launch_gemm_shape(p, s, 1, nsplit, L, label);
  return nsplit;
}

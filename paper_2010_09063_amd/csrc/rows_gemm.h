// C[M x N] = A[M x K] W  for a very tall A (one row per example and time step) and a small weight matrix: the LSTM's
// input projection (gates = x W_ih + b) and the gradient w.r.t. its input (dx = dgates W_ih^T), Appendix B's LSTM
// layer under Section 1's per-example backward pass.
//
// The weight matrix never goes through LDS: every wave keeps its share of it in registers, already in the layout
// of the MFMA's B operand (v_mfma_f32_16x16x4_f32: lane (n = lane % 16, k = lane / 16) of a k-step), for the whole
// life of the workgroup -- up to 100 registers a lane.  A workgroup of eight waves is persistent: it walks over
// tiles of 32 or 64 rows, staging rows x 100 floats of A per chunk in LDS (row-major with a row length of 100 words, which
// puts the 64 lanes of an A-operand read on 64 different banks), two buffers, one barrier per chunk, the next chunk
// in flight in registers meanwhile.  Wave w owns NBW blocks of 16 output columns for all 16-row blocks of the
// tile: NBW = 4 and one chunk per tile for the input projection (K = 100, N = 400), NBW = 1 and four chunks per
// tile for the input gradient (K = 400, N = 100).  With 16-wide blocks N = 400 and K = 100 are covered without
// padding (tiles of 32x32 blocks and 32-deep K tiles pad this work by a third).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

typedef float rg_f32x4 __attribute__((ext_vector_type(4)));

#define RG_THREADS 512
#define RG_KC 100    // columns of A per chunk (25 k-steps of 4)

struct RowsGemmArgs {
  const float *A;    // [M][K] row-major
  const float *W;    // B operand: element (k, n) = W[k * w_sk + n * w_sn]
  long w_sk, w_sn;
  const float *bias; // [N] added to every row, or null
  float *C;          // [M][N] row-major
  long M;
  int K, N;
};

// NBW column blocks per wave, NCH chunks of RG_KC columns of A per tile, MBT 16-row blocks per tile (the register
// budget decides: 100 weight registers + 16 NBW MBT accumulators + the chunk in flight must stay under 256)
template <int NBW, int NCH, int MBT>
__global__ __launch_bounds__(RG_THREADS) void rows_gemm_kernel(const RowsGemmArgs a) {
  constexpr int RG_ROWS = 16 * MBT;                                              // rows of A per tile
  constexpr int RG_ITEMS = (RG_ROWS * (RG_KC / 4) + RG_THREADS - 1) / RG_THREADS; // groups of four floats a thread stages per chunk
  extern __shared__ float lds[]; // two buffers of [RG_ROWS][RG_KC]
  const int tid = threadIdx.x, lane = tid & 63, i16 = lane & 15, kq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, N = a.N;
  const int n_blk0 = wave * NBW;

  // ---- this wave's share of W as B-operand fragments: w[chunk][k-step][column block]
  float w[NCH][RG_KC / 4][NBW];
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int ks = 0; ks < RG_KC / 4; ++ks)
#pragma unroll
      for (int j = 0; j < NBW; ++j) {
        const int k = c * RG_KC + 4 * ks + kq, n = (n_blk0 + j) * 16 + i16;
        const bool ok = k < K && n < N;
        const float v = a.W[ok ? k * a.w_sk + n * a.w_sn : 0];
        w[c][ks][j] = ok ? v : 0.f;
      }
  float bv[NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    const int n = (n_blk0 + j) * 16 + i16;
    const float v = a.bias ? a.bias[n < N ? n : 0] : 0.f;
    bv[j] = n < N ? v : 0.f;
  }

  // ---- staging items, fixed per thread: (row of the tile, group of four columns of the chunk)
  int s_lds[RG_ITEMS], s_row[RG_ITEMS], s_col[RG_ITEMS];
#pragma unroll
  for (int q = 0; q < RG_ITEMS; ++q) {
    const int it = tid + q * RG_THREADS, row = it / (RG_KC / 4), g = it - row * (RG_KC / 4);
    s_lds[q] = row < RG_ROWS ? row * RG_KC + 4 * g : -1;
    s_row[q] = row;
    s_col[q] = 4 * g;
  }
  const long n_tiles = (a.M + RG_ROWS - 1) / RG_ROWS;
  const long n_items = n_tiles * NCH; // item = (tile, chunk), chunks of a tile consecutive
  float4 ra[RG_ITEMS];
  auto fetch = [&](long item) { // unconditional loads from valid addresses; masked when written to LDS
    const long tile = item / NCH;
    const int kc = (int)(item - tile * NCH) * RG_KC;
#pragma unroll
    for (int q = 0; q < RG_ITEMS; ++q) {
      const long row = tile * RG_ROWS + s_row[q];
      const bool ok = s_lds[q] >= 0 && row < a.M && kc + s_col[q] < K;
      ra[q] = *reinterpret_cast<const float4 *>(a.A + (ok ? row * K + kc + s_col[q] : 0));
    }
  };
  auto stash = [&](float *As, long item) {
    const long tile = item / NCH;
    const int kc = (int)(item - tile * NCH) * RG_KC;
#pragma unroll
    for (int q = 0; q < RG_ITEMS; ++q) {
      const long row = tile * RG_ROWS + s_row[q];
      const bool ok = row < a.M && kc + s_col[q] < K; // K is a multiple of 4: a group is inside or outside
      float4 v = ra[q];
      v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
      if (s_lds[q] >= 0) *reinterpret_cast<float4 *>(As + s_lds[q]) = v;
    }
  };

  rg_f32x4 acc[MBT][NBW];
  long item = (long)blockIdx.x * NCH;
  const long stride = (long)gridDim.x * NCH;
  if (item < n_items) fetch(item);
  int buf = 0;
  for (; item < n_items; item += (item % NCH == NCH - 1) ? stride - (NCH - 1) : 1) {
    const int c = (int)(item % NCH);
    float *As = lds + buf * (RG_ROWS * RG_KC);
    stash(As, item);
    __syncthreads(); // this chunk is staged; every wave has finished the chunk before (it stashed after its multiplies)
    const long next = (c == NCH - 1) ? item + stride - (NCH - 1) : item + 1;
    if (next < n_items) fetch(next);
    if (c == 0) {
#pragma unroll
      for (int i = 0; i < MBT; ++i)
#pragma unroll
        for (int j = 0; j < NBW; ++j) acc[i][j] = (rg_f32x4){0.f, 0.f, 0.f, 0.f};
    }
    const float *ap = As + i16 * RG_KC + kq;
    auto chunk = [&](auto cc_) {
      constexpr int CC = decltype(cc_)::value;
#pragma unroll
      for (int ks = 0; ks < RG_KC / 4; ++ks) {
        float av[MBT];
#pragma unroll
        for (int i = 0; i < MBT; ++i) av[i] = ap[i * 16 * RG_KC + 4 * ks];
#pragma unroll
        for (int i = 0; i < MBT; ++i)
#pragma unroll
          for (int j = 0; j < NBW; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], w[CC][ks][j], acc[i][j], 0, 0, 0);
      }
    };
    // the chunk index selects registers, so it must be a constant where the weights are indexed
    if constexpr (NCH == 1) chunk(std::integral_constant<int, 0>{});
    else {
      if (c == 0) chunk(std::integral_constant<int, 0>{});
      else if (c == 1) chunk(std::integral_constant<int, 1 % NCH>{});
      else if (c == 2) chunk(std::integral_constant<int, 2 % NCH>{});
      else chunk(std::integral_constant<int, 3 % NCH>{});
    }
    if (c == NCH - 1) { // the tile is complete: accumulator register r of a lane is row 4 kq + r, column i16 of its block
      const long row0 = (item / NCH) * RG_ROWS;
#pragma unroll
      for (int i = 0; i < MBT; ++i)
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
          const int n = (n_blk0 + j) * 16 + i16;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const long row = row0 + i * 16 + 4 * kq + r;
            if (row < a.M && n < N) a.C[row * N + n] = acc[i][j][r] + bv[j];
          }
        }
    }
    buf ^= 1;
  }
}

static inline bool rows_gemm_fits(int K, int N, int nbw, int nch) {
  return K >= 4 && (K & 3) == 0 && K <= nch * RG_KC && N >= 1 && N <= 8 * nbw * 16;
}
static inline size_t rows_gemm_lds_bytes(int mbt) { return sizeof(float) * 2 * 16 * mbt * RG_KC; }

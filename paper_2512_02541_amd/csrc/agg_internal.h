// Internal declarations shared by the host API and the HIP kernels of libagg.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "agg.h"

namespace agg {

constexpr int kHeadDim = 64;    // the only head dimension the kernels are written for
constexpr int kTileRows = 64;   // compacted rows per fragment-order tile
constexpr int kTileElems = kTileRows * kHeadDim;  // 4096 bf16 = 8 KiB

// Geometry derived once on the host and passed to kernels by value.
struct Geom {
  int32_t B, N, L, P, n_h, n_w, H;
  int32_t s_h, s_w;
  int32_t keep_first;   // 1 when frame 0 is kept whole
  int32_t kw;           // kept patch columns per grid row  = ceil(n_w / s_w)
  int32_t kf;           // kept patches per subsampled frame = ceil(n_h/s_h) * kw
  int32_t rows_sub;     // kept rows per subsampled frame    = P + kf
  int32_t dw;           // dropped patches in a grid row that keeps some columns = n_w - kw
  int32_t df;           // dropped patches per subsampled frame = n_h*n_w - kf
  int64_t NQ;           // tokens per sequence = N * L
  int64_t M;            // kept rows per sequence
  int64_t M_pad;        // M rounded up to a multiple of kTileRows
  int64_t n_dropped;    // dropped patches per sequence
};

// Compacted row m (0 <= m < M)  ->  token id of the sequence.  The kept set in
// ascending order is: frame 0 whole (if kept), then per frame its special tokens
// followed by the kept patches in row-major order (Sec. 4.3).
__host__ __device__ inline int64_t kept_row_to_token(const Geom& g, int64_t m) {
  int64_t frame;
  int32_t j;
  // m < M <= N*L < 2^31: 32-bit division (much cheaper on the GPU than 64-bit)
  if (g.keep_first) {
    if (m < g.L) return m;
    const uint32_t r = (uint32_t)(m - g.L);
    frame = 1 + (int64_t)(r / (uint32_t)g.rows_sub);
    j = (int32_t)(r % (uint32_t)g.rows_sub);
  } else {
    const uint32_t r = (uint32_t)m;
    frame = (int64_t)(r / (uint32_t)g.rows_sub);
    j = (int32_t)(r % (uint32_t)g.rows_sub);
  }
  int32_t slot;
  if (j < g.P) {
    slot = j;
  } else {
    int32_t q = j - g.P;
    int32_t row = (q / g.kw) * g.s_h;
    int32_t col = (q % g.kw) * g.s_w;
    slot = g.P + row * g.n_w + col;
  }
  return frame * g.L + slot;
}

// Dropped patch number u (0 <= u < n_dropped, ascending token order) -> token id.
// A grid row r with r % s_h != 0 is dropped entirely (n_w patches); a row with
// r % s_h == 0 drops the columns c with c % s_w != 0 (dw patches).
__host__ __device__ inline int64_t dropped_to_token(const Geom& g, int64_t u) {
  // u < n_dropped <= N*L < 2^31: 32-bit division (much cheaper on the GPU than 64-bit)
  const uint32_t uu = (uint32_t)u;
  int64_t frame = (g.keep_first ? 1 : 0) + (int64_t)(uu / (uint32_t)g.df);
  int32_t j = (int32_t)(uu % (uint32_t)g.df);
  // rows come in groups of s_h: the first keeps some columns, the rest are dropped whole
  int32_t per_group = g.dw + (g.s_h - 1) * g.n_w;  // > 0 whenever anything is dropped
  if (per_group < 1) per_group = 1;
  int32_t grp = j / per_group;
  int32_t w = j % per_group;
  int32_t row, col;
  if (w < g.dw) {
    row = grp * g.s_h;
    // w-th column with c % s_w != 0:  c = w + w/(s_w-1) + 1
    col = w + w / (g.s_w > 1 ? g.s_w - 1 : 1) + 1;
  } else {
    int32_t x = w - g.dw;
    row = grp * g.s_h + 1 + x / g.n_w;
    col = x % g.n_w;
  }
  return frame * g.L + g.P + (int64_t)row * g.n_w + col;
}

// 1 when token `tok` is a patch that is not in the kept set.
__host__ __device__ inline int token_is_dropped(const Geom& g, int64_t tok) {
  int64_t frame = tok / g.L;
  int32_t slot = (int32_t)(tok % g.L);
  if (slot < g.P) return 0;
  if (frame == 0 && g.keep_first) return 0;
  int32_t p = slot - g.P;
  int32_t row = p / g.n_w, col = p % g.n_w;
  return (row % g.s_h != 0) || (col % g.s_w != 0);
}

// Element offsets of (row m, channel d) inside one (batch, head) block of the
// fragment-order compacted tensors (documented in agg.h).
__host__ __device__ inline int64_t kc_offset(int64_t m, int32_t d) {
  int64_t tile = m / kTileRows;
  int32_t km = (int32_t)(m % kTileRows);
  int32_t chunk = (((km / 32) * 4 + d / 16) * 2 + (d % 16) / 8) * 32 + km % 32;
  return tile * kTileElems + chunk * 8 + d % 8;
}
__host__ __device__ inline int64_t vc_offset(int64_t m, int32_t d) {
  int64_t tile = m / kTileRows;
  int32_t km = (int32_t)(m % kTileRows);
  int32_t u = km % 16;
  int32_t chunk = ((km / 16) * 2 + (u % 8) / 4) * 64 + d;
  return tile * kTileElems + chunk * 8 + (u / 8) * 4 + u % 4;
}

// Host-side validation + geometry (agg_api.cpp).
int make_geom(const agg_shape* s, Geom* g, bool dense);

// Kernel launchers (each returns hipGetLastError() of its launches).
// gather + index list, and (when kmean/vmean are non-null) the mean terms
hipError_t launch_subsample(const Geom& g, const void* K, const void* V, void* Kc, void* Vc,
                            int32_t* idx, float* kmean, float* vmean, void* workspace,
                            hipStream_t st);
hipError_t launch_attn(const Geom& g, uint32_t flags, float scale, float mean_bias, const void* Q,
                       const void* K, const void* V, const void* Kc, const void* Vc,
                       const float* kmean, const float* vmean, void* O, float* lse, hipStream_t st,
                       const uint32_t* kept_bits = nullptr, const int32_t* nd_dev = nullptr,
                       int src_mode = 0, const int32_t* list = nullptr, int64_t list_stride = 0);
// src_mode of launch_attn: where the key/value tiles come from
enum { kAttnSrcCompact = 0,   // Kc/Vc in fragment order
       kAttnSrcRows = 1,      // every token of K/V, in place (ordinary and per-frame attention)
       kAttnSrcIndexed = 2 }; // the rows of K/V that `list` names, in place

// Caller-supplied kept lists: g.M / g.M_pad hold the list length.
int64_t list_words(const Geom& g);               // uint32 words of one batch element's bitmap
size_t list_workspace_bytes(const Geom& g);
hipError_t launch_subsample_list(const Geom& g, const int32_t* list, const void* K, const void* V,
                                 void* Kc, void* Vc, float* kmean, float* vmean, uint32_t* bits,
                                 int32_t* nd_out, void* workspace, hipStream_t st);
hipError_t launch_select(const Geom& g, int rule, uint64_t seed, const void* K, int32_t* list,
                         hipStream_t st);
// compacted set whose rows are window means (cell-mean variant)
hipError_t launch_pool(const Geom& g, const void* K, const void* V, void* Kc, void* Vc,
                       hipStream_t st);

hipError_t launch_layernorm(const void* x, const float* gamma, const float* beta, void* y,
                            int64_t rows, int C, float eps, hipStream_t st);
// Y_i[rows, N] = A[rows, K] W_i[N, K]^T + bias_i (+ R) for i < count (1..3 weight matrices
// applied to the same input in one launch); bf16 tensors, float bias (may be null)
struct LinearOuts {
  const uint16_t* W[3];
  const float* bias[3];
  uint16_t* Y[3];
  int count;
};
hipError_t launch_linear(const void* A, const LinearOuts& outs, const void* R, int64_t rows, int N,
                         int K, hipStream_t st);

int mean_chunks(const Geom& g);  // number of partial-sum blocks the mean kernel uses

// Device array inside the library that stands in for the caller's workspace in
// agg_kv_subsample_static; static_scratch() returns its address on the current device.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
hipError_t static_scratch(void** ptr);

}  // namespace agg

// Grid gather and mean-fill reduction (Sec. 4.3 of the AVGGT paper: only the
// kept subset serves as keys/values; all dropped patches are summarised by one
// mean key/value pair).  HBM-bandwidth bound: one launch reads every K and V
// row exactly once (kept rows are copied, dropped rows are summed) and writes
// the kept rows once, in the fragment order agg.h documents.  Workgroups of
// that launch take one of two roles -- repack a 64-row tile of the compacted
// set, or sum a run of dropped rows -- so that both kinds of traffic share the
// memory system at the same time; a second, small launch adds the partial sums.
#include <atomic>

#include "agg_internal.h"

namespace agg {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSubThreads = 256;
constexpr int kHeadGroup = 4;  // heads repacked per workgroup: 64 rows x 4 heads x 128 B = 32 KiB
constexpr int kVPad = 72;      // padded row length (elements) of the raw V rows in LDS
constexpr int kVHead = kTileRows * kVPad + 64;  // elements between two heads' V rows in LDS

// LDS of the gather role
struct GatherLds {
  uint16_t k[kHeadGroup][kTileElems];        // K in fragment order
  // raw V rows, padded to kVPad; heads are a further 128 bytes apart so that the two heads a
  // 16-lane LDS access covers start in different halves of the 256-byte bank period
  uint16_t v[kHeadGroup * kVHead];
  int64_t tok[kTileRows];
  int32_t win[kTileRows];  // pooled variant: window rows << 8 | window columns of the row's cell
};

// Where fragment-order slot `slot` of head hl waits in LDS.  The 16 lanes that the 64-bank LDS
// serves together hold, on the fill side, the eight chunks of one row for two heads: their
// slots differ only in bits 5..7 (and in the head), so those bits are folded into the low four;
// the drain side reads 16 consecutive slots, which the fold permutes among themselves.
__device__ inline int k_lds_pos(int slot, int hl) {
  return slot ^ (((slot >> 5) & 7) | ((hl & 1) << 3));
}

// Gather role: one 64-row tile of the compacted set for kHeadGroup heads.  Reads are
// 128-byte row segments (512 B contiguous per token for the four heads); writes are whole
// 8 KiB tiles, fully coalesced.  K chunks are routed through LDS to their fragment-order
// slot; V is transposed through LDS (the PV MFMA wants eight keys of one channel in one
// 16-byte operand).
// Mean of `cells` 16-byte chunks of bf16 (a window's tokens at the same head and channels), in
// float, rounded to bf16 once.
__device__ inline u32x4 window_mean(const uint16_t* __restrict__ T, int64_t off0, int64_t row_stride,
                                    int64_t cell_stride, int wrows, int wcols) {
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int r = 0; r < wrows; ++r)
    for (int c = 0; c < wcols; ++c) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(T + off0 + r * row_stride + c * cell_stride);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += __uint_as_float(v[i] << 16);
        acc[2 * i + 1] += __uint_as_float(v[i] & 0xFFFF0000u);
      }
    }
  const float inv = 1.0f / (float)(wrows * wcols);
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  u32x4 out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f32x2 pr = {acc[2 * i] * inv, acc[2 * i + 1] * inv};
    out[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
  }
  return out;
}

// kPool: a kept patch of a subsampled frame stands for its whole window and the row written is
// the window's mean (the cell-mean variant of the supplementary ablation) instead of a copy.
template <bool kPool = false>
__device__ inline void gather_tile(const Geom& g, const uint16_t* __restrict__ K,
                                   const uint16_t* __restrict__ V, uint16_t* __restrict__ Kc,
                                   uint16_t* __restrict__ Vc, int32_t* __restrict__ idx,
                                   const int32_t* __restrict__ list, int64_t tile, int hgrp, int b,
                                   GatherLds& s) {
  const int tid = threadIdx.x;
  const int h0 = hgrp * kHeadGroup;
  const int64_t m0 = tile * kTileRows;
  const int nheads = min(kHeadGroup, g.H - h0);

  if (tid < kTileRows) {
    int64_t m = m0 + tid;
    int64_t tok = -1;
    if (m < g.M) {
      if (list) {  // caller's list: clamp so that a bad id cannot leave the tensor
        int64_t t = list[(int64_t)b * g.M + m];
        tok = t < 0 ? 0 : (t >= g.NQ ? g.NQ - 1 : t);
      } else {
        tok = kept_row_to_token(g, m);
      }
    }
    s.tok[tid] = tok;
    if (kPool) {
      int32_t win = (1 << 8) | 1;
      if (tok >= 0) {
        const int64_t frame = tok / g.L;
        const int32_t slot = (int32_t)(tok % g.L);
        if (slot >= g.P && !(frame == 0 && g.keep_first)) {
          const int32_t r = (slot - g.P) / g.n_w, c = (slot - g.P) % g.n_w;
          win = (min(g.s_h, g.n_h - r) << 8) | min(g.s_w, g.n_w - c);
        }
      }
      s.win[tid] = win;
    }
    if (idx && b == 0 && hgrp == 0 && m < g.M) idx[m] = (int32_t)tok;
  }
  __syncthreads();

  // stage 1: 16-byte chunks, (row, head, j) with j the fastest index
  const int chunks = kTileRows * nheads * 8;
  for (int c = tid; c < chunks; c += kSubThreads) {
    int j = c & 7;
    int hl = (c >> 3) % nheads;
    int row = (c >> 3) / nheads;
    int64_t tok = s.tok[row];
    u32x4 kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
    if (tok >= 0) {
      int64_t off = (((int64_t)b * g.NQ + tok) * g.H + (h0 + hl)) * kHeadDim + j * 8;
      if (kPool && s.win[row] != ((1 << 8) | 1)) {
        const int wrows = s.win[row] >> 8, wcols = s.win[row] & 255;
        const int64_t cell = (int64_t)g.H * kHeadDim;  // elements between neighbouring tokens
        kv = window_mean(K, off, cell * g.n_w, cell, wrows, wcols);
        vv = window_mean(V, off, cell * g.n_w, cell, wrows, wcols);
      } else {
        kv = *reinterpret_cast<const u32x4*>(K + off);
        vv = *reinterpret_cast<const u32x4*>(V + off);
      }
    }
    // K: chunk j covers channels 8j..8j+7 -> slot (((row/32)*4 + j/2)*2 + j%2)*32 + row%32
    int kslot = (((row >> 5) * 4 + (j >> 1)) * 2 + (j & 1)) * 32 + (row & 31);
    *reinterpret_cast<u32x4*>(&s.k[hl][k_lds_pos(kslot, hl) * 8]) = kv;
    *reinterpret_cast<u32x4*>(&s.v[hl * kVHead + row * kVPad + j * 8]) = vv;
  }
  __syncthreads();

  // stage 2: linear, coalesced tile writes
  const int64_t ntiles = g.M_pad / kTileRows;
  const int out_chunks = nheads * (kTileElems / 8);
  for (int c = tid; c < out_chunks; c += kSubThreads) {
    int hl = c / (kTileElems / 8);
    int slot = c % (kTileElems / 8);
    int64_t base = (((int64_t)b * g.H + (h0 + hl)) * ntiles + tile) * kTileElems + slot * 8;
    *reinterpret_cast<u32x4*>(Kc + base) =
        *reinterpret_cast<const u32x4*>(&s.k[hl][k_lds_pos(slot, hl) * 8]);
    // V slot = (t*2 + gg)*64 + d holds rows 16t + 8*(e/4) + 4gg + e%4, e = 0..7, of channel d
    int d = slot & 63;
    int gg = (slot >> 6) & 1;
    int t = slot >> 7;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      int ea = 2 * e2, eb = 2 * e2 + 1;
      int ra = 16 * t + 8 * (ea >> 2) + 4 * gg + (ea & 3);
      int rb = 16 * t + 8 * (eb >> 2) + 4 * gg + (eb & 3);
      w[e2] = (uint32_t)s.v[hl * kVHead + ra * kVPad + d] |
              ((uint32_t)s.v[hl * kVHead + rb * kVPad + d] << 16);
    }
    u32x4 out = {w[0], w[1], w[2], w[3]};
    *reinterpret_cast<u32x4*>(Vc + base) = out;
  }
}

// ---------------------------------------------------------------------------
// Mean component.  Stage 1 (mean role below): a workgroup sums a run of
// consecutive dropped rows (all H*64 channels of K and of V) in a fixed order
// and writes one partial.  Stage 2 (mean_final_kernel): the partials are added
// in a fixed order, in double, and divided by the number of dropped patches.
// No atomics: the result is bit-reproducible.
// ---------------------------------------------------------------------------
constexpr int kMeanBatch = 256;       // token ids resolved per pass through LDS
constexpr int kMeanMaxChunks = 4096;  // upper bound on partials per batch element

struct MeanLds {
  float red[kSubThreads][17];
  int32_t tok[kMeanBatch];
  int32_t wcnt[kSubThreads / 64];
};

// Geometry of the mean role, derived on the host
struct MeanPlan {
  int nchunks;         // partials per batch element
  int rows_per_chunk;  // dropped rows per partial
  int cpr_b;           // 16-byte chunks of a row handled by one workgroup (<= 256)
  int rpp;             // rows in flight per pass = 256 / cpr_b
  int ncolblk;         // workgroups side by side to cover a row (1 unless H > 32)
};

static MeanPlan mean_plan(const Geom& g) {
  MeanPlan p;
  // At least 512 rows per partial, at most kMeanMaxChunks partials.  Measured at 100 / 300 / 800
  // frames: 32 rows per partial 0.190 / 0.455 / 0.937 ms per call, 128: 0.184 / 0.446 / 0.937,
  // 512: 0.175 / 0.429 / 0.942, 1024: 0.193 / 0.458 / 0.962 (fewer partials are less traffic and a
  // shorter second stage, until single workgroups run long enough to form the tail of the launch).
  constexpr int kMinRowsPerChunk = 512;
  int64_t rows = (g.n_dropped + kMeanMaxChunks - 1) / kMeanMaxChunks;
  p.rows_per_chunk = (int)(rows < kMinRowsPerChunk ? kMinRowsPerChunk : rows);
  p.nchunks = (int)((g.n_dropped + p.rows_per_chunk - 1) / p.rows_per_chunk);
  const int cpr = g.H * kHeadDim / 8;
  p.cpr_b = cpr < kSubThreads ? cpr : kSubThreads;
  p.rpp = kSubThreads / p.cpr_b;
  p.ncolblk = (cpr + kSubThreads - 1) / kSubThreads;
  return p;
}

int mean_chunks(const Geom& g) { return mean_plan(g).nchunks; }

__device__ inline void add_bf16x8(float (&acc)[8], const u32x4& v) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc[2 * i] += __uint_as_float(v[i] << 16);
    acc[2 * i + 1] += __uint_as_float(v[i] & 0xFFFF0000u);
  }
}

// Adds the rows s.tok[0..n) (token ids) of K and V into the thread's accumulators.  Threads
// are laid out as (row lane rl, 16-byte chunk of the row); four rows per lane are requested
// before any is added, so that enough bytes are in flight to cover HBM latency.
__device__ inline void add_rows(const MeanLds& s, int n, int rl, int rpp, int C,
                                const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb,
                                float (&ak)[8], float (&av)[8]) {
  int r = rl;
  for (; r + 3 * rpp < n; r += 4 * rpp) {
    u32x4 kv[4], vv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t off = (int64_t)s.tok[r + j * rpp] * C;
      kv[j] = *reinterpret_cast<const u32x4*>(Kb + off);
      vv[j] = *reinterpret_cast<const u32x4*>(Vb + off);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      add_bf16x8(ak, kv[j]);
      add_bf16x8(av, vv[j]);
    }
  }
  for (; r < n; r += rpp) {
    const int64_t off = (int64_t)s.tok[r] * C;
    u32x4 kv = *reinterpret_cast<const u32x4*>(Kb + off);
    u32x4 vv = *reinterpret_cast<const u32x4*>(Vb + off);
    add_bf16x8(ak, kv);
    add_bf16x8(av, vv);
  }
}

// Combines the row lanes in ascending order (fixed order -> reproducible) and writes the
// workgroup's partial sums.
__device__ inline void write_partial(MeanLds& s, const float (&ak)[8], const float (&av)[8],
                                     float* __restrict__ partial, const MeanPlan& p, int chunk,
                                     int b, int rl, int cg, int col, int C) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    s.red[tid][i] = ak[i];
    s.red[tid][8 + i] = av[i];
  }
  __syncthreads();
  if (rl == 0 && col < C) {
    float sk[8], sv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) sk[i] = sv[i] = 0.f;
    for (int r = 0; r < p.rpp; ++r) {
      int t = r * p.cpr_b + cg;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        sk[i] += s.red[t][i];
        sv[i] += s.red[t][8 + i];
      }
    }
    float* pk = partial + (((int64_t)b * p.nchunks + chunk) * 2 + 0) * C + col;
    float* pv = partial + (((int64_t)b * p.nchunks + chunk) * 2 + 1) * C + col;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pk[i] = sk[i];
      pv[i] = sv[i];
    }
  }
}

// Mean role of the grid rule: the run's dropped rows are numbered arithmetically; their token
// ids are resolved kMeanBatch at a time into LDS (one integer division chain per row instead
// of one per load).
__device__ inline void mean_partial(const Geom& g, const uint16_t* __restrict__ K,
                                    const uint16_t* __restrict__ V, float* __restrict__ partial,
                                    const MeanPlan& p, int chunk, int colblk, int b, MeanLds& s) {
  const int tid = threadIdx.x;
  const int C = g.H * kHeadDim;
  const int cg = tid % p.cpr_b;                        // 16-byte chunk inside this channel block
  const int rl = tid / p.cpr_b;                        // row lane
  const int col = (colblk * kSubThreads + cg) * 8;     // first channel of this thread
  const bool active = (rl < p.rpp) && (col < C);
  const uint16_t* Kb = K + (int64_t)b * g.NQ * C + col;
  const uint16_t* Vb = V + (int64_t)b * g.NQ * C + col;

  float ak[8], av[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) ak[i] = av[i] = 0.f;

  const int64_t u0 = (int64_t)chunk * p.rows_per_chunk;
  const int64_t u1 = min(u0 + p.rows_per_chunk, g.n_dropped);
  for (int64_t base = u0; base < u1; base += kMeanBatch) {
    const int n = (int)min((int64_t)kMeanBatch, u1 - base);
    __syncthreads();  // previous batch consumed
    if (tid < n) s.tok[tid] = (int32_t)dropped_to_token(g, base + tid);
    __syncthreads();
    if (active) add_rows(s, n, rl, p.rpp, C, Kb, Vb, ak, av);
  }
  write_partial(s, ak, av, partial, p, chunk, b, rl, cg, col, C);
}

// Mean role for a caller's list: the run is a range of token ids; a token is summed when it is
// a patch (slot >= P) whose bit in kept_bits is clear.  Each pass tests kMeanBatch candidates
// and packs the survivors' ids into LDS in ascending order (ballot + prefix count).
__device__ inline void mean_partial_bits(const Geom& g, const uint16_t* __restrict__ K,
                                         const uint16_t* __restrict__ V,
                                         const uint32_t* __restrict__ bits, int64_t nwords,
                                         float* __restrict__ partial, int32_t* __restrict__ cnt,
                                         const MeanPlan& p, int chunk, int colblk, int b,
                                         MeanLds& s) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int C = g.H * kHeadDim;
  const int cg = tid % p.cpr_b;
  const int rl = tid / p.cpr_b;
  const int col = (colblk * kSubThreads + cg) * 8;
  const bool active = (rl < p.rpp) && (col < C);
  const uint16_t* Kb = K + (int64_t)b * g.NQ * C + col;
  const uint16_t* Vb = V + (int64_t)b * g.NQ * C + col;
  const uint32_t* bb = bits + (int64_t)b * nwords;

  float ak[8], av[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) ak[i] = av[i] = 0.f;

  const int64_t t0 = (int64_t)chunk * p.rows_per_chunk;
  const int64_t t1 = min(t0 + p.rows_per_chunk, g.NQ);
  int total = 0;
  for (int64_t base = t0; base < t1; base += kMeanBatch) {
    __syncthreads();  // previous batch consumed
    const int64_t t = base + tid;
    bool d = false;
    if (t < t1) {
      const uint32_t slot = (uint32_t)t % (uint32_t)g.L;
      if ((int32_t)slot >= g.P) d = ((bb[t >> 5] >> (t & 31)) & 1u) == 0u;
    }
    const unsigned long long mask = __ballot(d);
    if (lane == 0) s.wcnt[wave] = __popcll(mask);
    __syncthreads();
    int off = 0, n = 0;
#pragma unroll
    for (int w = 0; w < kSubThreads / 64; ++w) {
      if (w < wave) off += s.wcnt[w];
      n += s.wcnt[w];
    }
    if (d) s.tok[off + __popcll(mask & ((1ull << lane) - 1ull))] = (int32_t)t;
    __syncthreads();
    total += n;
    if (active) add_rows(s, n, rl, p.rpp, C, Kb, Vb, ak, av);
  }
  if (tid == 0 && colblk == 0) cnt[(int64_t)b * p.nchunks + chunk] = total;
  write_partial(s, ak, av, partial, p, chunk, b, rl, cg, col, C);
}

union SubLds {
  GatherLds gather;
  MeanLds mean;
};

// One launch, two roles.  Per batch element the first n_mean workgroups sum dropped rows,
// the remaining n_gather repack tiles; n_mean is 0 when no mean is wanted.
__global__ __launch_bounds__(kSubThreads) void subsample_kernel(
    Geom g, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    uint16_t* __restrict__ Kc, uint16_t* __restrict__ Vc, int32_t* __restrict__ idx,
    float* __restrict__ partial, MeanPlan plan, int n_mean, int n_gather, int nhg) {
  __shared__ __align__(16) SubLds lds;
  const int per_b = n_mean + n_gather;
  const int b = blockIdx.x / per_b;
  const int r = blockIdx.x % per_b;
  if (r < n_mean) {
    mean_partial(g, K, V, partial, plan, r / plan.ncolblk, r % plan.ncolblk, b, lds.mean);
  } else {
    const int rr = r - n_mean;
    gather_tile(g, K, V, Kc, Vc, idx, nullptr, rr / nhg, rr % nhg, b, lds.gather);
  }
}

// Second stage of the mean: a workgroup owns 32 consecutive channels (of K or of V); its 32
// row groups each add every 32nd partial in double, then the 32 sums are added in order.
constexpr int kFinalCols = 32;
constexpr int kFinalGroups = 32;
// With `cnt` (list variant) the number of averaged rows is the sum of the per-chunk counts
// and is also written to nd_out[b]; otherwise it is the grid rule's g.n_dropped.
__global__ __launch_bounds__(kFinalCols * kFinalGroups) void mean_final_kernel(
    Geom g, const float* __restrict__ partial, int nchunks, float* __restrict__ kmean,
    float* __restrict__ vmean, const int32_t* __restrict__ cnt, int32_t* __restrict__ nd_out) {
  __shared__ double red[kFinalGroups][kFinalCols];
  __shared__ int64_t nd_s;
  const int C = g.H * kHeadDim;
  const int cl = threadIdx.x % kFinalCols;
  const int rg = threadIdx.x / kFinalCols;
  const int c = blockIdx.x * kFinalCols + cl;  // 0 .. 2C-1 : K channels then V channels
  const int b = blockIdx.y;
  double s = 0.0;
  if (c < 2 * C) {
    const int which = c / C, col = c % C;
    const float* p = partial + ((int64_t)b * nchunks * 2 + which) * C + col;
#pragma unroll 8
    for (int k = rg; k < nchunks; k += kFinalGroups) s += (double)p[(int64_t)k * 2 * C];
  }
  red[rg][cl] = s;
  if (threadIdx.x == 0) {
    int64_t nd = g.n_dropped;
    if (cnt) {
      nd = 0;
      for (int k = 0; k < nchunks; ++k) nd += cnt[(int64_t)b * nchunks + k];
      if (blockIdx.x == 0) nd_out[b] = (int32_t)nd;
    }
    nd_s = nd;
  }
  __syncthreads();
  if (rg == 0 && c < 2 * C) {
    double t = 0.0;
    for (int r = 0; r < kFinalGroups; ++r) t += red[r][cl];
    const int64_t nd = nd_s;
    const float m = (nd > 0) ? (float)(t / (double)nd) : 0.f;
    const int which = c / C, col = c % C;
    (which ? vmean : kmean)[(int64_t)b * C + col] = m;
  }
}

// The index list alone (when no compacted copy is wanted): one thread per kept row.
__global__ __launch_bounds__(kSubThreads) void index_kernel(Geom g, int32_t* __restrict__ idx) {
  const int64_t m = (int64_t)blockIdx.x * kSubThreads + threadIdx.x;
  if (m < g.M) idx[m] = (int32_t)kept_row_to_token(g, m);
}

// Enqueues the gather (+ index list) and, when kmean/vmean are given, the mean terms.  Without
// Kc/Vc only the index list and the mean terms are produced.
hipError_t launch_subsample(const Geom& g, const void* K, const void* V, void* Kc, void* Vc,
                            int32_t* idx, float* kmean, float* vmean, void* workspace,
                            hipStream_t st) {
  const bool want_mean = (kmean != nullptr);
  const bool want_copy = (Kc != nullptr);
  const MeanPlan plan = mean_plan(g);
  const int nhg = (g.H + kHeadGroup - 1) / kHeadGroup;
  const int64_t n_gather = want_copy ? (g.M_pad / kTileRows) * nhg : 0;
  const int64_t n_mean = want_mean ? (int64_t)plan.nchunks * plan.ncolblk : 0;
  const int64_t groups = (n_gather + n_mean) * g.B;
  if (groups > 0x7FFFFFFF || n_gather > 0x3FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  if (!want_copy && idx) {
    hipLaunchKernelGGL(index_kernel, dim3((unsigned)((g.M + kSubThreads - 1) / kSubThreads)),
                       dim3(kSubThreads), 0, st, g, idx);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
  }
  if (groups > 0)
    hipLaunchKernelGGL(subsample_kernel, dim3((unsigned)groups), dim3(kSubThreads), 0, st, g,
                       (const uint16_t*)K, (const uint16_t*)V, (uint16_t*)Kc, (uint16_t*)Vc, idx,
                       (float*)workspace, plan, (int)n_mean, (int)n_gather, nhg);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !want_mean) return e;
  const int C = g.H * kHeadDim;
  dim3 grid2((unsigned)((2 * C + kFinalCols - 1) / kFinalCols), (unsigned)g.B);
  hipLaunchKernelGGL(mean_final_kernel, grid2, dim3(kFinalCols * kFinalGroups), 0, st, g,
                     (const float*)workspace, plan.nchunks, kmean, vmean, (const int32_t*)nullptr,
                     (int32_t*)nullptr);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Scratch for callers that cannot allocate (agg_kv_subsample_static): the partial sums of the
// mean live in a device array that is part of the library's code object.  In host code the
// array's name is only a handle; its device address differs per GPU and is looked up once per
// device (with that device current) and kept.  Nothing in it needs clearing: every partial that
// the second stage reads is written by the first stage of the same call.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> scratch_ptr[kMaxDevices];

hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
  }
  *out = p;
  return hipSuccess;
}

// Cell-mean variant: the compacted set holds, per window, the mean of its tokens.
__global__ __launch_bounds__(kSubThreads) void pool_kernel(Geom g, const uint16_t* __restrict__ K,
                                                           const uint16_t* __restrict__ V,
                                                           uint16_t* __restrict__ Kc,
                                                           uint16_t* __restrict__ Vc, int n_gather,
                                                           int nhg) {
  __shared__ __align__(16) GatherLds lds;
  const int b = blockIdx.x / n_gather;
  const int rr = blockIdx.x % n_gather;
  gather_tile<true>(g, K, V, Kc, Vc, nullptr, nullptr, rr / nhg, rr % nhg, b, lds);
}

hipError_t launch_pool(const Geom& g, const void* K, const void* V, void* Kc, void* Vc,
                       hipStream_t st) {
  const int nhg = (g.H + kHeadGroup - 1) / kHeadGroup;
  const int64_t n_gather = (g.M_pad / kTileRows) * nhg;
  const int64_t groups = n_gather * g.B;
  if (groups > 0x7FFFFFFF || n_gather > 0x3FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();
  hipLaunchKernelGGL(pool_kernel, dim3((unsigned)groups), dim3(kSubThreads), 0, st, g,
                     (const uint16_t*)K, (const uint16_t*)V, (uint16_t*)Kc, (uint16_t*)Vc,
                     (int)n_gather, nhg);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Caller-supplied kept lists (the token-selection ablation of the supplementary material)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bits_clear_kernel(uint32_t* __restrict__ bits, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    bits[i] = 0u;
}

__global__ __launch_bounds__(256) void bits_set_kernel(const int32_t* __restrict__ list, int64_t M,
                                                       int64_t NQ, int64_t nwords, int B,
                                                       uint32_t* __restrict__ bits) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= M * B) return;
  const int64_t b = i / M;
  int64_t t = list[i];
  t = t < 0 ? 0 : (t >= NQ ? NQ - 1 : t);
  atomicOr(&bits[b * nwords + (t >> 5)], 1u << (t & 31));
}

__global__ __launch_bounds__(kSubThreads) void subsample_list_kernel(
    Geom g, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    uint16_t* __restrict__ Kc, uint16_t* __restrict__ Vc, const int32_t* __restrict__ list,
    const uint32_t* __restrict__ bits, int64_t nwords, float* __restrict__ partial,
    int32_t* __restrict__ cnt, MeanPlan plan, int n_mean, int n_gather, int nhg) {
  __shared__ __align__(16) SubLds lds;
  const int per_b = n_mean + n_gather;
  const int b = blockIdx.x / per_b;
  const int r = blockIdx.x % per_b;
  if (r < n_mean) {
    mean_partial_bits(g, K, V, bits, nwords, partial, cnt, plan, r / plan.ncolblk,
                      r % plan.ncolblk, b, lds.mean);
  } else {
    const int rr = r - n_mean;
    gather_tile(g, K, V, Kc, Vc, nullptr, list, rr / nhg, rr % nhg, b, lds.gather);
  }
}

// The list variant's mean role walks token ids, not dropped-row numbers.
static MeanPlan mean_plan_list(const Geom& g) {
  Geom t = g;
  t.n_dropped = g.NQ;
  return mean_plan(t);
}

int64_t list_words(const Geom& g) { return (g.NQ + 31) / 32; }

size_t list_workspace_bytes(const Geom& g) {
  const MeanPlan p = mean_plan_list(g);
  const size_t partial = (size_t)g.B * p.nchunks * 2 * g.H * kHeadDim * sizeof(float);
  return partial + (size_t)g.B * p.nchunks * sizeof(int32_t);
}

hipError_t launch_subsample_list(const Geom& g, const int32_t* list, const void* K, const void* V,
                                 void* Kc, void* Vc, float* kmean, float* vmean, uint32_t* bits,
                                 int32_t* nd_out, void* workspace, hipStream_t st) {
  const MeanPlan plan = mean_plan_list(g);
  const int64_t nwords = list_words(g);
  const int nhg = (g.H + kHeadGroup - 1) / kHeadGroup;
  const int64_t n_gather = (g.M_pad / kTileRows) * nhg;
  const int64_t n_mean = (int64_t)plan.nchunks * plan.ncolblk;
  const int64_t groups = (n_gather + n_mean) * g.B;
  const int64_t set_groups = (g.M * g.B + 255) / 256;
  if (groups > 0x7FFFFFFF || n_gather > 0x3FFFFFFF || set_groups > 0x7FFFFFFF)
    return hipErrorInvalidConfiguration;
  float* partial = (float*)workspace;
  int32_t* cnt = (int32_t*)(partial + (size_t)g.B * plan.nchunks * 2 * g.H * kHeadDim);
  (void)hipGetLastError();
  const int64_t total_words = nwords * g.B;
  const unsigned clear_groups = (unsigned)((total_words + 255) / 256 < 2048 ? (total_words + 255) / 256 : 2048);
  hipLaunchKernelGGL(bits_clear_kernel, dim3(clear_groups), dim3(256), 0, st, bits, total_words);
  hipLaunchKernelGGL(bits_set_kernel, dim3((unsigned)set_groups), dim3(256), 0, st, list, g.M, g.NQ,
                     nwords, g.B, bits);
  hipLaunchKernelGGL(subsample_list_kernel, dim3((unsigned)groups), dim3(kSubThreads), 0, st, g,
                     (const uint16_t*)K, (const uint16_t*)V, (uint16_t*)Kc, (uint16_t*)Vc, list,
                     (const uint32_t*)bits, nwords, partial, cnt, plan, (int)n_mean, (int)n_gather,
                     nhg);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int C = g.H * kHeadDim;
  dim3 grid2((unsigned)((2 * C + kFinalCols - 1) / kFinalCols), (unsigned)g.B);
  hipLaunchKernelGGL(mean_final_kernel, grid2, dim3(kFinalCols * kFinalGroups), 0, st, g,
                     (const float*)partial, plan.nchunks, kmean, vmean, (const int32_t*)cnt,
                     nd_out);
  return hipGetLastError();
}

// One wavefront per (batch, kept position): which token of the position's window serves as
// key/value.  Special tokens and a whole-kept frame 0 map to themselves.
__device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(256) void select_kernel(Geom g, int rule, uint32_t seed32,
                                                     const uint16_t* __restrict__ K,
                                                     int32_t* __restrict__ list) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= g.M * g.B) return;  // uniform per wavefront
  const int b = (int)(row / g.M);
  const int64_t m = row % g.M;
  // position m -> (frame, j) exactly as the grid rule numbers its kept rows
  int64_t frame;
  int32_t j;
  if (g.keep_first && m < g.L) {
    if (lane == 0) list[row] = (int32_t)m;
    return;
  }
  {
    const uint32_t r = (uint32_t)(g.keep_first ? m - g.L : m);
    frame = (g.keep_first ? 1 : 0) + (int64_t)(r / (uint32_t)g.rows_sub);
    j = (int32_t)(r % (uint32_t)g.rows_sub);
  }
  if (j < g.P) {
    if (lane == 0) list[row] = (int32_t)(frame * g.L + j);
    return;
  }
  const int32_t win = j - g.P;  // row-major window number inside the frame
  const int32_t row0 = (win / g.kw) * g.s_h;
  const int32_t col0 = (win % g.kw) * g.s_w;
  const int32_t wrows = min(g.s_h, g.n_h - row0);
  const int32_t wcols = min(g.s_w, g.n_w - col0);
  const int32_t cells = wrows * wcols;
  int32_t pick = 0;
  if (rule == AGG_SELECT_RANDOM) {
    uint32_t x = mix32(seed32 ^ ((uint32_t)(b * g.N + (int32_t)frame) * 0x85EBCA77u));
    x = mix32(x ^ ((uint32_t)win * 0xC2B2AE3Du));
    pick = (int32_t)(x % (uint32_t)cells);
  } else if (rule == AGG_SELECT_HIGH || rule == AGG_SELECT_LOW) {
    const int C = g.H * kHeadDim;
    float best = 0.f;
    for (int32_t c = 0; c < cells; ++c) {
      const int64_t tok = frame * g.L + g.P + (int64_t)(row0 + c / wcols) * g.n_w + col0 + c % wcols;
      const uint16_t* kr = K + ((int64_t)b * g.NQ + tok) * C;
      float ss = 0.f;
      for (int ch = lane * 8; ch < C; ch += 512) {
        u32x4 v = *reinterpret_cast<const u32x4*>(kr + ch);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xFFFF0000u);
          ss += lo * lo;
          ss += hi * hi;
        }
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
      const bool better = (rule == AGG_SELECT_HIGH) ? (ss > best) : (ss < best);
      if (c == 0 || better) {
        best = ss;
        pick = c;
      }
    }
  }
  if (lane == 0)
    list[row] = (int32_t)(frame * g.L + g.P + (int64_t)(row0 + pick / wcols) * g.n_w + col0 +
                          pick % wcols);
}

hipError_t launch_select(const Geom& g, int rule, uint64_t seed, const void* K, int32_t* list,
                         hipStream_t st) {
  const int64_t groups = (g.M * g.B + 3) / 4;
  if (groups > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
  const uint32_t seed32 = (uint32_t)seed ^ ((uint32_t)(seed >> 32) * 0x9E3779B1u);
  (void)hipGetLastError();
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)groups), dim3(256), 0, st, g, rule, seed32,
                     (const uint16_t*)K, list);
  return hipGetLastError();
}

}  // namespace agg

// Grid gather and mean-fill reduction (Sec. 4.3 of the AVGGT paper: only the
// kept subset serves as keys/values; all dropped patches are summarised by one
// mean key/value pair).  HBM-bandwidth bound: one launch reads every K and V
// row exactly once (kept rows are copied, dropped rows are summed) and writes
// the kept rows once, in the fragment order agg.h documents.  Workgroups of
// that launch take one of two roles -- repack a 64-row tile of the compacted
// set, or sum a run of dropped rows -- so that both kinds of traffic share the
// memory system at the same time; a second, small launch adds the partial sums.
#include "agg_internal.h"

namespace agg {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSubThreads = 256;
constexpr int kHeadGroup = 4;  // heads repacked per workgroup: 64 rows x 4 heads x 128 B = 32 KiB
constexpr int kVPad = 72;      // padded row length (elements) of the raw V rows in LDS

// LDS of the gather role
struct GatherLds {
  uint16_t k[kHeadGroup][kTileElems];        // K in fragment order
  uint16_t v[kHeadGroup][kTileRows][kVPad];  // raw V rows
  int64_t tok[kTileRows];
};

// Gather role: one 64-row tile of the compacted set for kHeadGroup heads.  Reads are
// 128-byte row segments (512 B contiguous per token for the four heads); writes are whole
// 8 KiB tiles, fully coalesced.  K chunks are routed through LDS to their fragment-order
// slot; V is transposed through LDS (the PV MFMA wants eight keys of one channel in one
// 16-byte operand).
__device__ inline void gather_tile(const Geom& g, const uint16_t* __restrict__ K,
                                   const uint16_t* __restrict__ V, uint16_t* __restrict__ Kc,
                                   uint16_t* __restrict__ Vc, int32_t* __restrict__ idx,
                                   int64_t tile, int hgrp, int b, GatherLds& s) {
  const int tid = threadIdx.x;
  const int h0 = hgrp * kHeadGroup;
  const int64_t m0 = tile * kTileRows;
  const int nheads = min(kHeadGroup, g.H - h0);

  if (tid < kTileRows) {
    int64_t m = m0 + tid;
    int64_t tok = (m < g.M) ? kept_row_to_token(g, m) : -1;
    s.tok[tid] = tok;
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
      kv = *reinterpret_cast<const u32x4*>(K + off);
      vv = *reinterpret_cast<const u32x4*>(V + off);
    }
    // K: chunk j covers channels 8j..8j+7 -> slot (((row/32)*4 + j/2)*2 + j%2)*32 + row%32
    int kslot = (((row >> 5) * 4 + (j >> 1)) * 2 + (j & 1)) * 32 + (row & 31);
    *reinterpret_cast<u32x4*>(&s.k[hl][kslot * 8]) = kv;
    *reinterpret_cast<u32x4*>(&s.v[hl][row][j * 8]) = vv;
  }
  __syncthreads();

  // stage 2: linear, coalesced tile writes
  const int64_t ntiles = g.M_pad / kTileRows;
  const int out_chunks = nheads * (kTileElems / 8);
  for (int c = tid; c < out_chunks; c += kSubThreads) {
    int hl = c / (kTileElems / 8);
    int slot = c % (kTileElems / 8);
    int64_t base = (((int64_t)b * g.H + (h0 + hl)) * ntiles + tile) * kTileElems + slot * 8;
    *reinterpret_cast<u32x4*>(Kc + base) = *reinterpret_cast<const u32x4*>(&s.k[hl][slot * 8]);
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
      w[e2] = (uint32_t)s.v[hl][ra][d] | ((uint32_t)s.v[hl][rb][d] << 16);
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
  // at least 32 rows per partial, and few enough partials for a cheap second stage
  int64_t rows = (g.n_dropped + kMeanMaxChunks - 1) / kMeanMaxChunks;
  p.rows_per_chunk = (int)(rows < 32 ? 32 : rows);
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

// Mean role.  Threads are laid out as (row lane, 16-byte chunk of the row).  Token ids of the
// run are resolved kMeanBatch at a time into LDS (one integer division chain per row instead
// of one per load), and four rows per lane are requested before any is added, so that enough
// bytes are in flight to cover HBM latency.
__device__ inline void mean_partial(const Geom& g, const uint16_t* __restrict__ K,
                                    const uint16_t* __restrict__ V, float* __restrict__ partial,
                                    const MeanPlan& p, int chunk, int colblk, int b, MeanLds& s) {
  const int tid = threadIdx.x;
  const int C = g.H * kHeadDim;
  const int cg = tid % p.cpr_b;                        // 16-byte chunk inside this channel block
  const int rl = tid / p.cpr_b;                        // row lane
  const int col = (colblk * kSubThreads + cg) * 8;     // first channel of this thread
  const int rpp = p.rpp;
  const bool active = (rl < rpp) && (col < C);
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
    if (active) {
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
  }
  // combine the row lanes in ascending order (fixed order -> reproducible)
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
    for (int r = 0; r < rpp; ++r) {
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
    gather_tile(g, K, V, Kc, Vc, idx, rr / nhg, rr % nhg, b, lds.gather);
  }
}

// Second stage of the mean: a workgroup owns 32 consecutive channels (of K or of V); its 32
// row groups each add every 32nd partial in double, then the 32 sums are added in order.
constexpr int kFinalCols = 32;
constexpr int kFinalGroups = 32;
__global__ __launch_bounds__(kFinalCols * kFinalGroups) void mean_final_kernel(
    Geom g, const float* __restrict__ partial, int nchunks, float* __restrict__ kmean,
    float* __restrict__ vmean) {
  __shared__ double red[kFinalGroups][kFinalCols];
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
  __syncthreads();
  if (rg == 0 && c < 2 * C) {
    double t = 0.0;
    for (int r = 0; r < kFinalGroups; ++r) t += red[r][cl];
    const float m = (g.n_dropped > 0) ? (float)(t / (double)g.n_dropped) : 0.f;
    const int which = c / C, col = c % C;
    (which ? vmean : kmean)[(int64_t)b * C + col] = m;
  }
}

// Enqueues the gather (+ index list) and, when kmean/vmean are given, the mean terms.
hipError_t launch_subsample(const Geom& g, const void* K, const void* V, void* Kc, void* Vc,
                            int32_t* idx, float* kmean, float* vmean, void* workspace,
                            hipStream_t st) {
  const bool want_mean = (kmean != nullptr);
  const MeanPlan plan = mean_plan(g);
  const int nhg = (g.H + kHeadGroup - 1) / kHeadGroup;
  const int64_t n_gather = (g.M_pad / kTileRows) * nhg;
  const int64_t n_mean = want_mean ? (int64_t)plan.nchunks * plan.ncolblk : 0;
  const int64_t groups = (n_gather + n_mean) * g.B;
  if (groups > 0x7FFFFFFF || n_gather > 0x3FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  hipLaunchKernelGGL(subsample_kernel, dim3((unsigned)groups), dim3(kSubThreads), 0, st, g,
                     (const uint16_t*)K, (const uint16_t*)V, (uint16_t*)Kc, (uint16_t*)Vc, idx,
                     (float*)workspace, plan, (int)n_mean, (int)n_gather, nhg);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !want_mean) return e;
  const int C = g.H * kHeadDim;
  dim3 grid2((unsigned)((2 * C + kFinalCols - 1) / kFinalCols), (unsigned)g.B);
  hipLaunchKernelGGL(mean_final_kernel, grid2, dim3(kFinalCols * kFinalGroups), 0, st, g,
                     (const float*)workspace, plan.nchunks, kmean, vmean);
  return hipGetLastError();
}

}  // namespace agg

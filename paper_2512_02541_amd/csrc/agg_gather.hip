// Grid gather and mean-fill reduction (Sec. 4.3 of the AVGGT paper: only the
// kept subset serves as keys/values; all dropped patches are summarised by one
// mean key/value pair).  Both kernels are HBM-bandwidth bound: together they
// read every K and V row exactly once (kept rows are copied, dropped rows are
// summed) and write the kept rows once, in the fragment order agg.h documents.
#include "agg_internal.h"

namespace agg {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kGatherThreads = 256;
constexpr int kHeadGroup = 4;  // heads repacked per workgroup: 64 rows x 4 heads x 128 B = 32 KiB

// One workgroup repacks one 64-row tile of the compacted set for kHeadGroup
// heads.  Reads are 128-byte row segments (512 B contiguous per token for the
// four heads); writes are whole 8 KiB tiles, fully coalesced.  K chunks are
// routed through LDS to their fragment-order slot; V is transposed through LDS
// (the PV MFMA wants eight keys of one channel in one 16-byte operand).
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(Geom g, const uint16_t* __restrict__ K,
                                                                const uint16_t* __restrict__ V,
                                                                uint16_t* __restrict__ Kc,
                                                                uint16_t* __restrict__ Vc,
                                                                int32_t* __restrict__ idx) {
  __shared__ __align__(16) uint16_t sK[kHeadGroup][kTileElems];       // fragment order
  __shared__ __align__(16) uint16_t sV[kHeadGroup][kTileRows][72];    // raw rows, padded
  __shared__ int64_t sTok[kTileRows];

  const int tid = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int h0 = blockIdx.y * kHeadGroup;
  const int b = blockIdx.z;
  const int64_t m0 = tile * kTileRows;
  const int nheads = min(kHeadGroup, g.H - h0);

  if (tid < kTileRows) {
    int64_t m = m0 + tid;
    int64_t tok = (m < g.M) ? kept_row_to_token(g, m) : -1;
    sTok[tid] = tok;
    if (idx && b == 0 && blockIdx.y == 0 && m < g.M) idx[m] = (int32_t)tok;
  }
  __syncthreads();

  // stage 1: 16-byte chunks, (row, head, j) with j the fastest index
  const int chunks = kTileRows * nheads * 8;
  for (int c = tid; c < chunks; c += kGatherThreads) {
    int j = c & 7;
    int hl = (c >> 3) % nheads;
    int row = (c >> 3) / nheads;
    int64_t tok = sTok[row];
    u32x4 kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
    if (tok >= 0) {
      int64_t off = (((int64_t)b * g.NQ + tok) * g.H + (h0 + hl)) * kHeadDim + j * 8;
      kv = *reinterpret_cast<const u32x4*>(K + off);
      vv = *reinterpret_cast<const u32x4*>(V + off);
    }
    // K: chunk j covers channels 8j..8j+7 -> slot (((row/32)*4 + j/2)*2 + j%2)*32 + row%32
    int kslot = (((row >> 5) * 4 + (j >> 1)) * 2 + (j & 1)) * 32 + (row & 31);
    *reinterpret_cast<u32x4*>(&sK[hl][kslot * 8]) = kv;
    *reinterpret_cast<u32x4*>(&sV[hl][row][j * 8]) = vv;
  }
  __syncthreads();

  // stage 2: linear, coalesced tile writes
  const int64_t ntiles = g.M_pad / kTileRows;
  const int out_chunks = nheads * (kTileElems / 8);
  for (int c = tid; c < out_chunks; c += kGatherThreads) {
    int hl = c / (kTileElems / 8);
    int slot = c % (kTileElems / 8);
    int64_t base = (((int64_t)b * g.H + (h0 + hl)) * ntiles + tile) * kTileElems + slot * 8;
    *reinterpret_cast<u32x4*>(Kc + base) = *reinterpret_cast<const u32x4*>(&sK[hl][slot * 8]);
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
      w[e2] = (uint32_t)sV[hl][ra][d] | ((uint32_t)sV[hl][rb][d] << 16);
    }
    u32x4 out = {w[0], w[1], w[2], w[3]};
    *reinterpret_cast<u32x4*>(Vc + base) = out;
  }
}

// ---------------------------------------------------------------------------
// Mean component.  Stage 1: each workgroup sums a run of consecutive dropped
// rows (all H*64 channels of K and of V) in a fixed order and writes one
// partial.  Stage 2: the partials are added in a fixed order, in double, and
// divided by the number of dropped patches.  No atomics: the result is
// bit-reproducible.
// ---------------------------------------------------------------------------
constexpr int kMeanThreads = 256;
constexpr int kMeanBatch = 256;       // token ids resolved per pass through LDS
constexpr int kMeanMaxChunks = 4096;  // upper bound on partials per batch element

// dropped rows per partial: at least 32, and few enough partials for a cheap second stage
static int mean_rows_per_chunk(const Geom& g) {
  int64_t rows = (g.n_dropped + kMeanMaxChunks - 1) / kMeanMaxChunks;
  return (int)(rows < 32 ? 32 : rows);
}

int mean_chunks(const Geom& g) {
  const int rows = mean_rows_per_chunk(g);
  return (int)((g.n_dropped + rows - 1) / rows);
}

__device__ inline void add_bf16x8(float (&acc)[8], const u32x4& v) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc[2 * i] += __uint_as_float(v[i] << 16);
    acc[2 * i + 1] += __uint_as_float(v[i] & 0xFFFF0000u);
  }
}

// Threads are laid out as (row lane, 16-byte chunk of the row): cpr_b chunks per row, rpp
// rows in flight per pass.  Channel block blockIdx.y covers chunks [256*y, 256*y + cpr_b).
// Token ids of the run are resolved kMeanBatch at a time into LDS (one integer division
// chain per row instead of one per load), and four rows per lane are requested before any
// is added, so that enough bytes are in flight to cover HBM latency.
__global__ __launch_bounds__(kMeanThreads) void mean_partial_kernel(
    Geom g, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    float* __restrict__ partial, int nchunks, int rows_per_chunk, int cpr_b, int rpp) {
  __shared__ float red[kMeanThreads][17];
  __shared__ int32_t sTok[kMeanBatch];
  const int tid = threadIdx.x;
  const int chunk = blockIdx.x;
  const int b = blockIdx.z;
  const int C = g.H * kHeadDim;
  const int cg = tid % cpr_b;             // 16-byte chunk inside this channel block
  const int rl = tid / cpr_b;             // row lane
  const int col = (blockIdx.y * kMeanThreads + cg) * 8;  // first channel of this thread
  const bool active = (rl < rpp) && (col < C);
  const uint16_t* Kb = K + (int64_t)b * g.NQ * C + col;
  const uint16_t* Vb = V + (int64_t)b * g.NQ * C + col;

  float ak[8], av[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) ak[i] = av[i] = 0.f;

  const int64_t u0 = (int64_t)chunk * rows_per_chunk;
  const int64_t u1 = min(u0 + rows_per_chunk, g.n_dropped);
  for (int64_t base = u0; base < u1; base += kMeanBatch) {
    const int n = (int)min((int64_t)kMeanBatch, u1 - base);
    __syncthreads();  // previous batch consumed
    if (tid < n) sTok[tid] = (int32_t)dropped_to_token(g, base + tid);
    __syncthreads();
    if (active) {
      int r = rl;
      for (; r + 3 * rpp < n; r += 4 * rpp) {
        u32x4 kv[4], vv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t off = (int64_t)sTok[r + j * rpp] * C;
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
        const int64_t off = (int64_t)sTok[r] * C;
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
    red[tid][i] = ak[i];
    red[tid][8 + i] = av[i];
  }
  __syncthreads();
  if (rl == 0 && col < C) {
    float sk[8], sv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) sk[i] = sv[i] = 0.f;
    for (int r = 0; r < rpp; ++r) {
      int t = r * cpr_b + cg;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        sk[i] += red[t][i];
        sv[i] += red[t][8 + i];
      }
    }
    float* pk = partial + (((int64_t)b * nchunks + chunk) * 2 + 0) * C + col;
    float* pv = partial + (((int64_t)b * nchunks + chunk) * 2 + 1) * C + col;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pk[i] = sk[i];
      pv[i] = sv[i];
    }
  }
}

// Second stage: a workgroup owns 32 consecutive channels (of K or of V); its 32 row groups
// each add every 32nd partial in double, then the 32 sums are added in order.
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

hipError_t launch_gather(const Geom& g, const void* K, const void* V, void* Kc, void* Vc,
                         int32_t* idx, hipStream_t st) {
  dim3 grid((unsigned)(g.M_pad / kTileRows), (unsigned)((g.H + kHeadGroup - 1) / kHeadGroup),
            (unsigned)g.B);
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  hipLaunchKernelGGL(gather_kernel, grid, dim3(kGatherThreads), 0, st, g, (const uint16_t*)K,
                     (const uint16_t*)V, (uint16_t*)Kc, (uint16_t*)Vc, idx);
  return hipGetLastError();
}

hipError_t launch_mean(const Geom& g, const void* K, const void* V, float* kmean, float* vmean,
                       void* workspace, hipStream_t st) {
  const int C = g.H * kHeadDim;
  const int nchunks = mean_chunks(g);
  if (nchunks > 0) {
    const int cpr = C / 8;                                    // 16-byte chunks per row
    const int cpr_b = cpr < kMeanThreads ? cpr : kMeanThreads;
    const int rpp = kMeanThreads / cpr_b;
    dim3 grid((unsigned)nchunks, (unsigned)((cpr + kMeanThreads - 1) / kMeanThreads), (unsigned)g.B);
    (void)hipGetLastError();  // drop any stale error so the check below is this launch's
    hipLaunchKernelGGL(mean_partial_kernel, grid, dim3(kMeanThreads), 0, st, g, (const uint16_t*)K,
                       (const uint16_t*)V, (float*)workspace, nchunks, mean_rows_per_chunk(g), cpr_b,
                       rpp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  dim3 grid2((unsigned)((2 * C + kFinalCols - 1) / kFinalCols), (unsigned)g.B);
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  hipLaunchKernelGGL(mean_final_kernel, grid2, dim3(kFinalCols * kFinalGroups), 0, st, g,
                     (const float*)workspace, nchunks, kmean, vmean);
  return hipGetLastError();
}

}  // namespace agg

// The parts of a global-attention block around the attention itself (AVGGT Sec. 4.2: a
// block is converted or subsampled with all its other components unchanged):
// LayerNorm, the Q/K/V projections, the output projection with bias and residual.
// They are a few percent of a block's time next to attention over 10^5..10^6 tokens and
// follow the MFMA conventions of the attention kernel.
#include "agg_internal.h"

namespace agg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

union Frag {
  u32x4 u;
  bf16x8 h;
};

__device__ inline uint32_t pack2(float lo, float hi) {
  f32x2 p = {lo, hi};
  bf16x2 h = __builtin_convertvector(p, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}
__device__ inline float lo16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float hi16(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

}  // namespace

// ---------------------------------------------------------------------------
// LayerNorm over the channel dimension: one wavefront per token row, fp32 statistics
// (mean, then variance of the centred values), bf16 in and out.  C must be a multiple
// of 8; a lane owns 16-byte chunks lane, lane+64, ...
// ---------------------------------------------------------------------------
constexpr int kLnThreads = 256;
constexpr int kLnMaxChunks = 8;  // per lane: supports C <= 64*8*8 = 4096

// kChunks = 16-byte chunks per lane (4 up to 2048 channels, else 8): the row lives in registers,
// and the narrower instance keeps enough wavefronts resident to run at the memory rate
template <int kChunks>
__global__ __launch_bounds__(kLnThreads) void layernorm_kernel(const uint16_t* __restrict__ x,
                                                               const float* __restrict__ gamma,
                                                               const float* __restrict__ beta,
                                                               uint16_t* __restrict__ y, int64_t rows,
                                                               int C, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (kLnThreads / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nchunk = C / 8;
  const uint16_t* xr = x + row * C;
  float v[kChunks][8];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    const int ch = lane + 64 * c;
    if (ch < nchunk) {
      u32x4 raw = *reinterpret_cast<const u32x4*>(xr + ch * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[c][2 * i] = lo16(raw[i]);
        v[c][2 * i + 1] = hi16(raw[i]);
        sum += v[c][2 * i] + v[c][2 * i + 1];
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
  const float mean = sum / (float)C;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    const int ch = lane + 64 * c;
    if (ch < nchunk) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = v[c][i] - mean;
        sq += d * d;
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
  const float rstd = rsqrtf(sq / (float)C + eps);
  uint16_t* yr = y + row * C;
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    const int ch = lane + 64 * c;
    if (ch < nchunk) {
      float o[8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        o[i] = (v[c][i] - mean) * rstd * gamma[ch * 8 + i] + beta[ch * 8 + i];
      u32x4 w = {pack2(o[0], o[1]), pack2(o[2], o[3]), pack2(o[4], o[5]), pack2(o[6], o[7])};
      *reinterpret_cast<u32x4*>(yr + ch * 8) = w;
    }
  }
}

// ---------------------------------------------------------------------------
// Linear layer  Y[m, n] = sum_k A[m, k] W[n, k] + bias[n] (+ R[m, n]),  bf16 in/out,
// fp32 accumulation on v_mfma_f32_32x32x16_bf16.  A: [rows, K] row-major; W: [N, K]
// row-major (one row per output channel), so both operands are contiguous along k.
// One workgroup (8 wavefronts) computes a 256 x 256 tile with 64-wide k steps,
// double-buffered in LDS (128 KiB) through registers; each wavefront owns 64 tokens x 128
// channels: six fragment reads feed eight MFMAs, and a tile's operands are fetched from L2
// half as often as with 128 x 128 tiles.  LDS rows are 128
// bytes with the 16-byte chunk index XOR-ed by the row pair's number so that both the
// row-wise fills and the fragment reads spread over all banks.  The product is formed
// transposed (W rows as the MFMA A operand): a lane ends up with four consecutive output
// channels of one token, and the epilogue turns the tile through LDS so that rows leave in
// 128-byte runs.
// Requires K % 64 == 0 and N % 8 == 0.
//
// One launch serves up to three weight matrices applied to the same input (the Q, K and V
// projections): their output tiles of one token tile are neighbours in the launch order and
// run on the same XCD, so a token tile is fetched from HBM once and then served by that
// XCD's L2 to all of them.
// ---------------------------------------------------------------------------
constexpr int kGemmThreads = 512;
constexpr int kTM = 256, kTN = 256, kTK = 64;
constexpr int kGemmXcds = 8;
constexpr int kEpiStride = 64 + 4;  // floats per token row of the epilogue's LDS tile (padded)
constexpr int kStage = (kTM * 8) / kGemmThreads;  // 16-byte chunks per thread and operand (4)

// LDS has 64 banks of 4 bytes: a 16-byte access per lane is served 16 lanes at a time, which
// must then fall on 16 different 16-byte slots of the 256-byte bank period.  Two 128-byte rows
// share a period; XOR-ing the chunk with the row PAIR's number spreads 16 consecutive rows of
// one chunk column (a fragment read) as well as the 16 chunks of a row pair (a fill).
__device__ inline int swz(int row, int chunk) {
  return (row >> 1) * 16 + ((((row & 1) << 3) | chunk) ^ ((row >> 1) & 7));
}

template <bool kResidual>
__global__ __launch_bounds__(kGemmThreads, 1) void linear_kernel(
    const uint16_t* __restrict__ A, LinearOuts outs, const uint16_t* __restrict__ R, int64_t rows,
    int N, int K, int gm, int gn) {
  __shared__ __align__(16) u32x4 sA[2][kTM * 8];
  __shared__ __align__(16) u32x4 sW[2][kTN * 8];
  // workgroup id -> (token tile, output tile): consecutive ids go to consecutive XCDs; an XCD
  // walks all output tiles of one token tile before it moves to its next token tile
  const int xcd = blockIdx.x % kGemmXcds;
  const int seq = blockIdx.x / kGemmXcds;
  const int per_m = gn * outs.count;
  const int mt = (seq / per_m) * kGemmXcds + xcd;
  if (mt >= gm) return;  // uniform for the workgroup, before any barrier
  const int nt_all = seq % per_m;
  const int which = nt_all / gn;
  const uint16_t* __restrict__ W = outs.W[which];
  const float* __restrict__ bias = outs.bias[which];
  uint16_t* __restrict__ Y = outs.Y[which];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int g2 = lane >> 5;
  const int wm = (wave & 3) * 64;    // this wavefront's 64 token rows inside the tile
  const int wn = (wave >> 2) * 128;  // and its 128 output channels
  const int64_t m0 = (int64_t)mt * kTM;
  const int n0 = (nt_all % gn) * kTN;

  // staging: 256 rows x 8 chunks per operand = 2048 chunks, 4 per thread
  u32x4 ra[kStage], rw[kStage];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < kStage; ++i) {
      const int c = tid + i * kGemmThreads;
      const int r = c >> 3, j = c & 7;
      int64_t am = m0 + r;
      if (am >= rows) am = rows - 1;  // tail rows repeat the last row, never stored
      int wn_ = n0 + r;
      if (wn_ >= N) wn_ = N - 1;
      ra[i] = *reinterpret_cast<const u32x4*>(A + am * K + k0 + j * 8);
      rw[i] = *reinterpret_cast<const u32x4*>(W + (int64_t)wn_ * K + k0 + j * 8);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < kStage; ++i) {
      const int c = tid + i * kGemmThreads;
      const int r = c >> 3, j = c & 7;
      sA[buf][swz(r, j)] = ra[i];
      sW[buf][swz(r, j)] = rw[i];
    }
  };

  f32x16 acc[4][2];  // [channel block][token block]
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const int nk = K / kTK;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * kTK);
    // fragments of sub-step ks+1 are requested before the MFMAs of sub-step ks are issued, and
    // the scheduler is kept from sinking those reads back down next to their use
    Frag fw[2][4], fa[2][2];
    auto load_frags = [&](int ks, int set) {
#pragma unroll
      for (int a = 0; a < 4; ++a) fw[set][a].u = sW[buf][swz(wn + a * 32 + l32, ks * 2 + g2)];
#pragma unroll
      for (int b = 0; b < 2; ++b) fa[set][b].u = sA[buf][swz(wm + b * 32 + l32, ks * 2 + g2)];
    };
    load_frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < 3) load_frags(ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks & 1][a].h, fa[ks & 1][b].h,
                                                              acc[a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kt + 1 < nk) lstore(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  acc[a][b][r] is channel n0 + wn + 32a + 8(r/4) + 4g2 + r%4 of token
  // m0 + wm + 32b + l32: written straight from there a lane would store 8 bytes per 2 KiB-apart
  // row.  Instead each wavefront turns its tile through a private piece of the (now idle) LDS,
  // 32 tokens x 64 channels of float at a time, and writes whole 128-byte runs of a token row:
  // 16 lanes x 4 channels.  Bias and residual are added in float before the one rounding.
  float* epi = reinterpret_cast<float*>(wave < 4 ? &sA[0][0] : &sW[0][0]) + (wave & 3) * (32 * kEpiStride);
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int ch = (lane & 15) * 4;                  // channel inside this 64-channel run
      const int n = n0 + wn + half * 64 + ch;
      // residual values of the eight rows this lane will finish, requested before the LDS turn
      u32x2 rr[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int64_t m = m0 + wm + b * 32 + i * 4 + (lane >> 4);
        rr[i] = u32x2{0u, 0u};
        if (kResidual && m < rows && n < N) rr[i] = *reinterpret_cast<const u32x2*>(R + m * N + n);
      }
#pragma unroll
      for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int a = half * 2 + a2;
          f32x4 v4 = {acc[a][b][r4 * 4 + 0], acc[a][b][r4 * 4 + 1], acc[a][b][r4 * 4 + 2],
                      acc[a][b][r4 * 4 + 3]};
          *reinterpret_cast<f32x4*>(epi + l32 * kEpiStride + a2 * 32 + r4 * 8 + g2 * 4) = v4;
        }
      f32x4 bv = {0.f, 0.f, 0.f, 0.f};
      if (bias && n < N) {
#pragma unroll
        for (int i = 0; i < 4; ++i) bv[i] = bias[n + i];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = i * 4 + (lane >> 4);             // token inside this 32-token block
        const int64_t m = m0 + wm + b * 32 + t;
        f32x4 o = *reinterpret_cast<const f32x4*>(epi + t * kEpiStride + ch);
        if (m < rows && n < N) {
          o += bv;
          if (kResidual) {
            o[0] += lo16(rr[i][0]);
            o[1] += hi16(rr[i][0]);
            o[2] += lo16(rr[i][1]);
            o[3] += hi16(rr[i][1]);
          }
          u32x2 w = {pack2(o[0], o[1]), pack2(o[2], o[3])};
          *reinterpret_cast<u32x2*>(Y + m * N + n) = w;
        }
      }
    }
}

hipError_t launch_layernorm(const void* x, const float* gamma, const float* beta, void* y,
                            int64_t rows, int C, float eps, hipStream_t st) {
  if (C % 8 != 0 || C > 64 * 8 * kLnMaxChunks) return hipErrorInvalidValue;
  const int64_t groups = (rows + (kLnThreads / 64) - 1) / (kLnThreads / 64);
  if (groups > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();
  if (C <= 64 * 8 * 4)
    hipLaunchKernelGGL(layernorm_kernel<4>, dim3((unsigned)groups), dim3(kLnThreads), 0, st,
                       (const uint16_t*)x, gamma, beta, (uint16_t*)y, rows, C, eps);
  else
    hipLaunchKernelGGL(layernorm_kernel<kLnMaxChunks>, dim3((unsigned)groups), dim3(kLnThreads), 0,
                       st, (const uint16_t*)x, gamma, beta, (uint16_t*)y, rows, C, eps);
  return hipGetLastError();
}

hipError_t launch_linear(const void* A, const LinearOuts& outs, const void* R, int64_t rows, int N,
                         int K, hipStream_t st) {
  if (K % kTK != 0 || N % 8 != 0 || outs.count < 1 || outs.count > 3) return hipErrorInvalidValue;
  const int64_t gm = (rows + kTM - 1) / kTM;
  const int gn = (N + kTN - 1) / kTN;
  const int64_t groups = (gm + kGemmXcds - 1) / kGemmXcds * kGemmXcds * gn * outs.count;
  if (groups > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();
  if (R)
    hipLaunchKernelGGL(linear_kernel<true>, dim3((unsigned)groups), dim3(kGemmThreads), 0, st,
                       (const uint16_t*)A, outs, (const uint16_t*)R, rows, N, K, (int)gm, gn);
  else
    hipLaunchKernelGGL(linear_kernel<false>, dim3((unsigned)groups), dim3(kGemmThreads), 0, st,
                       (const uint16_t*)A, outs, (const uint16_t*)R, rows, N, K, (int)gm, gn);
  return hipGetLastError();
}

}  // namespace agg

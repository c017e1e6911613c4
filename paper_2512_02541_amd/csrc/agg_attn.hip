// Flash-style forward kernel for subsampled global attention (AVGGT Sec. 4.3):
// every query attends to the compacted key/value set, plus -- inside the same
// softmax -- its own key/value when its token was dropped and the mean pair of
// all dropped patches.  With an un-subsampled compacted set and no extras the
// same kernel is ordinary global attention (Sec. 4.2).
//
// Mapping to gfx950
//   * One workgroup = 4 wavefronts = 256 queries of one (batch, head); each
//     wavefront owns 64 queries (two 32-wide MFMA column blocks) for the whole
//     key loop and keeps Q and the output accumulator in registers.
//   * The score tile is computed transposed, S^T = K * Q^T, with
//     v_mfma_f32_32x32x16_bf16: a lane then holds 16 keys of ONE query, so row
//     sums are in-register plus one exchange with lane^32, and the
//     exponentiated tile is already in the B-operand layout of the second
//     product O^T += V^T * P^T.  P never touches LDS.
//   * K/V arrive in "fragment order" (agg.h): a 64-key tile is a linear 8 KiB
//     copy into LDS and every MFMA A operand is one conflict-free 16-byte read.
//     Three tiles are resident: the one in use, the next one (its first
//     fragments are fetched a block ahead) and the one being filled.  Tiles go
//     global -> LDS without passing through registers (global_load_lds_dwordx4),
//     one tile ahead; a wavefront waits for its own copies before the barrier
//     that ends an iteration.
//   * At head dimension 64 the vector ALU is as loaded as the matrix core (one
//     exponential per 256 MFMA flops) and a wavefront issues in order, so the
//     key loop is software-pipelined: while the matrix core runs K Q^T of block
//     j+1 (then P V of block j), the same wavefront's vector ALU exponentiates
//     half of block j (then half of block j+1).
//   * Fast path: Q is pre-multiplied by scale*log2(e) and the probabilities are
//     exp2 of the raw base-2 logits, with NO reference subtracted: softmax is
//     invariant to the reference, float/bf16 exponents cover 2^+-126, and the
//     per-score work shrinks to exp + convert + add.  A row whose sum leaves
//     [2^-90, 2^90] (logits beyond about +-60 nats) makes the whole workgroup
//     redo its rows in the general path below; ordinary attention logits never
//     get there.
//   * General path: classic online softmax with a running row maximum.
//   * The extras enter as the initial state (sum, accumulator) of either path, so
//     the three parts share one normalisation by construction.
//   * Workgroups are numbered so that the 8 XCDs each stream a different
//     (batch, head): all workgroups resident on one XCD read the same K/V
//     stream and share it through that XCD's L2.
#include "agg_internal.h"

namespace agg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kAttnThreads = 256;
constexpr int kQTile = 256;  // queries per workgroup
constexpr int kXcds = 8;
constexpr int kLdsTiles = 3;
constexpr int kEpiStride = kHeadDim + 8;  // bf16 per query row of the epilogue's LDS tile (padded)
constexpr int kChunks = kTileElems / 8;  // 16-byte chunks per K or V tile (512)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSumHi = 1.2379400392853803e27f;   // 2^90
constexpr float kSumLo = 8.077935669463161e-28f;   // 2^-90

union Frag {
  u32x4 u;
  bf16x8 h;
};

__device__ inline uint32_t pack_bf16(float lo, float hi) {
  f32x2 p = {lo, hi};
  bf16x2 h = __builtin_convertvector(p, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, h);
}
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup barrier that orders LDS traffic only: global loads issued for a later tile
// stay in flight across it.
__device__ inline void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Asynchronous copy of one 8 KiB tile (512 chunks of 16 bytes) global -> LDS without passing
// through registers: each wavefront lands 64 consecutive chunks per instruction.
__device__ inline void dma16(const u32x4* gsrc, uint32_t lds_wave_base) {
  // M0 carries the wavefront's LDS base; lane i lands its 16 bytes at base + 16 i.  Written as
  // assembly so that the compiler's wait-count pass does not serialise later LDS reads of
  // OTHER buffers behind this copy; the loop waits for it explicitly before the barrier.
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gsrc), "s"(lds_wave_base)
               : "memory");  // M0 is a reserved register the compiler sets right before each of
                             // its own uses (none in this kernel), so it is not listed
}
__device__ inline void tile_to_lds(const u32x4* __restrict__ src, u32x4* dst, int tid, int wave) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)(dst + wave * 64)));
  dma16(src + tid, base);
  dma16(src + kAttnThreads + tid, base + kAttnThreads * 16);
}
__device__ inline void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only

#define AGG_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a).h, (b).h, (c), 0, 0, 0)

// K fragments (A operand of S^T = K Q^T) of 32-key block kb of an LDS tile
__device__ inline void load_k_frags(const u32x4* __restrict__ tk, int kb, int l32, int g2,
                                    Frag (&a)[4]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) a[ks].u = tk[((kb * 4 + ks) * 2 + g2) * 32 + l32];
}
// V fragments (A operand of O^T += V^T P^T) of 32-key block kb; index = hf*2 + db
__device__ inline void load_v_frags(const u32x4* __restrict__ tv, int kb, int l32, int g2,
                                    Frag (&v)[4]) {
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int db = 0; db < 2; ++db)
      v[hf * 2 + db].u = tv[((kb * 2 + hf) * 2 + g2) * 64 + db * 32 + l32];
}

// scores of one 32-key block for both query blocks; the two accumulation chains alternate
__device__ inline void qk8(const Frag (&a)[4], const Frag (&Qf)[2][4], f32x16& S0, f32x16& S1) {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  S0 = AGG_MFMA(a[0], Qf[0][0], z);
  S1 = AGG_MFMA(a[0], Qf[1][0], z);
#pragma unroll
  for (int ks = 1; ks < 4; ++ks) {
    S0 = AGG_MFMA(a[ks], Qf[0][ks], S0);
    S1 = AGG_MFMA(a[ks], Qf[1][ks], S1);
  }
}

// O^T += V^T P^T for one 32-key block; query block 0 first (its P is the older one)
__device__ inline void pv8(const Frag (&v)[4], const Frag (&P0)[2], const Frag (&P1)[2],
                           f32x16 (&O)[2][2]) {
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int db = 0; db < 2; ++db) O[0][db] = AGG_MFMA(v[hf * 2 + db], P0[hf], O[0][db]);
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int db = 0; db < 2; ++db) O[1][db] = AGG_MFMA(v[hf * 2 + db], P1[hf], O[1][db]);
}

// fast path: probabilities of 16 raw base-2 logits, packed for the PV MFMA, and their sum
__device__ inline void exp16(const f32x16& S, Frag (&P)[2], float& l0, float& l1) {
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float e0 = fast_exp2(S[hf * 8 + 2 * i]);
      const float e1 = fast_exp2(S[hf * 8 + 2 * i + 1]);
      P[hf].u[i] = pack_bf16(e0, e1);
      l0 += e0;
      l1 += e1;
    }
}

// zero-padded rows of the last tile: key index inside the tile >= valid -> -inf
__device__ inline void mask16(f32x16& S, int kb, int valid, int g2) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int km = 32 * kb + 8 * (r >> 2) + 4 * g2 + (r & 3);
    if (km >= valid) S[r] = -INFINITY;
  }
}

__global__ __launch_bounds__(kAttnThreads, 2) void sga_attn_kernel(
    Geom g, uint32_t flags, float qscale, float mean_bias2, const uint16_t* __restrict__ Q,
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const uint16_t* __restrict__ Kc, const uint16_t* __restrict__ Vc,
    const float* __restrict__ kmean, const float* __restrict__ vmean, uint16_t* __restrict__ O,
    float* __restrict__ lse, int nqt, int npairs, const uint32_t* __restrict__ kept_bits,
    const int32_t* __restrict__ nd_dev) {
  __shared__ __align__(16) uint16_t sK[kLdsTiles][kTileElems];
  __shared__ __align__(16) uint16_t sV[kLdsTiles][kTileElems];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int g2 = lane >> 5;

  // workgroup -> ((batch, head) pair, query tile); consecutive ids go to consecutive XCDs
  const int bid = blockIdx.x;
  const int xcd = bid % kXcds;
  const int seq = bid / kXcds;
  const int pair = (seq / nqt) * kXcds + xcd;
  const int qt = seq % nqt;
  if (pair >= npairs) return;  // uniform for the whole workgroup, before any barrier
  const int b = pair / g.H;
  const int h = pair % g.H;

  const int ntiles = (int)(g.M_pad / kTileRows);
  const int last_valid = (int)(g.M - (int64_t)(ntiles - 1) * kTileRows);  // 1..64
  const int64_t bh_off = ((int64_t)b * g.H + h) * g.M_pad * kHeadDim;
  const u32x4* kc4 = reinterpret_cast<const u32x4*>(Kc + bh_off);
  const u32x4* vc4 = reinterpret_cast<const u32x4*>(Vc + bh_off);
  auto lds_k = [&](int buf) { return reinterpret_cast<u32x4*>(sK[buf]); };
  auto lds_v = [&](int buf) { return reinterpret_cast<u32x4*>(sV[buf]); };

  // ---- Q fragments (B operand of S^T = K Q^T), pre-multiplied by scale*log2(e) ----
  Frag Qf[2][4];
  bool dropped[2];
  float l_self[2], l_mean[2];  // base-2 logits of the extras (-inf when absent)
  // caller's list: membership comes from a bitmap, the dropped count from device memory
  const int64_t n_drop = nd_dev ? (int64_t)nd_dev[b] : g.n_dropped;
  const bool use_mean = (flags & AGG_MEAN) && n_drop > 0;
  const bool use_diag = (flags & AGG_DIAG) && (kept_bits != nullptr || n_drop > 0);
  const uint32_t* kb = kept_bits ? kept_bits + (int64_t)b * ((g.NQ + 31) / 32) : nullptr;
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int64_t q = (int64_t)qt * kQTile + wave * 64 + qb * 32 + l32;
    const int64_t qc = q < g.NQ ? q : g.NQ - 1;  // tail rows recompute the last query, never stored
    const int64_t qbase = (((int64_t)b * g.NQ + qc) * g.H + h) * kHeadDim;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 raw = *reinterpret_cast<const u32x4*>(Q + qbase + ks * 16 + g2 * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        Qf[qb][ks].u[i] = pack_bf16(bf16_lo(raw[i]) * qscale, bf16_hi(raw[i]) * qscale);
    }
    // logits of the extras: lanes l and l^32 hold the two halves of the channel range
    dropped[qb] = use_diag && q < g.NQ &&
                  (kb ? ((kb[q >> 5] >> (q & 31)) & 1u) == 0u : (bool)token_is_dropped(g, q));
    float dot_self = 0.f, dot_mean = 0.f;
    if (use_mean || use_diag) {
      const float* km = kmean + ((int64_t)b * g.H + h) * kHeadDim;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int d0 = ks * 16 + g2 * 8;
        float qv[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          qv[2 * i] = bf16_lo(Qf[qb][ks].u[i]);
          qv[2 * i + 1] = bf16_hi(Qf[qb][ks].u[i]);
        }
        if (use_mean) {
          f32x4 c0 = *reinterpret_cast<const f32x4*>(km + d0);
          f32x4 c1 = *reinterpret_cast<const f32x4*>(km + d0 + 4);
#pragma unroll
          for (int i = 0; i < 4; ++i) dot_mean += qv[i] * c0[i] + qv[4 + i] * c1[i];
        }
        if (dropped[qb]) {
          u32x4 kr = *reinterpret_cast<const u32x4*>(K + qbase + d0);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            dot_self += qv[2 * i] * bf16_lo(kr[i]) + qv[2 * i + 1] * bf16_hi(kr[i]);
        }
      }
    }
    dot_self += __shfl_xor(dot_self, 32);
    dot_mean += __shfl_xor(dot_mean, 32);
    l_self[qb] = dropped[qb] ? dot_self : -INFINITY;
    l_mean[qb] = use_mean ? dot_mean + mean_bias2 : -INFINITY;
  }

  // Initial accumulator = extras weighted by exp2(logit - m0):  O0[d] = w_self v_i[d] + w_mean vmean[d]
  auto init_extras = [&](int qb, float m0, f32x16 (&Oq)[2], float& lsum) {
    const float w_self = dropped[qb] ? fast_exp2(l_self[qb] - m0) : 0.f;
    const float w_mean = use_mean ? fast_exp2(l_mean[qb] - m0) : 0.f;
    lsum = (g2 == 0) ? (w_self + w_mean) : 0.f;  // lanes l and l^32 split a row's sum
    const int64_t q = (int64_t)qt * kQTile + wave * 64 + qb * 32 + l32;
    const int64_t qc = q < g.NQ ? q : g.NQ - 1;
    const int64_t qbase = (((int64_t)b * g.NQ + qc) * g.H + h) * kHeadDim;
    const float* vm = vmean + ((int64_t)b * g.H + h) * kHeadDim;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d0 = 32 * db + 8 * r4 + 4 * g2;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (use_mean) {
          f32x4 mv = *reinterpret_cast<const f32x4*>(vm + d0);
          acc = mv * w_mean;
        }
        if (dropped[qb]) {
          u32x2 vr = *reinterpret_cast<const u32x2*>(V + qbase + d0);
          acc[0] += w_self * bf16_lo(vr[0]);
          acc[1] += w_self * bf16_hi(vr[0]);
          acc[2] += w_self * bf16_lo(vr[1]);
          acc[3] += w_self * bf16_hi(vr[1]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) Oq[db][r4 * 4 + i] = acc[i];
      }
  };

  f32x16 Oacc[2][2];  // [query block][channel block] O^T; channel = 32db + 8(r/4) + 4g2 + r%4
  float m_fin[2] = {0.f, 0.f};  // reference of the final state (0 on the fast path)
  float l_fin[2];

  // =============================== fast path ===============================
  {
    float la[2][2];  // two partial row sums per query block
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float l0;
      init_extras(qb, 0.f, Oacc[qb], l0);
      la[qb][0] = l0;
      la[qb][1] = 0.f;
    }

    // tiles 0 and 1 -> LDS
    tile_to_lds(kc4, lds_k(0), tid, wave);
    tile_to_lds(vc4, lds_v(0), tid, wave);
    if (ntiles > 1) {
      tile_to_lds(kc4 + kChunks, lds_k(1), tid, wave);
      tile_to_lds(vc4 + kChunks, lds_v(1), tid, wave);
    }
    wait_vm0();
    lds_barrier();

    // pipeline prologue: scores of block 0 and probabilities of its first query block
    Frag a[4], v[4];
    Frag P0[2], P1[2];
    f32x16 S1;
    {
      f32x16 S0;
      load_k_frags(lds_k(0), 0, l32, g2, a);
      qk8(a, Qf, S0, S1);
      load_k_frags(lds_k(0), 1, l32, g2, a);
      exp16(S0, P0, la[0][0], la[0][1]);
    }

    // invariant at the top of iteration t: a = K fragments of block (t,1); S1 = scores of
    // block (t,0) for query block 1; P0 = probabilities of block (t,0) for query block 0
    int cur = 0;  // LDS buffer of tile t
    for (int t = 0; t + 1 < ntiles; ++t) {
      const int nxt = (cur == kLdsTiles - 1) ? 0 : cur + 1;
      const int wrt = (nxt == kLdsTiles - 1) ? 0 : nxt + 1;
      if (t + 2 < ntiles) {  // tile t+2 -> the buffer tile t-1 has left (barrier of t-1)
        tile_to_lds(kc4 + (int64_t)(t + 2) * kChunks, lds_k(wrt), tid, wave);
        tile_to_lds(vc4 + (int64_t)(t + 2) * kChunks, lds_v(wrt), tid, wave);
      }
      f32x16 Sn0, Sn1, Sm0;
      Frag P0b[2];
      // X(t,0): scores of block (t,1)        | probabilities of block (t,0), query block 1
      load_v_frags(lds_v(cur), 0, l32, g2, v);
      qk8(a, Qf, Sn0, Sn1);
      exp16(S1, P1, la[1][0], la[1][1]);
      // Y(t,0): P V of block (t,0)           | probabilities of block (t,1), query block 0
      load_k_frags(lds_k(nxt), 0, l32, g2, a);
      pv8(v, P0, P1, Oacc);
      exp16(Sn0, P0b, la[0][0], la[0][1]);
      // X(t,1): scores of block (t+1,0)      | probabilities of block (t,1), query block 1
      load_v_frags(lds_v(cur), 1, l32, g2, v);
      qk8(a, Qf, Sm0, S1);
      exp16(Sn1, P1, la[1][0], la[1][1]);
      // Y(t,1): P V of block (t,1)           | probabilities of block (t+1,0), query block 0
      load_k_frags(lds_k(nxt), 1, l32, g2, a);
      pv8(v, P0b, P1, Oacc);
      exp16(Sm0, P0, la[0][0], la[0][1]);
      wait_vm0();  // this wavefront's part of tile t+2 has landed
      lds_barrier();
      cur = nxt;
    }
    {  // last tile: no further scores to start; the only tile with zero-padded rows
      const int T = ntiles - 1;
      (void)T;
      f32x16 Sn0, Sn1;
      Frag P0b[2];
      load_v_frags(lds_v(cur), 0, l32, g2, v);
      qk8(a, Qf, Sn0, Sn1);
      exp16(S1, P1, la[1][0], la[1][1]);
      pv8(v, P0, P1, Oacc);
      exp16(Sn0, P0b, la[0][0], la[0][1]);
      load_v_frags(lds_v(cur), 1, l32, g2, v);
      exp16(Sn1, P1, la[1][0], la[1][1]);
      pv8(v, P0b, P1, Oacc);
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float lp = la[qb][0] + la[qb][1];
      // zero-padded keys have score exactly 0, probability exactly 1 and a zero value row:
      // they only add their count to the row sum
      l_fin[qb] = lp + __shfl_xor(lp, 32) - (float)(kTileRows - last_valid);
    }
  }

  // A row sum outside [2^-90, 2^90] (or NaN) means the unreferenced exponentials were not
  // safe for this row: every wavefront of the workgroup then recomputes with running maxima.
  // (with padded keys the lower bound is 1, so that removing their count loses no precision)
  const float sum_lo = (last_valid < kTileRows) ? 1.0f : kSumLo;
  const bool unsafe = !(l_fin[0] < kSumHi) || !(l_fin[0] > sum_lo) || !(l_fin[1] < kSumHi) ||
                      !(l_fin[1] > sum_lo);
  if (__syncthreads_or(unsafe ? 1 : 0)) {
    // ============================= general path =============================
    float m_run[2], l_part[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float m0 = fmaxf(l_self[qb], l_mean[qb]);
      m_run[qb] = m0;
      if (m0 > -INFINITY) {
        init_extras(qb, m0, Oacc[qb], l_part[qb]);
      } else {
        l_part[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) Oacc[qb][db][r] = 0.f;
      }
    }
    for (int t = 0; t < ntiles; ++t) {
      __syncthreads();  // previous tile fully consumed
      const int64_t off = (int64_t)t * kChunks + tid;
      lds_k(0)[tid] = kc4[off];
      lds_k(0)[tid + kAttnThreads] = kc4[off + kAttnThreads];
      lds_v(0)[tid] = vc4[off];
      lds_v(0)[tid + kAttnThreads] = vc4[off + kAttnThreads];
      __syncthreads();
      const int valid = (t == ntiles - 1) ? last_valid : kTileRows;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        Frag a[4], v[4];
        load_k_frags(lds_k(0), kb, l32, g2, a);
        load_v_frags(lds_v(0), kb, l32, g2, v);
        f32x16 S[2];
        qk8(a, Qf, S[0], S[1]);
        Frag P[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          if (valid < kTileRows) mask16(S[qb], kb, valid, g2);
          float mx = S[qb][0];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[qb][r]);
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          // finite from the first block on: compacted row 0 always exists (block 0 of tile 0)
          const float m_new = fmaxf(m_run[qb], mx);
          const float alpha = fast_exp2(m_run[qb] - m_new);  // -inf -> 0
          m_run[qb] = m_new;
          float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) S[qb][r] -= m_new;
          exp16(S[qb], P[qb], rs0, rs1);
          l_part[qb] = l_part[qb] * alpha + (rs0 + rs1);
#pragma unroll
          for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) Oacc[qb][db][r] *= alpha;
        }
        pv8(v, P[0], P[1], Oacc);
      }
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      m_fin[qb] = m_run[qb];
      l_fin[qb] = l_part[qb] + __shfl_xor(l_part[qb], 32);
    }
  }

  // ---- normalise and store ----
  // A lane holds four consecutive channels of one query per register group: stored from there,
  // every instruction would scatter 8-byte pieces over 64 rows that lie 2*H*64 bytes apart.
  // Each wavefront instead turns its 64 x 64 tile through a private piece of the (now idle) K/V
  // LDS and writes whole 128-byte (query, head) rows, eight per instruction.
  __syncthreads();  // every wavefront is done with the K/V tiles
  uint16_t* epi = (wave < 2 ? &sK[0][0] : &sV[0][0]) + (wave & 1) * (64 * kEpiStride);
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l = l_fin[qb];
    const float inv = 1.0f / l;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int d0 = 32 * db + 8 * r4 + 4 * g2;
        u32x2 w;
        w[0] = pack_bf16(Oacc[qb][db][r4 * 4 + 0] * inv, Oacc[qb][db][r4 * 4 + 1] * inv);
        w[1] = pack_bf16(Oacc[qb][db][r4 * 4 + 2] * inv, Oacc[qb][db][r4 * 4 + 3] * inv);
        *reinterpret_cast<u32x2*>(epi + (qb * 32 + l32) * kEpiStride + d0) = w;
      }
    const int64_t q = (int64_t)qt * kQTile + wave * 64 + qb * 32 + l32;
    if (lse && g2 == 0 && q < g.NQ)
      lse[((int64_t)b * g.H + h) * g.NQ + q] = (m_fin[qb] + log2f(l)) * kLn2;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = i * 8 + (lane >> 3);
    const int64_t q = (int64_t)qt * kQTile + wave * 64 + row;
    const u32x4 v = *reinterpret_cast<const u32x4*>(epi + row * kEpiStride + (lane & 7) * 8);
    if (q < g.NQ)
      *reinterpret_cast<u32x4*>(O + (((int64_t)b * g.NQ + q) * g.H + h) * kHeadDim + (lane & 7) * 8) = v;
  }
}

hipError_t launch_attn(const Geom& g, uint32_t flags, float scale, float mean_bias, const void* Q,
                       const void* K, const void* V, const void* Kc, const void* Vc,
                       const float* kmean, const float* vmean, void* O, float* lse, hipStream_t st,
                       const uint32_t* kept_bits, const int32_t* nd_dev) {
  const int nqt = (int)((g.NQ + kQTile - 1) / kQTile);
  const int npairs = g.B * g.H;
  const int64_t groups = (int64_t)((npairs + kXcds - 1) / kXcds) * kXcds * nqt;
  if (groups > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  hipLaunchKernelGGL(sga_attn_kernel, dim3((unsigned)groups), dim3(kAttnThreads), 0, st, g, flags,
                     scale * kLog2e, mean_bias * kLog2e, (const uint16_t*)Q, (const uint16_t*)K,
                     (const uint16_t*)V, (const uint16_t*)Kc, (const uint16_t*)Vc, kmean, vmean,
                     (uint16_t*)O, lse, nqt, npairs, kept_bits, nd_dev);
  return hipGetLastError();
}

}  // namespace agg

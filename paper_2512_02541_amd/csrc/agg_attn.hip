// Flash-style forward kernel for subsampled global attention (AVGGT Sec. 4.3):
// every query attends to the compacted key/value set, plus -- inside the same
// softmax -- its own key/value when its token was dropped and the mean pair of
// all dropped patches.  With an un-subsampled compacted set and no extras the
// same kernel is ordinary global attention (Sec. 4.2).
//
// Mapping to gfx950
//   * One workgroup = 4 wavefronts = 256 queries of one (batch, head); each
//     wavefront owns 64 queries (two 32-wide MFMA column blocks) for the whole
//     key loop and keeps Q, the softmax state and the output accumulator in
//     registers.
//   * The score tile is computed transposed, S^T = K * Q^T, with
//     v_mfma_f32_32x32x16_bf16: a lane then holds 16 keys of ONE query, so row
//     reductions are in-register plus one exchange with lane^32, and the
//     exponentiated tile is already in the B-operand layout of the second
//     product O^T += V^T * P^T.  P never touches LDS.
//   * K/V arrive in "fragment order" (agg.h): a 64-key tile is a linear 8 KiB
//     copy into LDS and every MFMA A operand is one conflict-free 16-byte read.
//   * At head dimension 64 the vector ALU, not the matrix core, is the tighter
//     pipe (one exponential per 256 MFMA flops), so the inner loop is stripped
//     to exp + convert + sum per score:
//       - Q is pre-multiplied by scale*log2(e), so scores are base-2 logits;
//       - the row reference -m is the INITIAL accumulator of the QK^T MFMA, so
//         the scores come out already shifted;
//       - the reference is not the running maximum but any value that keeps
//         exp2(s - m) inside float range: softmax is invariant to it.  It is
//         raised (with the usual rescale of sum and accumulator) only when a
//         tile's partial row sum exceeds 2^30, which also covers the first
//         tile, where m = -inf.  That slow path recomputes the tile's true
//         maximum; it is wave-uniform and rare;
//       - row sums are taken from the bf16-rounded probabilities with
//         v_dot2c_f32_bf16 (two per instruction), the same values the PV MFMA
//         multiplies.
//   * The extras are folded in as the initial state of the online softmax
//     (reference, sum, accumulator), so the key loop is unmodified and the
//     three parts share one normalisation by construction.
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
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSumLimit = 1073741824.0f;  // 2^30: partial row sum that triggers a new reference

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
// acc + lo(w) + hi(w) for a packed bf16 pair
__device__ inline float add_pair(uint32_t w, float acc) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, acc, false);
}

struct SoftmaxState {
  float m_ref[2];    // per query block: the reference subtracted from the base-2 logits
  float l_part[2];   // this lane's share of the row sum (lanes l and l^32 split a row)
  f32x16 negM[2];    // -m_ref broadcast: initial accumulator of the QK^T MFMA
  f32x16 Oacc[2][2]; // [query block][channel block] O^T; channel = 32db + 8(r/4) + 4g2 + r%4
};

// exp2 of 16 shifted scores -> 8 packed bf16 pairs (two B operands) + their sum
__device__ inline float exp_pack(const f32x16& S, Frag (&Pf)[2]) {
  float rs = 0.f;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t w = pack_bf16(fast_exp2(S[hf * 8 + 2 * i]), fast_exp2(S[hf * 8 + 2 * i + 1]));
      Pf[hf].u[i] = w;
      rs = add_pair(w, rs);
    }
  return rs;
}

// One 64-key tile held in LDS (tk: K fragments, tv: V fragments) against this
// wavefront's 64 queries.  `valid` < 64 only on the zero-padded last tile.
template <bool kMasked>
__device__ inline void process_tile(const u32x4* __restrict__ tk, const u32x4* __restrict__ tv,
                                    int valid, const Frag (&Qf)[2][4], SoftmaxState& st, int l32,
                                    int g2) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    Frag a[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) a[ks].u = tk[((kb * 4 + ks) * 2 + g2) * 32 + l32];
    // one query block at a time keeps a single 16-register score tile live
    Frag Pf[2][2];
    float rs[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 S =
          __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0].h, Qf[qb][0].h, st.negM[qb], 0, 0, 0);
#pragma unroll
      for (int ks = 1; ks < 4; ++ks)
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks].h, Qf[qb][ks].h, S, 0, 0, 0);
      if (kMasked) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int km = 32 * kb + 8 * (r >> 2) + 4 * g2 + (r & 3);
          if (km >= valid) S[r] = -INFINITY;
        }
      }
      rs[qb] = exp_pack(S, Pf[qb]);
    }

    // Fast path ends here unless some row's probabilities left the safe range
    // (or the reference is still -inf): then redo this block against its true maximum.
    const bool bad = !(rs[0] <= kSumLimit) || !(rs[1] <= kSumLimit);
    if (__any(bad)) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        f32x16 T;
#pragma unroll
        for (int r = 0; r < 16; ++r) T[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          T = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks].h, Qf[qb][ks].h, T, 0, 0, 0);
        if (kMasked) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int km = 32 * kb + 8 * (r >> 2) + 4 * g2 + (r & 3);
            if (km >= valid) T[r] = -INFINITY;
          }
        }
        float mx = T[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, T[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(st.m_ref[qb], mx);
        // m_new is finite except when the block is fully masked and nothing came before,
        // which cannot happen: compacted row 0 always exists and is in block 0 of tile 0.
        const float alpha = fast_exp2(st.m_ref[qb] - m_new);  // m_ref = -inf -> 0
        st.m_ref[qb] = m_new;
        st.l_part[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) st.Oacc[qb][db][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          st.negM[qb][r] = -m_new;
          T[r] -= m_new;
        }
        rs[qb] = exp_pack(T, Pf[qb]);
      }
    }
    st.l_part[0] += rs[0];
    st.l_part[1] += rs[1];

#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int tt = kb * 2 + hf;
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        Frag v;
        v.u = tv[(tt * 2 + g2) * 64 + db * 32 + l32];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
          st.Oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v.h, Pf[qb][hf].h,
                                                                     st.Oacc[qb][db], 0, 0, 0);
      }
    }
  }
}

__global__ __launch_bounds__(kAttnThreads, 2) void sga_attn_kernel(
    Geom g, uint32_t flags, float qscale, float mean_bias2, const uint16_t* __restrict__ Q,
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const uint16_t* __restrict__ Kc, const uint16_t* __restrict__ Vc,
    const float* __restrict__ kmean, const float* __restrict__ vmean, uint16_t* __restrict__ O,
    float* __restrict__ lse, int nqt, int npairs) {
  __shared__ __align__(16) uint16_t sK[2][kTileElems];
  __shared__ __align__(16) uint16_t sV[2][kTileElems];

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

  const int64_t ntiles = g.M_pad / kTileRows;
  const int64_t bh_off = ((int64_t)b * g.H + h) * g.M_pad * kHeadDim;
  const u32x4* kc4 = reinterpret_cast<const u32x4*>(Kc + bh_off);
  const u32x4* vc4 = reinterpret_cast<const u32x4*>(Vc + bh_off);

  // ---- Q fragments (B operand of S^T = K Q^T), pre-multiplied by scale*log2(e) ----
  Frag Qf[2][4];
  int64_t qrow[2];
  int64_t qbase[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    int64_t q = (int64_t)qt * kQTile + wave * 64 + qb * 32 + l32;
    qrow[qb] = q;
    int64_t qc = q < g.NQ ? q : g.NQ - 1;  // tail rows recompute the last query, never stored
    qbase[qb] = (((int64_t)b * g.NQ + qc) * g.H + h) * kHeadDim;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 raw = *reinterpret_cast<const u32x4*>(Q + qbase[qb] + ks * 16 + g2 * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        Qf[qb][ks].u[i] = pack_bf16(bf16_lo(raw[i]) * qscale, bf16_hi(raw[i]) * qscale);
    }
  }

  // ---- online-softmax state; the extras (self term, mean term) are its initial value ----
  SoftmaxState st;
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    st.m_ref[qb] = -INFINITY;
    st.l_part[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.Oacc[qb][db][r] = 0.f;
  }

  const bool use_mean = (flags & AGG_MEAN) && g.n_dropped > 0;
  const bool use_diag = (flags & AGG_DIAG) && g.n_dropped > 0;
  if (use_mean || use_diag) {
    const float* km = kmean + ((int64_t)b * g.H + h) * kHeadDim;
    const float* vm = vmean + ((int64_t)b * g.H + h) * kHeadDim;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const bool dropped = use_diag && qrow[qb] < g.NQ && token_is_dropped(g, qrow[qb]);
      float dot_self = 0.f, dot_mean = 0.f;
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
          f32x4 a = *reinterpret_cast<const f32x4*>(km + d0);
          f32x4 c = *reinterpret_cast<const f32x4*>(km + d0 + 4);
#pragma unroll
          for (int i = 0; i < 4; ++i) dot_mean += qv[i] * a[i] + qv[4 + i] * c[i];
        }
        if (dropped) {
          u32x4 kr = *reinterpret_cast<const u32x4*>(K + qbase[qb] + d0);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            dot_self += qv[2 * i] * bf16_lo(kr[i]) + qv[2 * i + 1] * bf16_hi(kr[i]);
        }
      }
      // lanes l and l^32 hold the two halves of the channel range
      dot_self += __shfl_xor(dot_self, 32);
      dot_mean += __shfl_xor(dot_mean, 32);
      const float l_self = dropped ? dot_self : -INFINITY;
      const float l_mean = use_mean ? dot_mean + mean_bias2 : -INFINITY;
      const float m0 = fmaxf(l_self, l_mean);
      if (m0 > -INFINITY) {
        const float w_self = dropped ? fast_exp2(l_self - m0) : 0.f;
        const float w_mean = use_mean ? fast_exp2(l_mean - m0) : 0.f;
        st.m_ref[qb] = m0;
        st.l_part[qb] = (g2 == 0) ? (w_self + w_mean) : 0.f;
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
            if (dropped) {
              u32x2 vr = *reinterpret_cast<const u32x2*>(V + qbase[qb] + d0);
              acc[0] += w_self * bf16_lo(vr[0]);
              acc[1] += w_self * bf16_hi(vr[0]);
              acc[2] += w_self * bf16_lo(vr[1]);
              acc[3] += w_self * bf16_hi(vr[1]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) st.Oacc[qb][db][r4 * 4 + i] = acc[i];
          }
      }
    }
  }
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.negM[qb][r] = -st.m_ref[qb];  // +inf until a reference exists

  // ---- key loop: double-buffered LDS tiles, next tile prefetched into registers ----
  u32x4 pk0, pk1, pv0, pv1;
  pk0 = kc4[tid];
  pk1 = kc4[tid + kAttnThreads];
  pv0 = vc4[tid];
  pv1 = vc4[tid + kAttnThreads];
  {
    u32x4* dk = reinterpret_cast<u32x4*>(sK[0]);
    u32x4* dv = reinterpret_cast<u32x4*>(sV[0]);
    dk[tid] = pk0;
    dk[tid + kAttnThreads] = pk1;
    dv[tid] = pv0;
    dv[tid + kAttnThreads] = pv1;
  }
  __syncthreads();

  const int last_valid = (int)(g.M - (ntiles - 1) * kTileRows);  // 1..64
  for (int64_t t = 0; t + 1 < ntiles; ++t) {
    const int buf = (int)(t & 1);
    {
      const u32x4* nk = kc4 + (t + 1) * (kTileElems / 8);
      const u32x4* nv = vc4 + (t + 1) * (kTileElems / 8);
      pk0 = nk[tid];
      pk1 = nk[tid + kAttnThreads];
      pv0 = nv[tid];
      pv1 = nv[tid + kAttnThreads];
    }
    process_tile<false>(reinterpret_cast<const u32x4*>(sK[buf]),
                        reinterpret_cast<const u32x4*>(sV[buf]), kTileRows, Qf, st, l32, g2);
    {
      u32x4* dk = reinterpret_cast<u32x4*>(sK[buf ^ 1]);
      u32x4* dv = reinterpret_cast<u32x4*>(sV[buf ^ 1]);
      dk[tid] = pk0;
      dk[tid + kAttnThreads] = pk1;
      dv[tid] = pv0;
      dv[tid + kAttnThreads] = pv1;
    }
    __syncthreads();
  }
  {  // last tile, outside the loop: the only one that can hold zero-padded rows
    const int buf = (int)((ntiles - 1) & 1);
    process_tile<true>(reinterpret_cast<const u32x4*>(sK[buf]),
                       reinterpret_cast<const u32x4*>(sV[buf]), last_valid, Qf, st, l32, g2);
  }

  // ---- normalise and store ----
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l = st.l_part[qb] + __shfl_xor(st.l_part[qb], 32);
    const float inv = 1.0f / l;
    if (qrow[qb] < g.NQ) {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int d0 = 32 * db + 8 * r4 + 4 * g2;
          u32x2 w;
          w[0] = pack_bf16(st.Oacc[qb][db][r4 * 4 + 0] * inv, st.Oacc[qb][db][r4 * 4 + 1] * inv);
          w[1] = pack_bf16(st.Oacc[qb][db][r4 * 4 + 2] * inv, st.Oacc[qb][db][r4 * 4 + 3] * inv);
          *reinterpret_cast<u32x2*>(O + qbase[qb] + d0) = w;
        }
      if (lse && g2 == 0)
        lse[((int64_t)b * g.H + h) * g.NQ + qrow[qb]] = (st.m_ref[qb] + log2f(l)) * kLn2;
    }
  }
}

hipError_t launch_attn(const Geom& g, uint32_t flags, float scale, float mean_bias, const void* Q,
                       const void* K, const void* V, const void* Kc, const void* Vc,
                       const float* kmean, const float* vmean, void* O, float* lse, hipStream_t st) {
  const int nqt = (int)((g.NQ + kQTile - 1) / kQTile);
  const int npairs = g.B * g.H;
  const int64_t groups = (int64_t)((npairs + kXcds - 1) / kXcds) * kXcds * nqt;
  if (groups > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  hipLaunchKernelGGL(sga_attn_kernel, dim3((unsigned)groups), dim3(kAttnThreads), 0, st, g, flags,
                     scale * kLog2e, mean_bias * kLog2e, (const uint16_t*)Q, (const uint16_t*)K,
                     (const uint16_t*)V, (const uint16_t*)Kc, (const uint16_t*)Vc, kmean, vmean,
                     (uint16_t*)O, lse, nqt, npairs);
  return hipGetLastError();
}

}  // namespace agg

// Flash-style forward kernel for subsampled global attention (AVGGT Sec. 4.3):
// every query attends to the compacted key/value set, plus -- inside the same
// softmax -- its own key/value when its token was dropped and the mean pair of
// all dropped patches.  With an un-subsampled compacted set and no extras the
// same kernel is ordinary global attention (Sec. 4.2).
//
// Mapping to gfx950
//   * One workgroup = 4 wavefronts; a wavefront owns kQB blocks of 32 queries for the
//     whole key loop and keeps Q and the output accumulator in registers.
//   * Both products run on v_mfma_f32_16x16x32_bf16, which accumulates 32 products per pass
//     through its four accumulator registers: half the accumulator traffic per flop of the
//     32x32x16 shape, and the part is power-limited on this kernel (measured on hashed
//     operands, MFMAs alone: 1.94 against 1.74 PFLOP/s).
//   * The score tile is computed transposed, S^T = K * Q^T: a lane then holds keys of ONE
//     query (four per 16-key tile), so row sums are in-register plus a reduction over the four
//     lanes c, c+16, c+32, c+48, and the exponentiated tiles are already the B operand of the
//     second product O^T += V^T * P^T.  P never touches LDS.  A 32-key block is scored as two
//     16-key tiles whose rows are assigned to the block's keys such that the eight probabilities
//     of a lane belong to exactly one 16-byte chunk of the compacted V tile (row_key below).
//     On the fast path the row sums are a ninth product of the same shape per query tile, a
//     row of ones against P^T (+12.5 % MFMAs): the vector ALU, which has to issue twice as
//     many MFMAs as with the larger shape, then does nothing per score but exponentiate and
//     convert, and every lane ends up with its query's whole sum.
//   * K/V arrive in "fragment order" (agg.h): a 64-key tile is a linear 8 KiB
//     copy into LDS and every MFMA A operand is one conflict-free 16-byte read.
//     Three tiles are resident: the one in use, the next one and the one being
//     filled.  Tiles go global -> LDS without passing through registers
//     (global_load_lds_dwordx4 with a scalar base, so advancing a tile costs two
//     scalar adds); a wavefront waits for its own copies before the barrier that
//     ends an iteration.  The tile loop is unrolled over the three buffers, so every
//     LDS read uses an immediate offset: the loop spends no vector instruction on
//     addresses.
//   * At head dimension 64 the vector ALU is as loaded as the matrix core (one
//     exponential per 256 MFMA flops) and a wavefront issues in order, so the key
//     loop is a software pipeline over "units" (32 keys x 32 queries).  Step u
//     exponentiates unit u on the vector ALU while the matrix core computes the
//     scores of unit u + kQB - 1 and then P V of unit u - 1.  K fragments of a
//     32-key block are fetched from LDS once per kQB units, V fragments likewise.
//   * Fast path: Q is pre-multiplied by scale*log2(e) and the probabilities are
//     exp2 of the raw base-2 logits, with NO reference subtracted: softmax is
//     invariant to the reference, float/bf16 exponents cover 2^+-126, and the
//     per-score work shrinks to exp + convert.  A row whose sum leaves
//     [2^-90, 2^90] (logits beyond about +-60 nats) makes the whole workgroup
//     redo its rows in the general path (a second kernel behind this one, see
//     the end of the file); ordinary attention logits never get there.  The
//     sums are checked every few tiles, so an overflow ends the fast pass early.
//   * General path: the same pipeline with a per-row reference.  The score MFMAs start from
//     an accumulator holding minus the reference instead of zero, so the scores come out
//     relative to it and the vector ALU does no more per score than on the fast path.  The
//     reference starts at the largest of the extras and the first 32 keys and is raised
//     lazily: a unit's row sums show when a score exceeds it by more than 2^100; only then
//     (a rare, wavefront-uniform branch) is the unit's maximum taken, the accumulator
//     rescaled and the unit redone.  No running maximum is computed otherwise.
//   * The zero-padded rows of the last tile are masked there (the last tile is
//     peeled), nowhere else.
//   * The extras enter as the initial state (sum, accumulator) of either path, so
//     the three parts share one normalisation by construction.
//   * Workgroups are numbered so that the 8 XCDs each stream a different
//     (batch, head): all workgroups resident on one XCD read the same K/V
//     stream and share it through that XCD's L2.
#include "agg_internal.h"

namespace agg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#ifndef AGG_QB
#define AGG_QB 2
#endif
#ifndef AGG_WAVES
#define AGG_WAVES 4
#endif

constexpr int kQB = AGG_QB;             // 32-query blocks per wavefront
constexpr int kWaves = AGG_WAVES;       // wavefronts per workgroup
constexpr int kAttnThreads = 64 * kWaves;
constexpr int kWaveQ = 32 * kQB;        // queries per wavefront
constexpr int kQTile = kWaves * kWaveQ; // queries per workgroup
constexpr int kBlocksPerCu = 8 / (kWaves * (kQB == 2 ? 1 : 2));  // two wavefronts per SIMD at kQB = 2
constexpr int kXcds = 8;
constexpr int kLdsTiles = 3;
constexpr int kEpiStride = kHeadDim + 8;  // bf16 per query row of the epilogue's LDS tile (padded)
constexpr int kChunks = kTileElems / 8;  // 16-byte chunks per K or V tile (512)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSumHi = 1.2379400392853803e27f;   // 2^90
constexpr float kSumLo = 8.077935669463161e-28f;   // 2^-90
constexpr float kLazy = 60.0f;  // general path: a unit may exceed the row's reference by 2^60
constexpr float kUnitHi = 1.2676506002282294e30f;  // 2^100: a unit's row sum that forces a look

union Frag {
  u32x4 u;
  bf16x8 h;
};

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 p = {lo, hi};
  bf16x2 h = __builtin_convertvector(p, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange between lanes l and l ^ 32.  v_permlane32_swap exchanges the upper 32 lanes of its
// first operand with the lower 32 of its second; fed the same value twice it returns
// (own, partner) in one order or the other, and both uses below are symmetric.
__device__ __forceinline__ float pair_max(float x) {
  const uint32_t b = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const uint32_t b = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Workgroup barrier that orders LDS traffic only: global loads issued for a later tile
// stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Asynchronous copy global -> LDS without passing through registers: lane i of the wavefront
// lands the 16 bytes at `base + voff(i)` at LDS address m0 + 16 i.  Written as assembly so that
// the compiler's wait-count pass does not serialise later LDS reads of OTHER buffers behind this
// copy; the loop waits for it explicitly before the barrier.  M0 is a register the compiler
// reserves and sets right before each of its own uses; this kernel has none (a build test checks
// that no compiler-emitted instruction of it reads M0).
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t m0) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(base), "s"(m0)
               : "memory");
}
// a pointer every lane agrees on, as two scalar registers (what the copy's base operand needs)
__device__ __forceinline__ const uint16_t* uniform_ptr(const uint16_t* q) {
  const uint64_t v = (uint64_t)(uintptr_t)q;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const uint16_t*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only

#define AGG_MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16((a).h, (b).h, (c), 0, 0, 0)

// Lane geometry of v_mfma_f32_16x16x32_bf16: c = lane & 15 is the row of the A operand, the
// column of the B operand and of the result; G = lane >> 4 selects eight of the 32 contraction
// elements (8 G .. 8 G + 7) in A and B, and result rows 4 G .. 4 G + 3.
//
// A 32-key block is scored as two 16-key tiles.  Tile kt takes the block's keys
//     row i  ->  key (i & 7) + 16 (i >> 3) + 8 kt          (tile 0: 0-7, 16-23; tile 1: 8-15, 24-31)
// so that the eight probabilities a lane holds after both tiles (rows 4 G .. 4 G + 3 of each) are
// exactly the eight keys of ONE 16-byte chunk of the compacted V tile (agg.h: chunk (t, g) holds
// keys 16 t + 4 g + {0..3, 8..11}; here t = 2 kb + (G >> 1), g = G & 1): the exponentiated scores
// are the B operand of O^T += V^T P^T as they stand, and V fragments are plain 16-byte reads.
__device__ __forceinline__ int row_key(int i) { return (i & 7) + 16 * (i >> 3); }

// sum / maximum over the four lanes c, c + 16, c + 32, c + 48 that share a query
__device__ __forceinline__ float quad_sum(float x) {
  x += __shfl_xor(x, 16);
  return pair_sum(x);
}
__device__ __forceinline__ float quad_max(float x) {
  x = fmaxf(x, __shfl_xor(x, 16));
  return pair_max(x);
}

// zero-padded rows of the last tile: key index inside the tile >= valid -> -inf
__device__ __forceinline__ void mask_unit(f32x4 (&S)[4], int kb, int valid, int G) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int km = 32 * kb + 8 * kt + row_key(4 * G + r);
      if (km >= valid) {
        S[2 * kt][r] = -INFINITY;
        S[2 * kt + 1][r] = -INFINITY;
      }
    }
}

// Everything a wavefront keeps in registers across the key loop.  qb = 32-query block, j = its
// 16-query tile, kt = 16-key tile of a key block, h = half of the channel range, dt = 16-channel
// tile of the output.
struct Wave {
  Frag Qf[kQB][4];      // [qb][2 j + h]: B operand of S^T = K Q^T, pre-multiplied by scale*log2(e)
  f32x4 O[kQB][2][4];   // [qb][j][dt]: O^T accumulator; channel = 16 dt + 4 G + r, query = c
  f32x4 S[kQB][4];      // [qb][2 kt + j]: score tiles in flight; key = row_key(4 G + r) + 8 kt
  f32x4 L[kQB][2];      // [qb][j]: fast path: the whole row sum, kept by the matrix core (four equal copies)
  float la[kQB][2];     // [qb][j]: general path: this lane's part of the row sum
  float mref[kQB][2];   // general path: the row's reference (base-2 logit)
  Frag a[4];            // [2 kt + h]: K fragments of the block whose scores are being computed
  Frag v[4];            // [dt]: V fragments of the block whose P V is being accumulated
  Frag P[2];            // [j]: probabilities of the previous unit
};

// Probabilities of the 16 base-2 logits a lane holds for a unit, packed as the B operands of
// the PV MFMAs: for query tile j, contraction elements 8 G .. 8 G + 7 are key tile 0's rows, then
// key tile 1's.  The two query tiles alternate in the instruction stream.
__device__ __forceinline__ void exp_unit(const f32x4 (&S)[4], Frag (&P)[2]) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        P[j].u[2 * kt + i] = pack_bf16(fast_exp2(S[2 * kt + j][2 * i]), fast_exp2(S[2 * kt + j][2 * i + 1]));
}

// General path: the same, and the sums of each query tile's part (there the vector ALU keeps
// the sums: the unit's own sum is what tells that a score has run away from the row's reference,
// and it is needed before the probabilities reach the matrix core)
__device__ __forceinline__ void exp_unit_sum(const f32x4 (&S)[4], Frag (&P)[2], float& l0, float& l1) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float& l = j ? l1 : l0;
        const float e0 = fast_exp2(S[2 * kt + j][2 * i]);
        const float e1 = fast_exp2(S[2 * kt + j][2 * i + 1]);
        P[j].u[2 * kt + i] = pack_bf16(e0, e1);
        l += e0;
        l += e1;
      }
}

// Where the key/value tiles come from.
//   kSrcCompact: the fragment-order compacted tensors of agg_kv_subsample: a tile is a linear
//                8 KiB copy and already in MFMA operand order.
//   kSrcRows:    consecutive rows of the token-major K and V themselves (ordinary and per-frame
//                attention: every token is a key), no compacted copy.
//   kSrcIndexed: rows of K and V picked through a list of token ids (Sec. 4.3 restricts keys
//                and values to a subset of the tokens; here the subset is read in place).
// In the two row modes a tile lies in LDS row-major, 128 bytes per key, with the 16-byte chunk
// number XOR-ed by a function of the row so that the fragment reads spread over all 64 banks:
// K fragments (eight channels of one key per lane) are plain 16-byte reads; V fragments (eight
// keys of one channel per lane) come from the transposing read ds_read_b64_tr_b16, which hands
// lane i of a 16-lane group the i-th 16-bit column of the four 8-byte rows the group's lanes
// 4j .. 4j+3 point at.
enum { kSrcCompact = 0, kSrcRows = 1, kSrcIndexed = 2 };

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

// chunk swizzle of a K row in the row modes: the 16 rows a lane group reads (i, i + 16 for eight
// consecutive i) must fall on 16 different 16-byte slots of the 256-byte bank period
__device__ __forceinline__ uint32_t k_swizzle(uint32_t row) {
  return ((row >> 1) & 3u) | (((row >> 4) & 1u) << 2);
}

// per-lane LDS byte offsets of the fragment reads (row modes) or chunk numbers (compact mode)
struct FragAddr {
  int lane;
  int kc[2];             // compact: chunk of tile kt inside a (key block, channel half) run
  int vc;                // compact: chunk inside a key block's V run (plus 16 dt)
  uint32_t k[4];         // rows: K fragment [2 kt + h]
  uint32_t v[4];         // rows: V fragment of channel tile dt (first four keys; +8 rows: the others)
};

__device__ __forceinline__ FragAddr frag_addr(int lane) {
  FragAddr f;
  const int c = lane & 15, G = lane >> 4;
  f.lane = lane;
  // compact K tile in LDS: [kb][h][G][32 keys], a key at position (key with bits 3 and 4
  // exchanged): tile kt's sixteen keys are then consecutive
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) f.kc[kt] = G * 32 + 16 * kt + c;
  f.vc = G * 64 + c;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t row = (uint32_t)(row_key(c) + 8 * kt);
      f.k[2 * kt + h] = row * 128u + (((uint32_t)(4 * h + G) ^ k_swizzle(row)) * 16u);
    }
  // V: the lanes 4 i' .. 4 i' + 3 of a 16-lane group point at row i' of the group's first four
  // keys (16 (G >> 1) + 4 (G & 1) + i'), each at 8 of the 32 bytes of channels 16 dt .. 16 dt + 15;
  // chunk bit 2 is flipped on rows 2, 3 mod 4
  const int row = 16 * (G >> 1) + 4 * (G & 1) + (c >> 2);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    const int chunk = (2 * dt + ((c & 3) >> 1)) ^ (4 * ((row >> 1) & 1));
    f.v[dt] = (uint32_t)(row * 128 + chunk * 16 + (c & 1) * 8);
  }
  return f;
}

template <int kSrc>
__device__ __forceinline__ void load_k_frags(const u32x4* __restrict__ lds, int buf, int kb,
                                             const FragAddr& f, Frag (&a)[4]) {
  if (kSrc == kSrcCompact) {
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int h = 0; h < 2; ++h)
        a[2 * kt + h].u = lds[buf * kChunks + kb * 256 + h * 128 + f.kc[kt]];
  } else {
    const lds_char* base = (const lds_char*)lds + buf * (kChunks * 16) + kb * (32 * 128);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      a[i].u = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(base + f.k[i]);
  }
}
template <int kSrc>
__device__ __forceinline__ void load_v_frags(const u32x4* __restrict__ lds, int buf, int kb,
                                             const FragAddr& f, Frag (&v)[4]) {
  if (kSrc == kSrcCompact) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
      v[dt].u = lds[(kLdsTiles + buf) * kChunks + kb * 256 + dt * 16 + f.vc];
  } else {
    lds_char* base = (lds_char*)lds + (kLdsTiles + buf) * (kChunks * 16) + kb * (32 * 128);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      // the group's first four keys, then the four that lie eight rows further on: the order
      // the P operand has
      lds_char* at = base + f.v[dt];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)at);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(at + 8 * 128));
      const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
      v[dt].u = u32x4{l2[0], l2[1], h2[0], h2[1]};
    }
  }
}

// What a workgroup needs to know about its key/value source.
struct KvSource {
  const uint16_t *k, *v;   // compact: tile 0 of this (batch, head); rows: token 0's row of this head
  const int32_t* list;     // indexed: the batch element's token ids
  int64_t rows;            // number of keys (M, or the sequence length)
  uint32_t row_bytes;      // rows: distance between consecutive tokens' rows (H * 128)
  uint32_t max_token;      // indexed: largest valid token id (N*L - 1)
};

// Issues the asynchronous copy of tile t into LDS buffer `buf`.  Every wavefront lands 64
// consecutive 16-byte LDS slots per instruction; which global chunk a lane fetches for its slot
// is what differs between the modes.
template <int kSrc>
struct TileCopier {
  KvSource src;
  const uint16_t *knext, *vnext;  // compact, rows: where the next tile to be copied starts
  int64_t tnext;                  // its number (tiles are copied in order)
  uint32_t wbase;          // LDS byte address of this wavefront's first slot in buffer 0
  uint32_t vk[2], vv[2];   // byte offset of this lane's two chunks from the tile's (rows, compact)
                           // or the row's (indexed) start, for K and for V
  uint32_t row[2];         // row of the tile this lane's slots belong to (row modes)
  int32_t tok[2];          // indexed: token ids of those rows for the next tile to be copied

  __device__ __forceinline__ void init(const KvSource& s, const u32x4* lds, int tid, int wave) {
    src = s;
    knext = s.k;
    vnext = s.v;
    tnext = 0;
    const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)lds);
    wbase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)wave * 1024u);
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const uint32_t slot = (uint32_t)tid + hh * kAttnThreads;  // 0 .. 511
      row[hh] = slot >> 3;
      const uint32_t c = slot & 7;
      const uint32_t ck = (c ^ k_swizzle(row[hh])) * 16u;
      const uint32_t cv = (c ^ (4u * ((row[hh] >> 1) & 1))) * 16u;
      if (kSrc == kSrcCompact) {
        // K: the LDS slot of a key has bits 3 and 4 of the key number exchanged (frag_addr)
        const uint32_t key = slot & 31u;
        const uint32_t swapped = (key & 7u) | ((key & 8u) << 1) | ((key & 16u) >> 1);
        vk[hh] = ((slot & ~31u) | swapped) * 16u;
        vv[hh] = slot * 16u;
      } else if (kSrc == kSrcRows) {
        vk[hh] = row[hh] * s.row_bytes + ck;
        vv[hh] = row[hh] * s.row_bytes + cv;
      } else {
        vk[hh] = ck;
        vv[hh] = cv;
      }
      tok[hh] = 0;
    }
    if (kSrc == kSrcIndexed) fetch_tokens(0);
  }
  __device__ __forceinline__ void fetch_tokens(int64_t t) {  // indexed: ids of tile t's rows
    const uint32_t m0 = (uint32_t)t * kTileRows, last = (uint32_t)src.rows - 1u;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {  // rows past the end repeat the last one; masked later
      const uint32_t id = (uint32_t)src.list[min(m0 + row[hh], last)];
      tok[hh] = (int32_t)min(id, src.max_token);  // an id outside the sequence cannot leave it
    }
  }
  // copies tile tnext into LDS buffer `buf`
  __device__ __forceinline__ void issue(int buf) {
    const uint32_t mk = wbase + (uint32_t)buf * (kChunks * 16);
    const uint32_t mv = wbase + (uint32_t)(kLdsTiles + buf) * (kChunks * 16);
    constexpr int kInstr = kAttnThreads < kChunks ? 2 : 1;
    if (kSrc == kSrcCompact) {
#pragma unroll
      for (int hh = 0; hh < kInstr; ++hh) {
        dma16(knext, vk[hh], mk + hh * kAttnThreads * 16);
        dma16(vnext, vv[hh], mv + hh * kAttnThreads * 16);
      }
      knext += kTileElems;
      vnext += kTileElems;
    } else if (kSrc == kSrcRows) {
      // the tile's rows follow each other in memory
      if ((tnext + 1) * kTileRows <= src.rows) {
#pragma unroll
        for (int hh = 0; hh < kInstr; ++hh) {
          dma16(knext, vk[hh], mk + hh * kAttnThreads * 16);
          dma16(vnext, vv[hh], mv + hh * kAttnThreads * 16);
        }
      } else {  // last, partial tile: rows past the end repeat the last one; masked later
        const uint32_t last = (uint32_t)(src.rows - 1 - tnext * kTileRows);
#pragma unroll
        for (int hh = 0; hh < kInstr; ++hh) {
          const uint32_t back = row[hh] > last ? (row[hh] - last) * src.row_bytes : 0u;
          dma16(knext, vk[hh] - back, mk + hh * kAttnThreads * 16);
          dma16(vnext, vv[hh] - back, mv + hh * kAttnThreads * 16);
        }
      }
      knext += (size_t)kTileRows * (src.row_bytes / 2);
      vnext += (size_t)kTileRows * (src.row_bytes / 2);
    } else {
      // token ids were fetched a tile ahead; the next tile's are fetched once these are used
#pragma unroll
      for (int hh = 0; hh < kInstr; ++hh) {
        const uint32_t base = __umul24((uint32_t)tok[hh], src.row_bytes);
        dma16(src.k, base + vk[hh], mk + hh * kAttnThreads * 16);
        dma16(src.v, base + vv[hh], mv + hh * kAttnThreads * 16);
      }
      fetch_tokens(tnext + 1);
    }
    ++tnext;
  }
};

// Scores of one unit: the 32 keys of block fragments `a` against the 32 queries of block tq.
// General path: the accumulator starts at minus the row's reference instead of zero, so the
// scores come out relative to it at no cost (the reference is a float, nothing is split).
template <bool kGen>
__device__ __forceinline__ void score_unit(const Wave& w, int tq, f32x4 (&Sn)[4]) {
  f32x4 init[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float m = kGen ? -w.mref[tq][j] : 0.f;
    init[j] = f32x4{m, m, m, m};
  }
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int j = 0; j < 2; ++j) Sn[2 * kt + j] = AGG_MFMA16(w.a[2 * kt], w.Qf[tq][2 * j], init[j]);
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int j = 0; j < 2; ++j)
      Sn[2 * kt + j] = AGG_MFMA16(w.a[2 * kt + 1], w.Qf[tq][2 * j + 1], Sn[2 * kt + j]);
}
// O^T += V^T P^T for the unit whose probabilities are in w.P.  Fast path: the row sums are one
// more product, a row of ones against P^T: every row of that 16 x 16 result is the sum of the
// unit's 32 probabilities of a query, so each lane keeps the whole sum and the vector ALU adds
// nothing.
template <bool kGen>
__device__ __forceinline__ void pv_unit(Wave& w, int pq) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int j = 0; j < 2; ++j) w.O[pq][j][dt] = AGG_MFMA16(w.v[dt], w.P[j], w.O[pq][j][dt]);
  if (!kGen) {
    Frag ones;
    ones.u = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
#pragma unroll
    for (int j = 0; j < 2; ++j) w.L[pq][j] = AGG_MFMA16(ones, w.P[j], w.L[pq][j]);
  }
}

// One step of the pipeline inside tile `cur` (see the file header).  kLast: the tile is the
// last one (`valid` of its 64 rows exist, nothing follows).  kGen: general path.
template <int kSrc, bool kLast, bool kGen>
__device__ __forceinline__ void tile_steps(Wave& w, const u32x4* __restrict__ lds, int cur, int nxt,
                                           int valid, const FragAddr& fa, int G) {
#pragma unroll
  for (int sg = 0; sg < 2 * kQB; ++sg) {
    const int kb = sg / kQB, qb = sg % kQB;
    const int un = sg + kQB - 1;              // unit whose scores start now
    const int tq = un % kQB;                  // its query block
    const bool beyond = un >= 2 * kQB;        // it belongs to the next tile
    const int pq = (qb + kQB - 1) % kQB;      // query block of the previous unit

    // ---- matrix core, part 1: scores of unit `un` ----
    const bool do_qk = !(kLast && beyond);
    f32x4 Sn[4];
    if (do_qk) score_unit<kGen>(w, tq, Sn);
    if (tq == kQB - 1) {  // that was the block's last unit: fragments of the following block
      if (un / kQB == 0) load_k_frags<kSrc>(lds, cur, 1, fa, w.a);
      else if (!kLast) load_k_frags<kSrc>(lds, nxt, 0, fa, w.a);
    }

    // ---- vector ALU: probabilities of unit sg ----
    Frag Pn[2];
    float u0 = 0.f, u1 = 0.f;  // general path: the unit's own row sums
    {
      f32x4 (&S)[4] = w.S[qb];
      if (kLast && valid < kTileRows) mask_unit(S, kb, valid, G);
      if (!kGen) {
        exp_unit(S, Pn);
      } else {
        // the scores are already relative to the row's reference; whether it still holds is
        // looked at below, behind the step's last MFMA
        exp_unit_sum(S, Pn, u0, u1);
      }
    }
    if (do_qk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) w.S[tq][i] = Sn[i];
    }

    // ---- matrix core, part 2: P V of unit sg - 1 ----
    pv_unit<kGen>(w, pq);
    if (qb == 0) load_v_frags<kSrc>(lds, cur, kb, fa, w.v);  // the previous block is done with them
    w.P[0] = Pn[0];
    w.P[1] = Pn[1];
    // Issue order inside the step: MFMAs and exponentials alternate one by one, a conversion
    // after every second pair (general path: pairs of MFMAs, then their share of the vector work,
    // which there includes the additions).  Left to itself the scheduler bunches the MFMAs, and
    // the wavefront then stalls on the matrix pipe with vector work still to issue.
    if (!kGen) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // the row-sum products of the last unit
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);  // transcendental
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);  // the pair's conversion
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // conversion and two additions
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (kGen) {
      // The unit's sums tell whether the reference still holds: a score more than 2^100 above it
      // cannot hide in them.  Rare, wavefront-uniform: raise the reference of the rows that need
      // it (the others keep theirs: shift 0, factor 1), scale what they have accumulated, and
      // redo the unit's probabilities (its scores are untouched until the next step).
      if (__builtin_amdgcn_ballot_w64(!(u0 + u1 < kUnitHi)) != 0) {
        f32x4 (&S)[4] = w.S[qb];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          float mx = S[j][0];
#pragma unroll
          for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, S[2 * kt + j][r]);
          mx = quad_max(mx);  // the four lanes of a row agree
          const float old = w.mref[qb][j];
          if (mx > kLazy) w.mref[qb][j] = old + mx;
          const float d = w.mref[qb][j] - old;
          const float f = fast_exp2(-d);
#pragma unroll
          for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) S[2 * kt + j][r] -= d;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) w.O[qb][j][dt][r] *= f;
          w.la[qb][j] *= f;
        }
        u0 = 0.f;
        u1 = 0.f;
        exp_unit_sum(S, w.P, u0, u1);
      }
      w.la[qb][0] += u0;
      w.la[qb][1] += u1;
    }
  }
}

// The key loop of one path.  `first_tile` runs once tile 0 is resident and its first K fragments
// are loaded (the general path takes its reference there).  Returns false when the fast path
// found a row sum it cannot trust.
template <int kSrc, bool kGen, class FirstTile>
__device__ __forceinline__ bool key_loop(Wave& w, u32x4* __restrict__ lds, const KvSource& src,
                                         int ntiles, int last_valid, int tid, int wave,
                                         const FragAddr& fa, int G, FirstTile&& first_tile) {
  TileCopier<kSrc> copy;
  copy.init(src, lds, tid, wave);
  copy.issue(0);
  if (ntiles > 1) copy.issue(1);
  wait_vm0();
  lds_barrier();

  // fill: scores of units 0 .. kQB-2; nothing to multiply by V yet
  load_k_frags<kSrc>(lds, 0, 0, fa, w.a);
  first_tile();
#pragma unroll
  for (int i = 0; i < 4; ++i) w.v[i].u = u32x4{0u, 0u, 0u, 0u};
  w.P[0].u = u32x4{0u, 0u, 0u, 0u};
  w.P[1].u = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int qb = 0; qb + 1 < kQB; ++qb) score_unit<kGen>(w, qb, w.S[qb]);

  int t = 0, cur = 0;
  bool ok = true;
  // one iteration = three tiles, so that the LDS buffer of every access is a constant
  for (int round = 0;; ++round) {
#define AGG_TILE(CUR)                                                                       \
  if (t + 1 >= ntiles) {                                                                    \
    cur = CUR;                                                                              \
    break;                                                                                  \
  }                                                                                         \
  if (t + 2 < ntiles) copy.issue((CUR + 2) % kLdsTiles);                                    \
  tile_steps<kSrc, false, kGen>(w, lds, CUR, (CUR + 1) % kLdsTiles, kTileRows, fa, G);      \
  wait_vm0();                                                                               \
  lds_barrier();                                                                            \
  ++t;
    AGG_TILE(0)
    AGG_TILE(1)
    AGG_TILE(2)
#undef AGG_TILE
    if (!kGen && (round & 7) == 7) {  // an overflowing row ends the fast pass early
      bool bad = false;
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb)
        bad = bad || !(w.L[qb][0][0] < kSumHi) || !(w.L[qb][1][0] < kSumHi);
      if (__syncthreads_or(bad ? 1 : 0)) {
        ok = false;
        break;
      }
    }
  }
  if (!ok) return false;
  // last tile (runtime buffer number), then the P V of its last unit
  tile_steps<kSrc, true, kGen>(w, lds, cur, 0, last_valid, fa, G);
  pv_unit<kGen>(w, kQB - 1);
  return true;
}

// Kernel arguments.
struct AttnArgs {
  Geom g;
  uint32_t flags;
  float qscale, mean_bias2;  // scale*log2(e), mean_logit_bias*log2(e)
  const uint16_t *Q, *K, *V, *Kc, *Vc;
  const float *kmean, *vmean;
  uint16_t* O;
  float* lse;
  int nqt, npairs;
  const uint32_t* kept_bits;
  const int32_t* nd_dev;
  const int32_t* list;   // kSrcIndexed: token ids of the keys, [list_stride] per batch element
  int64_t list_stride;   // 0 when every batch element uses the same list
};

__shared__ __align__(16) uint16_t smem[2 * kLdsTiles * kTileElems];  // K tiles, then V tiles

// One workgroup's rows by one of the two paths.  Returns false, without storing anything, when
// the fast path met a row it cannot handle.
template <int kSrc, bool kGen>
__device__ __forceinline__ bool attend(const AttnArgs& p, int b, int h, int qt) {
  const Geom& g = p.g;
  u32x4* lds = reinterpret_cast<u32x4*>(smem);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int c = lane & 15;
  const int G = lane >> 4;
  const FragAddr fa = frag_addr(lane);

  const int ntiles = (int)(g.M_pad / kTileRows);
  const int last_valid = (int)(g.M - (int64_t)(ntiles - 1) * kTileRows);  // 1..64
  KvSource src;
  src.rows = g.M;
  src.row_bytes = (uint32_t)g.H * (kHeadDim * 2);
  src.max_token = (uint32_t)(g.NQ - 1);
  if (kSrc == kSrcCompact) {
    const int64_t bh_off = ((int64_t)b * g.H + h) * g.M_pad * kHeadDim;
    src.k = uniform_ptr(p.Kc + bh_off);
    src.v = uniform_ptr(p.Vc + bh_off);
    src.list = nullptr;
  } else {
    const int64_t bh_off = ((int64_t)b * g.NQ * g.H + h) * kHeadDim;
    src.k = uniform_ptr(p.K + bh_off);
    src.v = uniform_ptr(p.V + bh_off);
    src.list = kSrc == kSrcIndexed ? p.list + (int64_t)b * p.list_stride : nullptr;
  }

  Wave w;
  bool dropped[kQB][2];
  float l_self[kQB][2], l_mean[kQB][2];  // base-2 logits of the extras (-inf when absent)
  // caller's list: membership comes from a bitmap, the dropped count from device memory
  const int64_t n_drop = p.nd_dev ? (int64_t)p.nd_dev[b] : g.n_dropped;
  const bool use_mean = (p.flags & AGG_MEAN) && n_drop > 0;
  const bool use_diag = (p.flags & AGG_DIAG) && (p.kept_bits != nullptr || n_drop > 0);
  const uint32_t* kbits = p.kept_bits ? p.kept_bits + (int64_t)b * ((g.NQ + 31) / 32) : nullptr;
  const int64_t q_wave = (int64_t)qt * kQTile + wave * kWaveQ;
  // first element of query (qb, j, c)'s row of this head in Q, K, V and O
  auto row_base = [&](int qb, int j) {
    const int64_t q = q_wave + qb * 32 + j * 16 + c;
    const int64_t qc = q < g.NQ ? q : g.NQ - 1;  // tail rows recompute the last query, never stored
    return (((int64_t)b * g.NQ + qc) * g.H + h) * kHeadDim;
  };

  // ---- Q fragments and the logits of the extras ----
  // a lane holds channels 32 h + 8 G .. + 7 (h = 0, 1) of its query: the four lanes c + 16 G
  // share the channel range
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t q = q_wave + qb * 32 + j * 16 + c;
      const int64_t qbase = row_base(qb, j);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        u32x4 raw = *reinterpret_cast<const u32x4*>(p.Q + qbase + hh * 32 + G * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          w.Qf[qb][2 * j + hh].u[i] =
              pack_bf16(bf16_lo(raw[i]) * p.qscale, bf16_hi(raw[i]) * p.qscale);
      }
      dropped[qb][j] =
          use_diag && q < g.NQ &&
          (kbits ? ((kbits[q >> 5] >> (q & 31)) & 1u) == 0u : (bool)token_is_dropped(g, q));
      float dot_self = 0.f, dot_mean = 0.f;
      if (use_mean || use_diag) {
        const float* km = p.kmean + ((int64_t)b * g.H + h) * kHeadDim;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int d0 = hh * 32 + G * 8;
          float qv[8];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            qv[2 * i] = bf16_lo(w.Qf[qb][2 * j + hh].u[i]);
            qv[2 * i + 1] = bf16_hi(w.Qf[qb][2 * j + hh].u[i]);
          }
          if (use_mean) {
            f32x4 c0 = *reinterpret_cast<const f32x4*>(km + d0);
            f32x4 c1 = *reinterpret_cast<const f32x4*>(km + d0 + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) dot_mean += qv[i] * c0[i] + qv[4 + i] * c1[i];
          }
          if (dropped[qb][j]) {
            u32x4 kr = *reinterpret_cast<const u32x4*>(p.K + qbase + d0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              dot_self += qv[2 * i] * bf16_lo(kr[i]) + qv[2 * i + 1] * bf16_hi(kr[i]);
          }
        }
      }
      dot_self = quad_sum(dot_self);
      dot_mean = quad_sum(dot_mean);
      l_self[qb][j] = dropped[qb][j] ? dot_self : -INFINITY;
      l_mean[qb][j] = use_mean ? dot_mean + p.mean_bias2 : -INFINITY;
    }

  // Initial state = extras weighted by exp2(logit - m0):  O0[d] = w_self v_i[d] + w_mean vmean[d]
  auto init_extras = [&](int qb, int j, float m0) {
    const float w_self = dropped[qb][j] ? fast_exp2(l_self[qb][j] - m0) : 0.f;
    const float w_mean = use_mean ? fast_exp2(l_mean[qb][j] - m0) : 0.f;
    const float l0 = w_self + w_mean;
    if (kGen) w.la[qb][j] = (G == 0) ? l0 : 0.f;  // four lanes split a row's sum
    else w.L[qb][j] = f32x4{l0, l0, l0, l0};      // every lane keeps the whole sum
    const int64_t qbase = row_base(qb, j);
    const float* vm = p.vmean + ((int64_t)b * g.H + h) * kHeadDim;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const int d0 = 16 * dt + 4 * G;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      if (use_mean) {
        f32x4 mv = *reinterpret_cast<const f32x4*>(vm + d0);
        acc = mv * w_mean;
      }
      if (dropped[qb][j]) {
        u32x2 vr = *reinterpret_cast<const u32x2*>(p.V + qbase + d0);
        acc[0] += w_self * bf16_lo(vr[0]);
        acc[1] += w_self * bf16_hi(vr[0]);
        acc[2] += w_self * bf16_lo(vr[1]);
        acc[3] += w_self * bf16_hi(vr[1]);
      }
      w.O[qb][j][dt] = acc;
    }
  };

  if (!kGen) {
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        w.mref[qb][j] = 0.f;
        init_extras(qb, j, 0.f);
      }
  }
  // general path: the reference is the largest of the extras and of the first 32 keys (row 0
  // always exists); taken when the first tile's K fragments are in registers
  auto first_tile = [&]() {
    if (!kGen) return;
    const int valid0 = ntiles == 1 ? last_valid : kTileRows;
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
      w.mref[qb][0] = 0.f;
      w.mref[qb][1] = 0.f;
      f32x4 s[4];
      score_unit<kGen>(w, qb, s);
      if (valid0 < 32) mask_unit(s, 0, valid0, G);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float mx = s[j][0];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[2 * kt + j][r]);
        mx = quad_max(mx);
        mx = fmaxf(mx, fmaxf(l_self[qb][j], l_mean[qb][j]));
        // a NaN or infinite score cannot serve as reference; the row's result is NaN anyway
        if (!(fabsf(mx) < 3.0e38f)) mx = 0.f;
        w.mref[qb][j] = mx;
        init_extras(qb, j, mx);
      }
    }
  };

  const bool done = key_loop<kSrc, kGen>(w, lds, src, ntiles, last_valid, tid, wave, fa, G,
                                         first_tile);
  float l_fin[kQB][2];
  bool unsafe = false;
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      l_fin[qb][j] = kGen ? quad_sum(w.la[qb][j]) : w.L[qb][j][0];
      // a sum outside [2^-90, 2^90] (or NaN): the unreferenced exponentials were not safe
      unsafe = unsafe || !(l_fin[qb][j] < kSumHi) || !(l_fin[qb][j] > kSumLo);
    }
  if (!kGen) {
    if (!done) return false;  // uniform: decided by a workgroup-wide vote inside the loop
    if (__syncthreads_or(unsafe ? 1 : 0)) return false;
  }

  // ---- normalise and store ----
  // A lane holds four consecutive channels of one query per accumulator tile: stored from there,
  // every instruction would scatter 8-byte pieces over 16 rows that lie 2*H*64 bytes apart.
  // Each wavefront instead turns its tile, 32 queries at a time, through a private part of the
  // (now idle) K/V LDS and writes whole 128-byte (query, head) rows, eight per instruction.
  __syncthreads();  // every wavefront is done with the K/V tiles
  uint16_t* epi = smem + wave * (32 * kEpiStride);
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const int64_t q0 = q_wave + qb * 32;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float l = l_fin[qb][j];
      const float inv = 1.0f / l;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const int d0 = 16 * dt + 4 * G;
        u32x2 o2;
        o2[0] = pack_bf16(w.O[qb][j][dt][0] * inv, w.O[qb][j][dt][1] * inv);
        o2[1] = pack_bf16(w.O[qb][j][dt][2] * inv, w.O[qb][j][dt][3] * inv);
        *reinterpret_cast<u32x2*>(epi + (16 * j + c) * kEpiStride + d0) = o2;
      }
      if (p.lse && G == 0 && q0 + 16 * j + c < g.NQ)
        p.lse[((int64_t)b * g.H + h) * g.NQ + q0 + 16 * j + c] =
            ((kGen ? w.mref[qb][j] : 0.f) + log2f(l)) * kLn2;
    }
    // the wavefront's own writes, read back by other lanes of the same wavefront
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = i * 8 + (lane >> 3);
      const int64_t q = q0 + row;
      const u32x4 o4 = *reinterpret_cast<const u32x4*>(epi + row * kEpiStride + (lane & 7) * 8);
      if (q < g.NQ)
        *reinterpret_cast<u32x4*>(p.O + (((int64_t)b * g.NQ + q) * g.H + h) * kHeadDim +
                                  (lane & 7) * 8) = o4;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  }
  return true;
}

// A workgroup whose fast pass failed leaves this pattern (four bf16 NaNs with distinct payloads)
// in the first four channels of its first output row and stores nothing else; the second kernel
// redoes exactly the workgroups that carry it.  Should a correct result ever equal the pattern,
// the second kernel recomputes that workgroup, which is harmless.
constexpr uint64_t kRedoMark = 0x7F997FC37FA57FC1ull;

__device__ __forceinline__ uint64_t* redo_slot(const AttnArgs& p, int b, int h, int qt) {
  return reinterpret_cast<uint64_t*>(p.O + (((int64_t)b * p.g.NQ + (int64_t)qt * kQTile) * p.g.H + h) *
                                               kHeadDim);
}

// workgroup -> ((batch, head) pair, query tile); consecutive ids go to consecutive XCDs
__device__ __forceinline__ bool workgroup_tile(const AttnArgs& p, int& b, int& h, int& qt) {
  const int bid = blockIdx.x;
  const int xcd = bid % kXcds;
  const int seq = bid / kXcds;
  const int pair = (seq / p.nqt) * kXcds + xcd;
  qt = seq % p.nqt;
  if (pair >= p.npairs) return false;  // uniform for the whole workgroup
  b = pair / p.g.H;
  h = pair % p.g.H;
  return true;
}

template <int kSrc>
__global__ __launch_bounds__(kAttnThreads, kBlocksPerCu) void sga_attn_kernel(AttnArgs p) {
  int b, h, qt;
  if (!workgroup_tile(p, b, h, qt)) return;
  if (!attend<kSrc, false>(p, b, h, qt) && threadIdx.x == 0) *redo_slot(p, b, h, qt) = kRedoMark;
}

// The general path is a kernel of its own, launched behind the first on the same stream: it is
// rarely needed, starts over from the workgroup's inputs, and this way does not weigh on the
// register allocation of the fast path.  Workgroups without the mark leave at once.
template <int kSrc>
__global__ __launch_bounds__(kAttnThreads, kBlocksPerCu) void sga_attn_general_kernel(AttnArgs p) {
  int b, h, qt;
  if (!workgroup_tile(p, b, h, qt)) return;
  if (*redo_slot(p, b, h, qt) != kRedoMark) return;  // same value in every lane
  __syncthreads();  // every wavefront has read the mark before any of them overwrites it
  attend<kSrc, true>(p, b, h, qt);
}

hipError_t launch_attn(const Geom& g, uint32_t flags, float scale, float mean_bias, const void* Q,
                       const void* K, const void* V, const void* Kc, const void* Vc,
                       const float* kmean, const float* vmean, void* O, float* lse, hipStream_t st,
                       const uint32_t* kept_bits, const int32_t* nd_dev, int src_mode,
                       const int32_t* list, int64_t list_stride) {
  const int nqt = (int)((g.NQ + kQTile - 1) / kQTile);
  const int npairs = g.B * g.H;
  const int64_t groups = (int64_t)((npairs + kXcds - 1) / kXcds) * kXcds * nqt;
  if (groups > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
  // indexed rows are addressed with 32-bit byte offsets from the (batch, head) base, formed by
  // a 24-bit multiplication of token id and row length
  if (src_mode == kSrcIndexed && ((uint64_t)g.NQ * g.H * (kHeadDim * 2) > 0xFFFFFFFFull ||
                                  g.NQ > 0xFFFFFF || (uint64_t)g.H * (kHeadDim * 2) > 0xFFFFFF))
    return hipErrorInvalidValue;
  (void)hipGetLastError();  // drop any stale error so the check below is this launch's
  AttnArgs p;
  p.g = g;
  p.flags = flags;
  p.qscale = scale * kLog2e;
  p.mean_bias2 = mean_bias * kLog2e;
  p.Q = (const uint16_t*)Q;
  p.K = (const uint16_t*)K;
  p.V = (const uint16_t*)V;
  p.Kc = (const uint16_t*)Kc;
  p.Vc = (const uint16_t*)Vc;
  p.kmean = kmean;
  p.vmean = vmean;
  p.O = (uint16_t*)O;
  p.lse = lse;
  p.nqt = nqt;
  p.npairs = npairs;
  p.kept_bits = kept_bits;
  p.nd_dev = nd_dev;
  p.list = list;
  p.list_stride = list_stride;
  const dim3 grid((unsigned)groups), block(kAttnThreads);
  if (src_mode == kSrcCompact) {
    hipLaunchKernelGGL(sga_attn_kernel<kSrcCompact>, grid, block, 0, st, p);
    hipLaunchKernelGGL(sga_attn_general_kernel<kSrcCompact>, grid, block, 0, st, p);
  } else if (src_mode == kSrcRows) {
    hipLaunchKernelGGL(sga_attn_kernel<kSrcRows>, grid, block, 0, st, p);
    hipLaunchKernelGGL(sga_attn_general_kernel<kSrcRows>, grid, block, 0, st, p);
  } else {
    hipLaunchKernelGGL(sga_attn_kernel<kSrcIndexed>, grid, block, 0, st, p);
    hipLaunchKernelGGL(sga_attn_general_kernel<kSrcIndexed>, grid, block, 0, st, p);
  }
  return hipGetLastError();
}

}  // namespace agg

/*
 * agg -- subsampled global attention (SGA) for VGGT-style models on AMD MI355X (gfx950).
 *
 * C ABI of libagg.so.  The operation is the one the AVGGT paper defines in its
 * Sec. 4.3 ("Subsampling Global Attention") on the token layout of its Sec. 4.1:
 * a sequence is N frames of L = n_special + n_h*n_w tokens; every token is a
 * query; keys/values are all special tokens, all of frame 0 when the reference
 * frame is kept whole, and on every other patch grid the first token of each
 * s_h x s_w window; a query whose own token was dropped also sees its own
 * key/value ("diagonal preservation"); all dropped patches are represented by
 * one mean key/value pair; the three parts share one softmax.
 *
 * Conventions
 *   - Token id inside a sequence: i = f*L + t.  t < n_special is a special token,
 *     otherwise patch p = t - n_special at grid row p / n_w, column p % n_w.
 *   - Q, K, V, O: bf16, device memory, contiguous [B, N*L, H, D] (token-major:
 *     what a fused QKV projection writes and an output projection reads).
 *   - D must be 64.  Pointers to bf16 tensors, to workspaces and to kmean/vmean must be
 *     16-byte aligned; index, count, bitmap and lse pointers 4-byte aligned.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call only enqueues work on that stream: no allocation, no
 *     synchronisation, no retained pointers.  The caller owns every buffer.
 *   - Return value: AGG_OK or a negative agg_status.  All argument validation
 *     happens before the first launch, so every error except AGG_ERR_LAUNCH is
 *     reported without touching the GPU.  Faults inside a kernel surface at the
 *     caller's next synchronisation, as with any HIP launch.
 *
 * Compacted key/value format ("fragment order")
 *   Kc and Vc hold, per (batch, head), the M kept rows padded with zero rows to
 *   M_pad = 64*ceil(M/64), as consecutive 64-row tiles of 4096 bf16 (8 KiB).
 *   Inside a tile the elements are grouped in 16-byte chunks (eight channels of
 *   one key for Kc, eight keys of one channel for Vc) such that a copy into LDS
 *   chunk by chunk lets every wavefront lane fetch its MFMA operand as one
 *   16-byte read:
 *     Kc: row m, channel d  ->  tile m/64, then with km = m%64
 *         ((( (km/32)*4 + d/16 )*2 + (d%16)/8 )*32 + km%32)*8 + d%8
 *     Vc: row m, channel d  ->  tile m/64, then with km = m%64, u = km%16
 *         ((( km/16 )*2 + (u%8)/4 )*64 + d)*8 + (u/8)*4 + u%4
 *   agg_kc_offset()/agg_vc_offset() evaluate these on the host.  Row m of the
 *   compacted set is token idx[m]; idx is ascending.
 */
#ifndef AGG_H_
#define AGG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct agg_shape {
  int32_t B, N;             /* batch size, frames                       (Sec. 4.1) */
  int32_t n_h, n_w;         /* patch grid                               (Sec. 4.1) */
  int32_t n_special;        /* special tokens per frame, stored before the patches */
  int32_t H, D;             /* heads, head dimension (D = 64)                      */
  int32_t s_h, s_w;         /* window strides; (1,1) = no subsampling   (Sec. 4.3) */
  int32_t keep_first_frame; /* 1: frame 0 kept whole (VGGT); 0: all frames (pi^3)  */
  uint32_t flags;           /* AGG_DIAG | AGG_MEAN                      (Sec. 4.3) */
  float scale;              /* softmax scale, 1/sqrt(D)                            */
  float mean_logit_bias;    /* added to the mean column's logit; 0 = one plain column */
} agg_shape;

enum { AGG_DIAG = 1u, AGG_MEAN = 2u };

typedef enum agg_status {
  AGG_OK = 0,
  AGG_ERR_NULL = -1,        /* a required pointer is NULL                          */
  AGG_ERR_SHAPE = -2,       /* a dimension or stride is < 1, or flags unknown      */
  AGG_ERR_UNSUPPORTED = -3, /* D != 64; a block wider than 4096 channels           */
  AGG_ERR_ALIGN = -4,       /* a tensor pointer is not 16-byte aligned             */
  AGG_ERR_WORKSPACE = -5,   /* workspace smaller than the matching *_workspace_bytes */
  AGG_ERR_OVERFLOW = -6,    /* N*L, M_pad or a tensor's element count exceeds the index range */
  AGG_ERR_LAUNCH = -7       /* hipGetLastError() after a launch was not hipSuccess */
} agg_status;

const char* agg_status_string(int status);

/* Sec. 4.3 table: sigma in {2,4,6,9} -> (s_h, s_w) = (1,2),(2,2),(2,3),(3,3); sigma 1 -> (1,1).
 * Any other sigma: AGG_ERR_SHAPE. */
int agg_sigma_to_strides(int sigma, int32_t* s_h, int32_t* s_w);

/* Host only.  M = number of kept key/value rows per sequence,
 * n_dropped = number of patch tokens left out (Sec. 4.3).  Either output may be NULL. */
int agg_kv_count(const agg_shape* shape, int64_t* M, int64_t* n_dropped);

/* Host only.  The index set of Sec. 4.3 (special tokens, the reference frame when kept whole,
 * the first patch of every s_h x s_w window), as ascending token ids, into idx[M] (host memory):
 * what agg_kv_subsample writes on the device. */
int agg_kv_indices_host(const agg_shape* shape, int32_t* idx);

/* Host only.  Writes the ascending token ids of the dropped patches (the set the mean
 * component averages, Sec. 4.3) into idx[n_dropped] (host memory). */
int agg_dropped_indices_host(const agg_shape* shape, int32_t* idx);

/* Host only.  Size of ONE compacted tensor (Kc or Vc) in bytes, B*H*M_pad*D*2, and M_pad. */
int agg_kv_compact_bytes(const agg_shape* shape, size_t* bytes, int64_t* M_pad);

/* Host only.  Element offsets inside one (batch, head) block of Kc / Vc (see above). */
int64_t agg_kc_offset(int64_t m, int32_t d);
int64_t agg_vc_offset(int64_t m, int32_t d);

/* Host only.  Scratch bytes agg_kv_subsample needs: the partial sums from which the mean
 * component of Sec. 4.3 (one mean key/value pair over all dropped patches) is formed in a fixed
 * order. */
size_t agg_workspace_bytes(const agg_shape* shape);

/*
 * Sec. 4.3, subsampling + mean component.  Builds on the device:
 *   idx   [M] int32        ascending kept token ids (same for every batch element/head/layer)
 *   Kc,Vc bf16, agg_kv_compact_bytes() each, fragment order, zero padded
 *   kmean,vmean [B,H,D] float32: mean of K resp. V over all dropped patch tokens of the
 *         sequence (zeros when nothing is dropped).  Accumulated in a fixed order:
 *         results are bit-reproducible run to run.
 * K, V: device bf16 [B, N*L, H, D].  workspace: device, >= agg_workspace_bytes().
 * idx may be NULL (not written).  kmean/vmean must be non-NULL.  Kc and Vc may BOTH be NULL:
 * then no compacted copy is made and only idx and the mean terms are produced, which is all
 * that agg_global_attn_fwd_idx needs.
 */
int agg_kv_subsample(const agg_shape* shape, const void* K, const void* V, void* Kc, void* Vc,
                     int32_t* idx, float* kmean, float* vmean, void* workspace,
                     size_t workspace_bytes, void* hip_stream);

/*
 * agg_kv_subsample for callers that cannot allocate device memory and so cannot bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results, minus the workspace: the
 * partial sums of the mean go to a device array that is part of the library (each GPU the
 * library runs on holds agg_static_scratch_bytes() = 32 MiB of it until the process ends).
 * The call allocates nothing.  Shapes whose agg_workspace_bytes() exceeds
 * agg_static_scratch_bytes() are refused with AGG_ERR_WORKSPACE before anything is launched.
 * The first call on a device looks the array's address up (with that device current, which it
 * must be for every call).  All calls on one GPU share the array: two calls whose work may
 * overlap on that GPU (different streams) race; calls on one stream do not.
 */
size_t agg_static_scratch_bytes(void);
int agg_kv_subsample_static(const agg_shape* shape, const void* K, const void* V, void* Kc,
                            void* Vc, int32_t* idx, float* kmean, float* vmean, void* hip_stream);

/*
 * Sec. 4.3, the attention itself.  For every query i of every (batch, head):
 *   softmax over { scale*<q_i, Kc[m]> : m < M }
 *                u { scale*<q_i, k_i> }                    if AGG_DIAG and token i was dropped
 *                u { scale*<q_i, kmean> + mean_logit_bias } if AGG_MEAN and n_dropped > 0
 *   O[i] = sum of the probabilities times the matching value rows (Vc[m], v_i, vmean).
 * Q, K, V: device bf16 [B, N*L, H, D] (K, V are read only for the self terms).
 * Kc, Vc, kmean, vmean: as written by agg_kv_subsample for the same shape.
 * O: device bf16 [B, N*L, H, D].  lse: device float32 [B, H, N*L] (natural-log
 * log-sum-exp of each row's logits) or NULL.
 * With s_h = s_w = 1 nothing is dropped and the result is ordinary global attention.
 */
int agg_global_attn_fwd(const agg_shape* shape, const void* Q, const void* K, const void* V,
                        const void* Kc, const void* Vc, const float* kmean, const float* vmean,
                        void* O, float* lse, void* hip_stream);

/*
 * Sec. 4.3 again, without a compacted copy: the same attention as agg_global_attn_fwd, with the
 * kernel fetching the kept rows of K and V in place through idx (the paper's statement is just
 * that: only a subset of the tokens serves as keys and values).  idx: device int32 [M], the
 * ascending kept token ids as agg_kv_subsample writes them; kmean, vmean: as above.  Results are
 * bit-identical to agg_global_attn_fwd.  Needs N*L < 2^24 and N*L*H*D*2 < 2^32 (rows are
 * addressed with 32-bit offsets inside one batch element's head); otherwise AGG_ERR_OVERFLOW.
 */
int agg_global_attn_fwd_idx(const agg_shape* shape, const void* Q, const void* K, const void* V,
                            const int32_t* idx, const float* kmean, const float* vmean, void* O,
                            float* lse, void* hip_stream);

/*
 * Sec. 4.2: ordinary global attention over the (B, N*L, C) layout -- every token of the
 * sequence is a key -- the s = 1 baseline SGA is measured against.  shape->s_h, s_w,
 * flags and keep_first_frame are ignored.  K and V are read in place (no copy, no workspace).
 */
int agg_dense_global_attn_fwd(const agg_shape* shape, const void* Q, const void* K, const void* V,
                              void* O, float* lse, void* hip_stream);

/*
 * Sec. 4.2, Global-to-Frame conversion: attention applied independently inside every frame,
 * i.e. on the (B*N, L, C) layout -- what an early global block becomes when its rearrangement
 * to (B, N*L, C) is skipped.  Q, K, V, O: the same device tensors as above (a frame's tokens are
 * contiguous in them).  lse: device float32 [B*N, H, L] or NULL.  shape->s_h, s_w, flags and
 * keep_first_frame are ignored.
 */
int agg_frame_attn_fwd(const agg_shape* shape, const void* Q, const void* K, const void* V, void* O,
                       float* lse, void* hip_stream);

/*
 * One global-attention block around the calls above (Sec. 4.2: a converted or subsampled
 * block keeps all its other components and parameters):
 *     y = x + W_o * Attn( Q, K, V ) + b_o,   [Q|K|V] = W_{q,k,v} * LayerNorm(x) + b_{q,k,v}
 * with Attn chosen by `mode`.  x, y: device bf16 [B, N*L, C], C = H*D (y may not alias x).
 * Weights: device memory; w_*: bf16 [C, C], one row per OUTPUT channel (y = x W^T);
 * b_* (may be NULL), ln_gamma, ln_beta: float32 [C].  Q, K, V and the attention output
 * are bf16 tensors in the workspace, as in the calls above.  Rotary embeddings or
 * query/key normalisation, which the paper's text does not describe, are not applied.
 * C may be at most 4096 (64 heads): wider blocks return AGG_ERR_UNSUPPORTED.
 */
typedef struct agg_block_weights {
  const float* ln_gamma;
  const float* ln_beta;
  float ln_eps;
  const void *w_q, *w_k, *w_v, *w_o;
  const float *b_q, *b_k, *b_v, *b_o;
} agg_block_weights;

enum {
  AGG_BLOCK_SGA = 0,   /* subsampled global attention, Sec. 4.3 (shape's strides and flags) */
  AGG_BLOCK_FRAME = 1, /* frame attention: the Global-to-Frame conversion, Sec. 4.2         */
  AGG_BLOCK_DENSE = 2  /* ordinary global attention                                         */
};

/* Host only.  Scratch bytes agg_global_block_fwd needs for `mode` (0 on an invalid shape). */
size_t agg_block_workspace_bytes(const agg_shape* shape, int mode);

int agg_global_block_fwd(const agg_shape* shape, int mode, const agg_block_weights* weights,
                         const void* x, void* y, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * ---- Caller-supplied key/value sets (supplementary ablation on the grid strategy) ----
 * The paper compares its fixed choice (first token of each window) with other choices of one
 * token per window: a random one, the one with the highest and the one with the lowest feature
 * magnitude.  These calls run the same attention over ANY list of kept tokens:
 *   list       device int32 [B, M_list]: token ids (0 <= id < N*L) whose K/V rows serve as
 *              keys/values of that batch element, in any order.  Ids outside the range are
 *              clamped into it (memory-safe, meaningless result); a repeated id counts twice.
 *   kept_bits  device uint32 [B, ceil(N*L/32)]: bit t%32 of word t/32 set <=> token t is listed
 *   n_dropped  device int32 [B]: patch tokens (slot >= n_special) that are not listed
 * The self term (AGG_DIAG) applies to every query whose token is not listed, the mean
 * component (AGG_MEAN) averages K resp. V over the unlisted patch tokens and is present when
 * n_dropped[b] > 0.  shape->s_h, s_w, keep_first_frame matter only to agg_select_kv_indices.
 */
enum {
  AGG_SELECT_FIRST = 0,  /* top-left token of each window: the paper's rule (Sec. 4.3)        */
  AGG_SELECT_RANDOM = 1, /* a pseudo-random token of each window                              */
  AGG_SELECT_HIGH = 2,   /* the token of each window with the largest sum of squares of its K */
  AGG_SELECT_LOW = 3     /* ... with the smallest                                             */
};

/*
 * Writes list[B, M] (M of agg_kv_count): row m of batch b is the token chosen for the m-th
 * kept position of the grid rule -- special tokens and (keep_first_frame) frame 0 map to
 * themselves, the m-th window of a subsampled frame to one of its tokens by `rule`:
 *   RANDOM: cell number  mix(mix(s ^ (b*N+frame)*0x85EBCA77) ^ window*0xC2B2AE3D) % cells,
 *           s = (uint32)seed ^ (uint32)(seed>>32)*0x9E3779B1, window = row-major window number
 *           inside the frame, cells counted row-major inside the (possibly clipped) window,
 *           mix(x): x^=x>>16; x*=0x7FEB352D; x^=x>>15; x*=0x846CA68B; x^=x>>16  (32-bit);
 *   HIGH/LOW: magnitude = sum over all H*D channels of K[b, token]^2 in float32; ties go to
 *           the earlier cell.
 * K: device bf16 [B, N*L, H, D]; read only for HIGH/LOW (may be NULL otherwise).
 */
int agg_select_kv_indices(const agg_shape* shape, int rule, uint64_t seed, const void* K,
                          int32_t* list, void* hip_stream);

/*
 * The cell-mean variant of the same ablation: Kc/Vc (agg_kv_compact_bytes each, M rows as for
 * agg_kv_subsample) where the row of a window is the MEAN of the window's tokens (float32
 * accumulation, rounded to bf16 once) instead of its first token; special tokens and a
 * whole-kept frame 0 are copied.  The paper runs this variant without the self term and without
 * the mean component: call agg_global_attn_fwd on the result with flags = 0.
 */
int agg_kv_pool(const agg_shape* shape, const void* K, const void* V, void* Kc, void* Vc,
                void* hip_stream);

/* Host only.  Size of ONE compacted tensor for a list of M_list rows, and its M_pad. */
int agg_list_compact_bytes(const agg_shape* shape, int64_t M_list, size_t* bytes, int64_t* M_pad);

/* Host only.  Scratch bytes agg_kv_subsample_list needs (0 on an invalid shape). */
size_t agg_list_workspace_bytes(const agg_shape* shape);

/* As agg_kv_subsample, for a caller's list: Kc/Vc (agg_list_compact_bytes each; row m of batch
 * b = token list[b, m]), kmean/vmean [B,H,D], kept_bits and n_dropped as defined above. */
int agg_kv_subsample_list(const agg_shape* shape, const int32_t* list, int64_t M_list,
                          const void* K, const void* V, void* Kc, void* Vc, float* kmean,
                          float* vmean, uint32_t* kept_bits, int32_t* n_dropped, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/* As agg_global_attn_fwd, over what agg_kv_subsample_list wrote for the same shape and M_list. */
int agg_global_attn_fwd_list(const agg_shape* shape, int64_t M_list, const void* Q, const void* K,
                             const void* V, const void* Kc, const void* Vc, const float* kmean,
                             const float* vmean, const uint32_t* kept_bits,
                             const int32_t* n_dropped, void* O, float* lse, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AGG_H_ */

// Host side of libagg: argument validation, geometry, counts, index list and
// the extern "C" entry points declared in agg.h.  Nothing here allocates device
// memory or synchronises; every check runs before the first launch.
#include <limits.h>
#include <string.h>

#include "agg_internal.h"

namespace agg {

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Fills Geom from the caller's shape.  `dense` ignores the subsampling fields
// and treats every token as kept (Sec. 4.2: plain global attention).
int make_geom(const agg_shape* s, Geom* g, bool dense) {
  if (!s || !g) return AGG_ERR_NULL;
  if (s->B < 1 || s->N < 1 || s->n_h < 1 || s->n_w < 1 || s->n_special < 0 || s->H < 1 ||
      s->D < 1)
    return AGG_ERR_SHAPE;
  if (!dense) {
    if (s->s_h < 1 || s->s_w < 1) return AGG_ERR_SHAPE;
    if (s->flags & ~(uint32_t)(AGG_DIAG | AGG_MEAN)) return AGG_ERR_SHAPE;
    if (s->keep_first_frame != 0 && s->keep_first_frame != 1) return AGG_ERR_SHAPE;
  }
  if (!(s->scale > 0.0f) || !(s->scale < 1e30f)) return AGG_ERR_SHAPE;
  if (!(s->mean_logit_bias > -1e30f && s->mean_logit_bias < 1e30f)) return AGG_ERR_SHAPE;
  if (s->D != kHeadDim) return AGG_ERR_UNSUPPORTED;

  int64_t T = (int64_t)s->n_h * s->n_w;
  int64_t L = T + s->n_special;
  if (L > INT32_MAX) return AGG_ERR_OVERFLOW;
  int64_t NQ = (int64_t)s->N * L;
  // token ids and compacted row numbers are int32; tile padding must also fit
  if (NQ > (int64_t)INT32_MAX - 2 * kTileRows) return AGG_ERR_OVERFLOW;
  // element offsets are 64-bit in the kernels, but keep one tensor under 2^62 bytes
  if ((int64_t)s->B * s->H > ((int64_t)1 << 40) / NQ) return AGG_ERR_OVERFLOW;

  g->B = s->B;
  g->N = s->N;
  g->L = (int32_t)L;
  g->P = s->n_special;
  g->n_h = s->n_h;
  g->n_w = s->n_w;
  g->H = s->H;
  g->s_h = dense ? 1 : s->s_h;
  g->s_w = dense ? 1 : s->s_w;
  g->keep_first = dense ? 0 : s->keep_first_frame;
  // a stride larger than the grid keeps one row/column of windows (edge windows count)
  g->kw = (int32_t)ceil_div(s->n_w, g->s_w);
  g->kf = (int32_t)(ceil_div(s->n_h, g->s_h) * g->kw);
  g->rows_sub = g->P + g->kf;
  g->dw = g->n_w - g->kw;
  g->df = (int32_t)(T - g->kf);
  g->NQ = NQ;
  int64_t f0 = g->keep_first ? 1 : 0;
  g->M = f0 * L + ((int64_t)s->N - f0) * g->rows_sub;
  g->M_pad = ceil_div(g->M, kTileRows) * kTileRows;
  g->n_dropped = ((int64_t)s->N - f0) * g->df;
  return AGG_OK;
}

static bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

}  // namespace agg

using namespace agg;

extern "C" {

const char* agg_status_string(int status) {
  switch (status) {
    case AGG_OK: return "ok";
    case AGG_ERR_NULL: return "a required pointer is NULL";
    case AGG_ERR_SHAPE: return "invalid shape, stride, scale or flag";
    case AGG_ERR_UNSUPPORTED: return "unsupported head dimension (D must be 64)";
    case AGG_ERR_ALIGN: return "tensor pointer is not 16-byte aligned";
    case AGG_ERR_WORKSPACE: return "workspace too small";
    case AGG_ERR_OVERFLOW: return "sequence too long for 32-bit token ids";
    case AGG_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

int agg_sigma_to_strides(int sigma, int32_t* s_h, int32_t* s_w) {
  if (!s_h || !s_w) return AGG_ERR_NULL;
  // Sec. 4.3: sigma = s_h * s_w with the factorisations the paper lists
  static const int table[][3] = {{1, 1, 1}, {2, 1, 2}, {4, 2, 2}, {6, 2, 3}, {9, 3, 3}};
  for (const auto& row : table)
    if (row[0] == sigma) {
      *s_h = row[1];
      *s_w = row[2];
      return AGG_OK;
    }
  return AGG_ERR_SHAPE;
}

int agg_kv_count(const agg_shape* shape, int64_t* M, int64_t* n_dropped) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (M) *M = g.M;
  if (n_dropped) *n_dropped = g.n_dropped;
  return AGG_OK;
}

int agg_kv_indices_host(const agg_shape* shape, int32_t* idx) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!idx) return AGG_ERR_NULL;
  for (int64_t m = 0; m < g.M; ++m) idx[m] = (int32_t)kept_row_to_token(g, m);
  return AGG_OK;
}

int agg_dropped_indices_host(const agg_shape* shape, int32_t* idx) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!idx) return AGG_ERR_NULL;
  for (int64_t u = 0; u < g.n_dropped; ++u) idx[u] = (int32_t)dropped_to_token(g, u);
  return AGG_OK;
}

int agg_kv_compact_bytes(const agg_shape* shape, size_t* bytes, int64_t* M_pad) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (bytes) *bytes = (size_t)g.B * g.H * g.M_pad * kHeadDim * 2;
  if (M_pad) *M_pad = g.M_pad;
  return AGG_OK;
}

int64_t agg_kc_offset(int64_t m, int32_t d) { return kc_offset(m, d); }
int64_t agg_vc_offset(int64_t m, int32_t d) { return vc_offset(m, d); }

size_t agg_workspace_bytes(const agg_shape* shape) {
  Geom g;
  if (make_geom(shape, &g, false) != AGG_OK) return 0;
  // [B][chunks][2 (K,V)][H*D] float partial sums; never zero so that a valid pointer is required
  size_t n = (size_t)g.B * (size_t)mean_chunks(g) * 2 * g.H * kHeadDim * sizeof(float);
  return n ? n : 256;
}

int agg_kv_subsample(const agg_shape* shape, const void* K, const void* V, void* Kc, void* Vc,
                     int32_t* idx, float* kmean, float* vmean, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!K || !V || !kmean || !vmean || !workspace) return AGG_ERR_NULL;
  if ((Kc == nullptr) != (Vc == nullptr)) return AGG_ERR_NULL;  // both or neither
  if (misaligned(K) || misaligned(V) || misaligned(Kc) || misaligned(Vc) || misaligned(workspace) ||
      misaligned(kmean) || misaligned(vmean) || ((uintptr_t)idx & 3u))
    return AGG_ERR_ALIGN;
  if (workspace_bytes < agg_workspace_bytes(shape)) return AGG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (launch_subsample(g, K, V, Kc, Vc, idx, kmean, vmean, workspace, st) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

size_t agg_static_scratch_bytes(void) { return kStaticScratchBytes; }

int agg_kv_subsample_static(const agg_shape* shape, const void* K, const void* V, void* Kc,
                            void* Vc, int32_t* idx, float* kmean, float* vmean, void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!K || !V || !kmean || !vmean) return AGG_ERR_NULL;
  if ((Kc == nullptr) != (Vc == nullptr)) return AGG_ERR_NULL;  // both or neither
  if (misaligned(K) || misaligned(V) || misaligned(Kc) || misaligned(Vc) || misaligned(kmean) ||
      misaligned(vmean) || ((uintptr_t)idx & 3u))
    return AGG_ERR_ALIGN;
  if (agg_workspace_bytes(shape) > kStaticScratchBytes) return AGG_ERR_WORKSPACE;
  void* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return AGG_ERR_LAUNCH;
  hipStream_t st = (hipStream_t)hip_stream;
  if (launch_subsample(g, K, V, Kc, Vc, idx, kmean, vmean, ws, st) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

int agg_global_attn_fwd(const agg_shape* shape, const void* Q, const void* K, const void* V,
                        const void* Kc, const void* Vc, const float* kmean, const float* vmean,
                        void* O, float* lse, void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!Q || !K || !V || !Kc || !Vc || !kmean || !vmean || !O) return AGG_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(Kc) || misaligned(Vc) ||
      misaligned(O) || misaligned(kmean) || misaligned(vmean) || ((uintptr_t)lse & 3u))
    return AGG_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  if (launch_attn(g, shape->flags, shape->scale, shape->mean_logit_bias, Q, K, V, Kc, Vc, kmean,
                  vmean, O, lse, st) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

// Whether the in-place row modes of the attention kernel can address this geometry: indexed
// rows use 32-bit byte offsets from the (batch, head) base formed by a 24-bit multiplication.
static bool rows_addressable(const Geom& g) {
  return (uint64_t)g.NQ * g.H * (kHeadDim * 2) <= 0xFFFFFFFFull && g.NQ <= 0xFFFFFF &&
         (uint64_t)g.H * (kHeadDim * 2) <= 0xFFFFFF;
}

int agg_global_attn_fwd_idx(const agg_shape* shape, const void* Q, const void* K, const void* V,
                            const int32_t* idx, const float* kmean, const float* vmean, void* O,
                            float* lse, void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!Q || !K || !V || !idx || !kmean || !vmean || !O) return AGG_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(kmean) ||
      misaligned(vmean) || ((uintptr_t)idx & 3u) || ((uintptr_t)lse & 3u))
    return AGG_ERR_ALIGN;
  if (!rows_addressable(g)) return AGG_ERR_OVERFLOW;
  if (launch_attn(g, shape->flags, shape->scale, shape->mean_logit_bias, Q, K, V, nullptr, nullptr,
                  kmean, vmean, O, lse, (hipStream_t)hip_stream, nullptr, nullptr, kAttnSrcIndexed,
                  idx, 0) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

int agg_dense_global_attn_fwd(const agg_shape* shape, const void* Q, const void* K, const void* V,
                              void* O, float* lse, void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, true);
  if (rc != AGG_OK) return rc;
  if (!Q || !K || !V || !O) return AGG_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || ((uintptr_t)lse & 3u))
    return AGG_ERR_ALIGN;
  // every token is a key: the kernel reads the rows of K and V where they are, no extras
  if (launch_attn(g, 0u, shape->scale, 0.0f, Q, K, V, nullptr, nullptr, nullptr, nullptr, O, lse,
                  (hipStream_t)hip_stream, nullptr, nullptr, kAttnSrcRows) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

// Frame attention is ordinary attention over B*N independent sequences of one frame each:
// the token-major tensors already hold a frame's L tokens contiguously.
static int frame_shape(const agg_shape* shape, agg_shape* per_frame) {
  if (!shape) return AGG_ERR_NULL;
  if (shape->B < 1 || shape->N < 1) return AGG_ERR_SHAPE;
  if ((int64_t)shape->B * shape->N > INT32_MAX) return AGG_ERR_OVERFLOW;
  *per_frame = *shape;
  per_frame->B = shape->B * shape->N;
  per_frame->N = 1;
  return AGG_OK;
}

int agg_frame_attn_fwd(const agg_shape* shape, const void* Q, const void* K, const void* V, void* O,
                       float* lse, void* hip_stream) {
  agg_shape f;
  int rc = frame_shape(shape, &f);
  if (rc != AGG_OK) return rc;
  return agg_dense_global_attn_fwd(&f, Q, K, V, O, lse, hip_stream);
}

// ---- caller-supplied kept lists ---------------------------------------------------------
// Geometry of the list variants: the grid fields stay (the select kernel needs them), the
// compacted length becomes the list's.
static int list_geom(const agg_shape* shape, int64_t M_list, Geom* g) {
  int rc = make_geom(shape, g, false);
  if (rc != AGG_OK) return rc;
  if (M_list < 1) return AGG_ERR_SHAPE;
  if (M_list > (int64_t)INT32_MAX - 2 * kTileRows) return AGG_ERR_OVERFLOW;
  g->M = M_list;
  g->M_pad = ceil_div(M_list, kTileRows) * kTileRows;
  if ((int64_t)g->B * g->H > ((int64_t)1 << 40) / g->M_pad) return AGG_ERR_OVERFLOW;
  return AGG_OK;
}

int agg_select_kv_indices(const agg_shape* shape, int rule, uint64_t seed, const void* K,
                          int32_t* list, void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (rule < AGG_SELECT_FIRST || rule > AGG_SELECT_LOW) return AGG_ERR_SHAPE;
  const bool needs_k = (rule == AGG_SELECT_HIGH || rule == AGG_SELECT_LOW);
  if (!list || (needs_k && !K)) return AGG_ERR_NULL;
  if ((needs_k && misaligned(K)) || ((uintptr_t)list & 3u)) return AGG_ERR_ALIGN;
  if (launch_select(g, rule, seed, K, list, (hipStream_t)hip_stream) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

int agg_kv_pool(const agg_shape* shape, const void* K, const void* V, void* Kc, void* Vc,
                void* hip_stream) {
  Geom g;
  int rc = make_geom(shape, &g, false);
  if (rc != AGG_OK) return rc;
  if (!K || !V || !Kc || !Vc) return AGG_ERR_NULL;
  if (misaligned(K) || misaligned(V) || misaligned(Kc) || misaligned(Vc)) return AGG_ERR_ALIGN;
  if (launch_pool(g, K, V, Kc, Vc, (hipStream_t)hip_stream) != hipSuccess) return AGG_ERR_LAUNCH;
  return AGG_OK;
}

int agg_list_compact_bytes(const agg_shape* shape, int64_t M_list, size_t* bytes, int64_t* M_pad) {
  Geom g;
  int rc = list_geom(shape, M_list, &g);
  if (rc != AGG_OK) return rc;
  if (bytes) *bytes = (size_t)g.B * g.H * g.M_pad * kHeadDim * 2;
  if (M_pad) *M_pad = g.M_pad;
  return AGG_OK;
}

size_t agg_list_workspace_bytes(const agg_shape* shape) {
  Geom g;
  if (make_geom(shape, &g, false) != AGG_OK) return 0;
  return list_workspace_bytes(g);
}

int agg_kv_subsample_list(const agg_shape* shape, const int32_t* list, int64_t M_list,
                          const void* K, const void* V, void* Kc, void* Vc, float* kmean,
                          float* vmean, uint32_t* kept_bits, int32_t* n_dropped, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = list_geom(shape, M_list, &g);
  if (rc != AGG_OK) return rc;
  if (!list || !K || !V || !Kc || !Vc || !kmean || !vmean || !kept_bits || !n_dropped || !workspace)
    return AGG_ERR_NULL;
  if (misaligned(K) || misaligned(V) || misaligned(Kc) || misaligned(Vc) || misaligned(workspace) ||
      misaligned(kmean) || misaligned(vmean) || ((uintptr_t)list & 3u) ||
      ((uintptr_t)kept_bits & 3u) || ((uintptr_t)n_dropped & 3u))
    return AGG_ERR_ALIGN;
  if (workspace_bytes < list_workspace_bytes(g)) return AGG_ERR_WORKSPACE;
  if (launch_subsample_list(g, list, K, V, Kc, Vc, kmean, vmean, kept_bits, n_dropped, workspace,
                            (hipStream_t)hip_stream) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

int agg_global_attn_fwd_list(const agg_shape* shape, int64_t M_list, const void* Q, const void* K,
                             const void* V, const void* Kc, const void* Vc, const float* kmean,
                             const float* vmean, const uint32_t* kept_bits,
                             const int32_t* n_dropped, void* O, float* lse, void* hip_stream) {
  Geom g;
  int rc = list_geom(shape, M_list, &g);
  if (rc != AGG_OK) return rc;
  if (!Q || !K || !V || !Kc || !Vc || !kmean || !vmean || !kept_bits || !n_dropped || !O)
    return AGG_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(Kc) || misaligned(Vc) ||
      misaligned(O) || misaligned(kmean) || misaligned(vmean) || ((uintptr_t)lse & 3u) ||
      ((uintptr_t)kept_bits & 3u) || ((uintptr_t)n_dropped & 3u))
    return AGG_ERR_ALIGN;
  if (launch_attn(g, shape->flags, shape->scale, shape->mean_logit_bias, Q, K, V, Kc, Vc, kmean,
                  vmean, O, lse, (hipStream_t)hip_stream, kept_bits, n_dropped) != hipSuccess)
    return AGG_ERR_LAUNCH;
  return AGG_OK;
}

// ---- one global-attention block --------------------------------------------------------
namespace {

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Workspace layout of agg_global_block_fwd: LayerNorm output, Q, K, V, attention output,
// then whatever the chosen attention needs.
struct BlockPlan {
  size_t act;      // bytes of one [B, N*L, C] bf16 activation
  size_t attn_ws;  // bytes behind the five activations
  size_t compact;  // SGA: bytes of one compacted tensor
  size_t total;
};

int plan_block(const agg_shape* shape, int mode, BlockPlan* p) {
  Geom g;
  int rc = make_geom(shape, &g, mode != AGG_BLOCK_SGA);
  if (rc != AGG_OK) return rc;
  if (mode != AGG_BLOCK_SGA && mode != AGG_BLOCK_FRAME && mode != AGG_BLOCK_DENSE)
    return AGG_ERR_SHAPE;
  p->act = align256((size_t)g.B * g.NQ * g.H * kHeadDim * 2);
  p->compact = 0;
  if (mode == AGG_BLOCK_SGA) {
    p->compact = align256((size_t)g.B * g.H * g.M_pad * kHeadDim * 2);
    const size_t means = align256((size_t)g.B * g.H * kHeadDim * sizeof(float));
    p->attn_ws = 2 * p->compact + 2 * means + align256(agg_workspace_bytes(shape));
  } else {
    p->attn_ws = 0;  // per-frame and ordinary attention read K and V in place
  }
  p->total = 5 * p->act + p->attn_ws;
  return AGG_OK;
}

}  // namespace

size_t agg_block_workspace_bytes(const agg_shape* shape, int mode) {
  BlockPlan p;
  if (plan_block(shape, mode, &p) != AGG_OK) return 0;
  return p.total;
}

int agg_global_block_fwd(const agg_shape* shape, int mode, const agg_block_weights* w,
                         const void* x, void* y, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  BlockPlan p;
  int rc = plan_block(shape, mode, &p);
  if (rc != AGG_OK) return rc;
  if (!w || !x || !y || !workspace || !w->ln_gamma || !w->ln_beta || !w->w_q || !w->w_k ||
      !w->w_v || !w->w_o)
    return AGG_ERR_NULL;
  if (misaligned(x) || misaligned(y) || misaligned(workspace) || misaligned(w->w_q) ||
      misaligned(w->w_k) || misaligned(w->w_v) || misaligned(w->w_o))
    return AGG_ERR_ALIGN;
  if (x == y) return AGG_ERR_SHAPE;
  if (!(w->ln_eps > 0.0f)) return AGG_ERR_SHAPE;
  if (workspace_bytes < p.total) return AGG_ERR_WORKSPACE;
  const int C = shape->H * kHeadDim;
  if (C > 4096) return AGG_ERR_UNSUPPORTED;  // LayerNorm kernel: a row lives in one wavefront's registers
  const int64_t rows = (int64_t)shape->B * shape->N * ((int64_t)shape->n_h * shape->n_w + shape->n_special);
  hipStream_t st = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  void* xn = base;
  void* Q = base + p.act;
  void* K = base + 2 * p.act;
  void* V = base + 3 * p.act;
  void* A = base + 4 * p.act;  // attention output
  char* aws = base + 5 * p.act;

  if (launch_layernorm(x, w->ln_gamma, w->ln_beta, xn, rows, C, w->ln_eps, st) != hipSuccess)
    return AGG_ERR_LAUNCH;
  const LinearOuts qkv = {{(const uint16_t*)w->w_q, (const uint16_t*)w->w_k, (const uint16_t*)w->w_v},
                          {w->b_q, w->b_k, w->b_v},
                          {(uint16_t*)Q, (uint16_t*)K, (uint16_t*)V},
                          3};
  if (launch_linear(xn, qkv, nullptr, rows, C, C, st) != hipSuccess)
    return AGG_ERR_LAUNCH;
  if (mode == AGG_BLOCK_SGA) {
    const size_t means = align256((size_t)shape->B * shape->H * kHeadDim * sizeof(float));
    void* Kc = aws;
    void* Vc = aws + p.compact;
    float* kmean = (float*)(aws + 2 * p.compact);
    float* vmean = (float*)(aws + 2 * p.compact + means);
    void* mws = aws + 2 * p.compact + 2 * means;
    rc = agg_kv_subsample(shape, K, V, Kc, Vc, nullptr, kmean, vmean, mws,
                          agg_workspace_bytes(shape), hip_stream);
    if (rc != AGG_OK) return rc;
    rc = agg_global_attn_fwd(shape, Q, K, V, Kc, Vc, kmean, vmean, A, nullptr, hip_stream);
  } else if (mode == AGG_BLOCK_FRAME) {
    rc = agg_frame_attn_fwd(shape, Q, K, V, A, nullptr, hip_stream);
  } else {
    rc = agg_dense_global_attn_fwd(shape, Q, K, V, A, nullptr, hip_stream);
  }
  if (rc != AGG_OK) return rc;
  const LinearOuts out = {{(const uint16_t*)w->w_o, nullptr, nullptr},
                          {w->b_o, nullptr, nullptr},
                          {(uint16_t*)y, nullptr, nullptr},
                          1};
  if (launch_linear(A, out, x, rows, C, C, st) != hipSuccess) return AGG_ERR_LAUNCH;
  return AGG_OK;
}

}  // extern "C"

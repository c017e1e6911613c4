/*
 * CPU oracle for subsampled global attention (SGA) -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It shares no code, header, table or constant with the HIP path and
 * must only be used from tests, the smoke check and the benchmark's CPU
 * baseline leg.  Nothing in the product path may call it.
 *
 * What it computes (AVGGT paper, Sec. 4.1 "Notation", Sec. 4.3 "Subsampling
 * Global Attention", caption of the SGA figure):
 *
 *   - N frames, each with n_special special tokens followed by an n_h x n_w
 *     row-major grid of patch tokens; L = n_special + n_h*n_w tokens per frame;
 *     a sequence is the N*L tokens of all frames, frame after frame.
 *   - Every token is a query.  The key/value set S keeps every special token,
 *     every token of frame 0 when keep_first_frame is set (the VGGT rule), and
 *     of every other patch grid only the first (top-left) token of each
 *     s_h x s_w window, windows starting at the grid origin (Sec. 4.3,
 *     "Subsampling Strategy").
 *   - "Diagonal preservation": a query whose own token was dropped from S also
 *     attends to its own key/value.  "Mean component": one extra key/value
 *     pair, the mean over every dropped patch token of the sequence.  The kept
 *     set, the self term and the mean term are normalised by ONE softmax
 *     (Sec. 4.3, "Enhanced Subsampling with Diagonal Preservation").
 *
 * Arithmetic: inputs are bf16 bit patterns; they are widened exactly to double
 * and every sum, product, exponential and division is done in double.  There is
 * no blocking, fusion or reordering: each query row builds its explicit column
 * list and runs a two-pass max-subtracted softmax over it.
 *
 * Layouts (all host memory, contiguous):
 *   Q, K, V : uint16 bf16 bits, [B, N*L, H, D]      (token-major)
 *   Kc, Vc  : uint16 bf16 bits, [B, H, M, D]        (explicit compacted copy)
 *   idx     : int32 [M], ascending token ids of S
 *   kmean, vmean : double [B, H, D]
 *   rows    : int64 [nrows] query token ids to evaluate
 *   O       : double [B, nrows, H, D];  lse : double [B, H, nrows]
 *   P       : optional double [B, H, nrows, M + 2] (kept columns, self, mean;
 *             absent extras hold 0)
 *
 * Pins (tests/test_oracle_pins.py): the sigma table and the window rule as the
 * paper prints them; kept-token counts against the paper's FLOPs tables; the
 * s = 1 path against textbook attention; subset / self / mean logic against a
 * masked dense attention that never builds a compacted copy; the closed form
 * when all dropped tokens are identical; softmax rows summing to one.  The
 * weight given to the mean column (one ordinary column, plus an optional logit
 * bias) is a reading of the text that no printed number discriminates: parity
 * unpinned for that choice alone.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct osga_shape {
  int32_t B, N;
  int32_t n_h, n_w;
  int32_t n_special;
  int32_t H, D;
  int32_t s_h, s_w;
  int32_t keep_first_frame;
  uint32_t flags; /* bit 0: self term, bit 1: mean term */
  float scale;
  float mean_logit_bias;
} osga_shape;

#define OSGA_DIAG 1u
#define OSGA_MEAN 2u

static double bf16_to_double(uint16_t bits) {
  uint32_t w = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

int osga_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Sec. 4.3: the factorisation sigma = s_h * s_w the paper uses. */
int osga_sigma_to_strides(int sigma, int32_t* s_h, int32_t* s_w) {
  switch (sigma) {
    case 1: *s_h = 1; *s_w = 1; return 0; /* no subsampling */
    case 2: *s_h = 1; *s_w = 2; return 0;
    case 4: *s_h = 2; *s_w = 2; return 0;
    case 6: *s_h = 2; *s_w = 3; return 0;
    case 9: *s_h = 3; *s_w = 3; return 0;
    default: return -1;
  }
}

static int64_t tokens_per_frame(const osga_shape* s) {
  return (int64_t)s->n_special + (int64_t)s->n_h * s->n_w;
}

/* 1 if token `tok` (0 <= tok < N*L) belongs to the kept key/value set S. */
int osga_is_kept(const osga_shape* s, int64_t tok) {
  int64_t L = tokens_per_frame(s);
  int64_t frame = tok / L;
  int64_t slot = tok % L;
  if (slot < s->n_special) return 1;              /* special tokens stay */
  if (frame == 0 && s->keep_first_frame) return 1; /* reference view stays whole */
  int64_t patch = slot - s->n_special;
  int64_t row = patch / s->n_w;
  int64_t col = patch % s->n_w;
  /* first token of its s_h x s_w window, windows anchored at (0, 0) */
  return (row % s->s_h == 0) && (col % s->s_w == 0);
}

/* Counts by enumeration of every token (the definition, not a closed form). */
void osga_counts(const osga_shape* s, int64_t* kept, int64_t* dropped) {
  int64_t total = (int64_t)s->N * tokens_per_frame(s);
  int64_t k = 0;
  for (int64_t t = 0; t < total; ++t) k += osga_is_kept(s, t);
  *kept = k;
  *dropped = total - k;
}

/* Ascending token ids of S; idx must hold osga_counts().kept entries. */
void osga_kept_indices(const osga_shape* s, int32_t* idx) {
  int64_t total = (int64_t)s->N * tokens_per_frame(s);
  int64_t m = 0;
  for (int64_t t = 0; t < total; ++t)
    if (osga_is_kept(s, t)) idx[m++] = (int32_t)t;
}

/* Explicit materialisation of the kept rows, head-major. */
void osga_gather(const osga_shape* s, const uint16_t* K, const uint16_t* V, const int32_t* idx,
                 int64_t M, uint16_t* Kc, uint16_t* Vc) {
  int64_t NQ = (int64_t)s->N * tokens_per_frame(s);
  int64_t H = s->H, D = s->D;
  for (int64_t b = 0; b < s->B; ++b)
    for (int64_t h = 0; h < H; ++h)
      for (int64_t m = 0; m < M; ++m) {
        const uint16_t* ksrc = K + ((b * NQ + idx[m]) * H + h) * D;
        const uint16_t* vsrc = V + ((b * NQ + idx[m]) * H + h) * D;
        uint16_t* kdst = Kc + ((b * H + h) * M + m) * D;
        uint16_t* vdst = Vc + ((b * H + h) * M + m) * D;
        for (int64_t d = 0; d < D; ++d) {
          kdst[d] = ksrc[d];
          vdst[d] = vsrc[d];
        }
      }
}

/* Mean key and value over every dropped patch token of a sequence, per batch
 * element and head.  Writes zeros when nothing is dropped. */
void osga_mean(const osga_shape* s, const uint16_t* K, const uint16_t* V, double* kmean,
               double* vmean) {
  int64_t NQ = (int64_t)s->N * tokens_per_frame(s);
  int64_t H = s->H, D = s->D;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t b = 0; b < s->B; ++b)
    for (int64_t h = 0; h < H; ++h) {
      double* km = kmean + (b * H + h) * D;
      double* vm = vmean + (b * H + h) * D;
      for (int64_t d = 0; d < D; ++d) km[d] = vm[d] = 0.0;
      int64_t n = 0;
      for (int64_t t = 0; t < NQ; ++t) {
        if (osga_is_kept(s, t)) continue;
        const uint16_t* kr = K + ((b * NQ + t) * H + h) * D;
        const uint16_t* vr = V + ((b * NQ + t) * H + h) * D;
        for (int64_t d = 0; d < D; ++d) {
          km[d] += bf16_to_double(kr[d]);
          vm[d] += bf16_to_double(vr[d]);
        }
        ++n;
      }
      if (n > 0)
        for (int64_t d = 0; d < D; ++d) {
          km[d] /= (double)n;
          vm[d] /= (double)n;
        }
    }
}

/*
 * SGA for the listed query rows.  For query i the column list is
 *   Kc/Vc rows 0..M-1, then (flag DIAG and i dropped) its own K/V row,
 *   then (flag MEAN and something was dropped) the mean pair,
 * and one softmax runs over that list.
 */
void osga_attn_rows(const osga_shape* s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                    const uint16_t* Kc, const uint16_t* Vc, int64_t M, const double* kmean,
                    const double* vmean, int64_t n_dropped, const int64_t* rows, int64_t nrows,
                    double* O, double* lse, double* P) {
  int64_t NQ = (int64_t)s->N * tokens_per_frame(s);
  int64_t H = s->H, D = s->D;
  int use_mean = (s->flags & OSGA_MEAN) && n_dropped > 0;
  int64_t ncol = M + 2;
  int64_t work = (int64_t)s->B * nrows * H;
#pragma omp parallel
  {
    double* logit = (double*)malloc((size_t)ncol * sizeof(double));
    double* q = (double*)malloc((size_t)D * sizeof(double));
#pragma omp for schedule(dynamic, 1)
    for (int64_t w = 0; w < work; ++w) {
      int64_t b = w / (nrows * H);
      int64_t r = (w / H) % nrows;
      int64_t h = w % H;
      int64_t i = rows[r];
      int use_self = (s->flags & OSGA_DIAG) && !osga_is_kept(s, i);
      const uint16_t* qr = Q + ((b * NQ + i) * H + h) * D;
      for (int64_t d = 0; d < D; ++d) q[d] = bf16_to_double(qr[d]);
      const uint16_t* kc = Kc + (b * H + h) * M * D;
      const uint16_t* vc = Vc + (b * H + h) * M * D;
      const uint16_t* kself = K + ((b * NQ + i) * H + h) * D;
      const uint16_t* vself = V + ((b * NQ + i) * H + h) * D;
      const double* km = kmean + (b * H + h) * D;
      const double* vm = vmean + (b * H + h) * D;

      double mx = -INFINITY;
      for (int64_t m = 0; m < M; ++m) {
        double acc = 0.0;
        for (int64_t d = 0; d < D; ++d) acc += q[d] * bf16_to_double(kc[m * D + d]);
        logit[m] = (double)s->scale * acc;
        if (logit[m] > mx) mx = logit[m];
      }
      logit[M] = -INFINITY;
      if (use_self) {
        double acc = 0.0;
        for (int64_t d = 0; d < D; ++d) acc += q[d] * bf16_to_double(kself[d]);
        logit[M] = (double)s->scale * acc;
        if (logit[M] > mx) mx = logit[M];
      }
      logit[M + 1] = -INFINITY;
      if (use_mean) {
        double acc = 0.0;
        for (int64_t d = 0; d < D; ++d) acc += q[d] * km[d];
        logit[M + 1] = (double)s->scale * acc + (double)s->mean_logit_bias;
        if (logit[M + 1] > mx) mx = logit[M + 1];
      }
      double denom = 0.0;
      for (int64_t c = 0; c < ncol; ++c) {
        logit[c] = (logit[c] == -INFINITY) ? 0.0 : exp(logit[c] - mx);
        denom += logit[c];
      }
      double* o = O + ((b * nrows + r) * H + h) * D;
      for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
      for (int64_t m = 0; m < M; ++m) {
        double p = logit[m] / denom;
        for (int64_t d = 0; d < D; ++d) o[d] += p * bf16_to_double(vc[m * D + d]);
      }
      if (use_self) {
        double p = logit[M] / denom;
        for (int64_t d = 0; d < D; ++d) o[d] += p * bf16_to_double(vself[d]);
      }
      if (use_mean) {
        double p = logit[M + 1] / denom;
        for (int64_t d = 0; d < D; ++d) o[d] += p * vm[d];
      }
      if (lse) lse[(b * H + h) * nrows + r] = mx + log(denom);
      if (P) {
        double* pr = P + ((b * H + h) * nrows + r) * ncol;
        for (int64_t c = 0; c < ncol; ++c) pr[c] = logit[c] / denom;
      }
    }
    free(logit);
    free(q);
  }
}

/* Ordinary global attention for the listed query rows: every token of the
 * sequence is a column (Sec. 4.2: attention over the (B, N*L, C) layout). */
void osga_dense_rows(const osga_shape* s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     const int64_t* rows, int64_t nrows, double* O, double* lse) {
  int64_t NQ = (int64_t)s->N * tokens_per_frame(s);
  int64_t H = s->H, D = s->D;
  int64_t work = (int64_t)s->B * nrows * H;
#pragma omp parallel
  {
    double* logit = (double*)malloc((size_t)NQ * sizeof(double));
    double* q = (double*)malloc((size_t)D * sizeof(double));
#pragma omp for schedule(dynamic, 1)
    for (int64_t w = 0; w < work; ++w) {
      int64_t b = w / (nrows * H);
      int64_t r = (w / H) % nrows;
      int64_t h = w % H;
      int64_t i = rows[r];
      const uint16_t* qr = Q + ((b * NQ + i) * H + h) * D;
      for (int64_t d = 0; d < D; ++d) q[d] = bf16_to_double(qr[d]);
      double mx = -INFINITY;
      for (int64_t j = 0; j < NQ; ++j) {
        const uint16_t* kr = K + ((b * NQ + j) * H + h) * D;
        double acc = 0.0;
        for (int64_t d = 0; d < D; ++d) acc += q[d] * bf16_to_double(kr[d]);
        logit[j] = (double)s->scale * acc;
        if (logit[j] > mx) mx = logit[j];
      }
      double denom = 0.0;
      for (int64_t j = 0; j < NQ; ++j) {
        logit[j] = exp(logit[j] - mx);
        denom += logit[j];
      }
      double* o = O + ((b * nrows + r) * H + h) * D;
      for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
      for (int64_t j = 0; j < NQ; ++j) {
        const uint16_t* vr = V + ((b * NQ + j) * H + h) * D;
        double p = logit[j] / denom;
        for (int64_t d = 0; d < D; ++d) o[d] += p * bf16_to_double(vr[d]);
      }
      if (lse) lse[(b * H + h) * nrows + r] = mx + log(denom);
    }
    free(logit);
    free(q);
  }
}

/* Frame attention (Sec. 4.2, Global-to-Frame conversion): the rearrangement to the
 * (B, N*L, C) layout is skipped, so a query only sees the tokens of its own frame.
 * rows are token ids of the sequence; lse is [B, H, nrows]. */
void osga_frame_rows(const osga_shape* s, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     const int64_t* rows, int64_t nrows, double* O, double* lse) {
  int64_t L = tokens_per_frame(s);
  int64_t NQ = (int64_t)s->N * L;
  int64_t H = s->H, D = s->D;
  int64_t work = (int64_t)s->B * nrows * H;
#pragma omp parallel
  {
    double* logit = (double*)malloc((size_t)L * sizeof(double));
    double* q = (double*)malloc((size_t)D * sizeof(double));
#pragma omp for schedule(dynamic, 1)
    for (int64_t w = 0; w < work; ++w) {
      int64_t b = w / (nrows * H);
      int64_t r = (w / H) % nrows;
      int64_t h = w % H;
      int64_t i = rows[r];
      int64_t first = (i / L) * L; /* first token of the query's frame */
      const uint16_t* qr = Q + ((b * NQ + i) * H + h) * D;
      for (int64_t d = 0; d < D; ++d) q[d] = bf16_to_double(qr[d]);
      double mx = -INFINITY;
      for (int64_t j = 0; j < L; ++j) {
        const uint16_t* kr = K + ((b * NQ + first + j) * H + h) * D;
        double acc = 0.0;
        for (int64_t d = 0; d < D; ++d) acc += q[d] * bf16_to_double(kr[d]);
        logit[j] = (double)s->scale * acc;
        if (logit[j] > mx) mx = logit[j];
      }
      double denom = 0.0;
      for (int64_t j = 0; j < L; ++j) {
        logit[j] = exp(logit[j] - mx);
        denom += logit[j];
      }
      double* o = O + ((b * nrows + r) * H + h) * D;
      for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
      for (int64_t j = 0; j < L; ++j) {
        const uint16_t* vr = V + ((b * NQ + first + j) * H + h) * D;
        double p = logit[j] / denom;
        for (int64_t d = 0; d < D; ++d) o[d] += p * bf16_to_double(vr[d]);
      }
      if (lse) lse[(b * H + h) * nrows + r] = mx + log(denom);
    }
    free(logit);
    free(q);
  }
}

/*
 * ReAttention per-layer hot path -- fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * path computes, written from the paper (Method section: Eq. 1 cache partition,
 * Eq. 2 position-agnostic top-k selection, Eq. 3 concatenation + sequential
 * positional embedding + self-attention; Appendix pseudocode for the prefilling
 * and decoding phases).  It shares no code with the HIP library and must never
 * be reached from the product path; only the test-suite, the smoke check and the
 * benchmark's CPU-baseline leg may call it.
 *
 * All arithmetic is IEEE double.  Inputs arrive as the exact stored bytes of the
 * device tensors (fp32, or bf16 as raw uint16) and are widened exactly.  There
 * is no blocking, fusion or reordering: every loop is the formula as printed.
 * OpenMP only distributes independent outer iterations over host cores.
 *
 * Readings taken where the paper is silent or garbled (each also listed in the
 * design notes of the repository):
 *  - heads of one GQA group are combined by summing their raw dot products;
 *  - selection is token-level; selected entries keep their original order;
 *  - the appendix's concat slices are read as [:l_global], [idx], [-l_local:];
 *  - indices returned are absolute cache positions (middle offset added);
 *  - the query sits at the re-assigned position of its own key;
 *  - stage-1 scores carry no 1/sqrt(D) factor and no rotary encoding;
 *  - rotary pairing is (i, i + D/2) with angular frequency theta^(-2i/D);
 *  - ties: higher score first, then lower index;
 *  - k larger than the middle is clamped; an empty middle means plain attention.
 *
 * Vote selection (paper, "Full-Context Cache Selection", last paragraph; Setup: k = 4,
 * k' = 127, span 32), readings:
 *  - every (query row, query HEAD) casts one vote for each of its own top-k middle
 *    tokens by raw score (no group sum here);
 *  - votes of all heads and all query rows of the chunk are pooled: one set per layer;
 *  - the k' centres are the tokens with the most votes (ties: lower index), zero-vote
 *    tokens are never centres;
 *  - the span of centre c is the m consecutive tokens [c - m/2, c - m/2 + m) clipped to
 *    the middle; the selection is the union of the spans, ascending.
 *
 * Pins (tests/test_oracle_pins.py): brute-force causal RoPE attention when k
 * covers the middle, rotary closed forms / norm / shift invariance, hand-written
 * top-k toys + argsort brute force, softmax mean/convexity, GQA reductions,
 * exact bf16 widening; vote selection: hand-written toys, an independent
 * dictionary-and-sort restatement, reductions to plain top-k and to full attention,
 * needle spans.  Nothing here is "parity unpinned" except the use of the
 * sum aggregation itself, which is a reading (see above), not a computed value.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { RO_F32 = 0, RO_BF16 = 1, RO_F16 = 2 };
enum { RO_AGG_SUM = 0, RO_AGG_MAX = 1 };

typedef struct {
  int32_t n_q_heads;     /* Hq */
  int32_t n_kv_heads;    /* Hkv, divides Hq */
  int32_t head_dim;      /* D, even */
  int32_t dtype;         /* RO_F32 / RO_BF16 / RO_F16: storage of q, K, V */
  int64_t n_ctx;         /* N cached tokens (current tokens already appended) */
  int32_t n_sink;        /* l_global */
  int32_t n_local;       /* l_local */
  int32_t top_k;         /* k */
  int32_t agg;           /* RO_AGG_* */
  double rope_theta;
  double softmax_scale;  /* <= 0 means 1/sqrt(D) */
  int64_t k_stride_head, k_stride_tok; /* in elements */
  int64_t v_stride_head, v_stride_tok;
} ro_shape;

/* ---- exact widening of one stored element ------------------------------- */
/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) from its definition. */
static double ro_half(uint16_t h) {
  const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
  double v;
  if (e == 0) v = ldexp((double)f, -24);                       /* subnormal: f * 2^-10 * 2^-14 */
  else if (e == 31) v = f ? NAN : INFINITY;
  else v = ldexp(1.0 + (double)f / 1024.0, e - 15);
  return sign ? -v : v;
}

static double ro_load(const void* base, int64_t i, int dtype) {
  if (dtype == RO_F32) return (double)((const float*)base)[i];
  if (dtype == RO_F16) return ro_half(((const uint16_t*)base)[i]);
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[i]) << 16; /* bf16 = top half of fp32 */
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

double ro_widen_bf16(uint16_t h) { return ro_load(&h, 0, RO_BF16); }
double ro_widen_f16(uint16_t h) { return ro_load(&h, 0, RO_F16); }

/* ---- Eq. 1: partition ---------------------------------------------------- */
/* sink = [0, s), middle = [s, N - l), local = [N - l, N).  When the cache is
 * shorter than sink + local the middle is empty and the two kept parts are
 * clamped so that together they are exactly the whole cache. */
void ro_partition(int64_t n_ctx, int32_t n_sink, int32_t n_local, int32_t top_k,
                  int64_t* s_eff, int64_t* l_eff, int64_t* n_mid, int64_t* k_eff) {
  int64_t s = n_sink < n_ctx ? n_sink : n_ctx;
  int64_t l = n_local < n_ctx - s ? n_local : n_ctx - s;
  int64_t mid = n_ctx - s - l;
  int64_t k = top_k < mid ? top_k : mid;
  if (k < 0) k = 0;
  *s_eff = s; *l_eff = l; *n_mid = mid; *k_eff = k;
}

/* ---- Eq. 2, first line: position-agnostic scores ------------------------- */
/* scores[i][h][j - s] = agg_g ( sum_c q[i][h*G+g][c] * K[h][j][c] ),  j in middle.
 * q: [n_query][Hq][D] contiguous.  No rotary encoding, no scaling. */
int ro_score(const ro_shape* sh, int32_t n_query, const void* q, const void* k_cache,
             double* scores) {
  int64_t s, l, mid, k;
  ro_partition(sh->n_ctx, sh->n_sink, sh->n_local, sh->top_k, &s, &l, &mid, &k);
  const int Hq = sh->n_q_heads, Hkv = sh->n_kv_heads, D = sh->head_dim, G = Hq / Hkv;
  if (Hq % Hkv) return -1;
  for (int i = 0; i < n_query; ++i)
    for (int h = 0; h < Hkv; ++h) {
      double* row = scores + ((int64_t)i * Hkv + h) * mid;
#pragma omp parallel for schedule(static)
      for (int64_t j = 0; j < mid; ++j) {
        const int64_t koff = (int64_t)h * sh->k_stride_head + (s + j) * sh->k_stride_tok;
        double agg = 0.0;
        for (int g = 0; g < G; ++g) {
          const int64_t qoff = ((int64_t)i * Hq + (int64_t)h * G + g) * D;
          double dot = 0.0;
          for (int c = 0; c < D; ++c)
            dot += ro_load(q, qoff + c, sh->dtype) * ro_load(k_cache, koff + c, sh->dtype);
          if (sh->agg == RO_AGG_MAX) agg = (g == 0 || dot > agg) ? dot : agg;
          else agg += dot;
        }
        row[j] = agg;
      }
    }
  return 0;
}

/* ---- Eq. 2: top-k over one row of middle scores -------------------------- */
typedef struct { double s; int64_t j; } ro_pair;

static int ro_cmp_score_desc(const void* a, const void* b) {
  const ro_pair* x = a; const ro_pair* y = b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->j > y->j) - (x->j < y->j); /* equal score: lower index first */
}
static int ro_cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Sort all candidates by (score desc, index asc), keep the first k, then return
 * them in ascending index order (selected entries keep their relative order).
 * idx receives absolute cache indices (index_base + position in the row).
 * *kth receives the k-th largest score (0 when k == 0). */
int ro_topk_row(const double* row, int64_t n, int64_t k, int64_t index_base,
                int32_t* idx, double* kth) {
  if (k > n) k = n;
  if (kth) *kth = 0.0;
  if (k <= 0) return 0;
  ro_pair* p = (ro_pair*)malloc((size_t)n * sizeof *p);
  if (!p) return -2;
  for (int64_t j = 0; j < n; ++j) { p[j].s = row[j]; p[j].j = j; }
  qsort(p, (size_t)n, sizeof *p, ro_cmp_score_desc);
  for (int64_t r = 0; r < k; ++r) idx[r] = (int32_t)(index_base + p[r].j);
  if (kth) *kth = p[k - 1].s;
  free(p);
  qsort(idx, (size_t)k, sizeof *idx, ro_cmp_i32);
  return 0;
}

/* All rows: scores [n_rows][n_mid] -> idx [n_rows][k_eff], kth [n_rows]. */
int ro_topk(const double* scores, int64_t n_rows, int64_t n_mid, int64_t k_eff,
            int64_t index_base, int32_t* idx, double* kth) {
  int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < n_rows; ++r) {
    int e = ro_topk_row(scores + r * n_mid, n_mid, k_eff, index_base,
                        idx + r * k_eff, kth ? kth + r : 0);
    if (e) {
#pragma omp critical
      rc = e;
    }
  }
  return rc;
}

/* ---- vote selection over heads and query rows ----------------------------- */
/* Per-head scores: scores[i][hq][j - s] = sum_c q[i][hq][c] * K[hq/G][j][c], j in middle. */
int ro_head_scores(const ro_shape* sh, int32_t n_query, const void* q, const void* k_cache,
                   double* scores) {
  int64_t s, l, mid, k;
  ro_partition(sh->n_ctx, sh->n_sink, sh->n_local, sh->top_k, &s, &l, &mid, &k);
  const int Hq = sh->n_q_heads, Hkv = sh->n_kv_heads, D = sh->head_dim, G = Hq / Hkv;
  if (Hq % Hkv) return -1;
  for (int i = 0; i < n_query; ++i)
    for (int hq = 0; hq < Hq; ++hq) {
      double* row = scores + ((int64_t)i * Hq + hq) * mid;
      const int64_t qoff = ((int64_t)i * Hq + hq) * D;
#pragma omp parallel for schedule(static)
      for (int64_t j = 0; j < mid; ++j) {
        const int64_t koff = (int64_t)(hq / G) * sh->k_stride_head + (s + j) * sh->k_stride_tok;
        double dot = 0.0;
        for (int c = 0; c < D; ++c)
          dot += ro_load(q, qoff + c, sh->dtype) * ro_load(k_cache, koff + c, sh->dtype);
        row[j] = dot;
      }
    }
  return 0;
}

typedef struct { int32_t votes; int64_t j; } ro_vote;
static int ro_cmp_votes_desc(const void* a, const void* b) {
  const ro_vote* x = a; const ro_vote* y = b;
  if (x->votes != y->votes) return x->votes > y->votes ? -1 : 1;
  return (x->j > y->j) - (x->j < y->j);  /* equal votes: lower index first */
}

/* head_topk: [n_rows][vote_k] absolute indices (the top-k list of every (query row, head));
 * votes: [n_mid] out (may be NULL); centres: [n_centres] out, ascending, padded with -1;
 * sel: [n_centres * span] out, ascending absolute indices; *n_sel their number. */
int ro_vote_merge(const int32_t* head_topk, int64_t n_rows, int64_t vote_k, int64_t n_mid,
                  int64_t index_base, int64_t n_centres, int64_t span, int32_t* votes,
                  int32_t* centres, int32_t* sel, int64_t* n_sel) {
  *n_sel = 0;
  for (int64_t c = 0; c < n_centres; ++c) centres[c] = -1;
  if (n_mid <= 0 || n_centres <= 0 || span <= 0) return 0;
  ro_vote* v = (ro_vote*)malloc((size_t)n_mid * sizeof *v);
  unsigned char* keep = (unsigned char*)calloc((size_t)n_mid, 1);
  if (!v || !keep) { free(v); free(keep); return -2; }
  for (int64_t j = 0; j < n_mid; ++j) { v[j].votes = 0; v[j].j = j; }
  for (int64_t r = 0; r < n_rows; ++r)                      /* every head and query row votes */
    for (int64_t t = 0; t < vote_k; ++t) {
      const int64_t j = (int64_t)head_topk[r * vote_k + t] - index_base;
      if (j < 0 || j >= n_mid) { free(v); free(keep); return -3; }
      v[j].votes += 1;
    }
  if (votes) for (int64_t j = 0; j < n_mid; ++j) votes[j] = v[j].votes;
  qsort(v, (size_t)n_mid, sizeof *v, ro_cmp_votes_desc);    /* most votes first */
  int64_t nc = 0;
  for (int64_t r = 0; r < n_mid && nc < n_centres && v[r].votes > 0; ++r) {
    const int64_t c = v[r].j;
    centres[nc++] = (int32_t)(index_base + c);
    const int64_t lo = c - span / 2, hi = lo + span;        /* m neighbouring entries as a whole */
    for (int64_t j = lo < 0 ? 0 : lo; j < hi && j < n_mid; ++j) keep[j] = 1;   /* overlaps deduplicated */
  }
  qsort(centres, (size_t)nc, sizeof *centres, ro_cmp_i32);
  int64_t n = 0;
  for (int64_t j = 0; j < n_mid; ++j) if (keep[j]) sel[n++] = (int32_t)(index_base + j);
  *n_sel = n;
  free(v); free(keep);
  return 0;
}

/* ---- Eq. 3: rotary embedding at a re-assigned position ------------------- */
/* Pair (x_i, x_{i+D/2}) turns by angle p * theta^(-2i/D). */
static void ro_rope(const double* x, int D, double pos, double theta, double* y) {
  const int half = D / 2;
  for (int i = 0; i < half; ++i) {
    const double w = pow(theta, -2.0 * (double)i / (double)D);
    const double c = cos(pos * w), sn = sin(pos * w);
    y[i]        = x[i] * c - x[i + half] * sn;
    y[i + half] = x[i + half] * c + x[i] * sn;
  }
}

/* Number of kept entries seen by a query whose own token is q_tok (causal cut
 * inside the local part, or inside the global part when the query is one of the
 * first l_global tokens), and the list itself.  list must hold s+k+l entries. */
static int64_t ro_concat(const ro_shape* sh, int64_t s, int64_t l, int64_t k,
                         const int32_t* idx_row, int64_t q_tok, int64_t* list) {
  int64_t n = 0;
  for (int64_t j = 0; j < s && j <= q_tok; ++j) list[n++] = j;         /* K_global (up to itself for a query inside it:
                                                                          the first prefill chunk holds l_global + l_local tokens) */
  for (int64_t r = 0; r < k; ++r) list[n++] = idx_row[r];              /* K_select, ascending */
  for (int64_t j = sh->n_ctx - l; j <= q_tok && j < sh->n_ctx; ++j)    /* K_local up to itself */
    list[n++] = j;
  return n;
}

/* Materialised form of the concatenation for one query: K rotated at positions
 * pos_offset + r, V copied.  k_sel, v_sel: [Hkv][S][D] doubles where
 * S = s + k_eff + l; rows past the causal cut are left untouched.
 * idx: [Hkv][k_eff] absolute indices for this query.  Returns the kept length. */
int64_t ro_gather_rope(const ro_shape* sh, const void* k_cache, const void* v_cache,
                       const int32_t* idx, int64_t q_tok, double pos_offset,
                       double* k_sel, double* v_sel) {
  int64_t s, l, mid, k;
  ro_partition(sh->n_ctx, sh->n_sink, sh->n_local, sh->top_k, &s, &l, &mid, &k);
  const int Hkv = sh->n_kv_heads, D = sh->head_dim;
  const int64_t S = s + k + l;
  int64_t* list = (int64_t*)malloc((size_t)(S > 0 ? S : 1) * sizeof *list);
  double* tmp = (double*)malloc((size_t)D * sizeof *tmp);
  int64_t n = 0;
  for (int h = 0; h < Hkv; ++h) {
    n = ro_concat(sh, s, l, k, idx + (int64_t)h * k, q_tok, list);
    for (int64_t r = 0; r < n; ++r) {
      const int64_t koff = (int64_t)h * sh->k_stride_head + list[r] * sh->k_stride_tok;
      const int64_t voff = (int64_t)h * sh->v_stride_head + list[r] * sh->v_stride_tok;
      for (int c = 0; c < D; ++c) tmp[c] = ro_load(k_cache, koff + c, sh->dtype);
      ro_rope(tmp, D, pos_offset + (double)r, sh->rope_theta, k_sel + ((int64_t)h * S + r) * D);
      for (int c = 0; c < D; ++c)
        v_sel[((int64_t)h * S + r) * D + c] = ro_load(v_cache, voff + c, sh->dtype);
    }
  }
  free(tmp); free(list);
  return n;
}

/* ---- Eq. 3: attention over [global, select, local] for given index sets --- */
/* q: [n_query][Hq][D]; q_tok[i]: absolute token index of query i (its own key
 * is that cache row; N-1 in decode); idx: [n_query][Hkv][k_eff];
 * out: [n_query][Hq][D] doubles.  pos_offset shifts every assigned position. */
int ro_attend(const ro_shape* sh, int32_t n_query, const void* q, const int64_t* q_tok,
              const void* k_cache, const void* v_cache, const int32_t* idx,
              double pos_offset, double* out) {
  int64_t s, l, mid, k;
  ro_partition(sh->n_ctx, sh->n_sink, sh->n_local, sh->top_k, &s, &l, &mid, &k);
  const int Hq = sh->n_q_heads, Hkv = sh->n_kv_heads, D = sh->head_dim, G = Hq / Hkv;
  if (Hq % Hkv || D % 2) return -1;
  const int64_t S = s + k + l;
  const double scale = sh->softmax_scale > 0.0 ? sh->softmax_scale : 1.0 / sqrt((double)D);
  int rc = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < n_query; ++i)
    for (int hq = 0; hq < Hq; ++hq) {
      const int h = hq / G;
      int64_t* list = (int64_t*)malloc((size_t)(S > 0 ? S : 1) * sizeof *list);
      double* a = (double*)malloc((size_t)(S > 0 ? S : 1) * sizeof *a);
      double* x = (double*)malloc((size_t)D * 4 * sizeof *x);
      if (!list || !a || !x) { rc = -2; free(list); free(a); free(x); continue; }
      double *qv = x, *qr = x + D, *kv = x + 2 * D, *kr = x + 3 * D;
      const int64_t n = ro_concat(sh, s, l, k, idx + ((int64_t)i * Hkv + h) * k, q_tok[i], list);
      /* the query's position is the slot of its own key, the last kept entry */
      for (int c = 0; c < D; ++c) qv[c] = ro_load(q, ((int64_t)i * Hq + hq) * D + c, sh->dtype);
      ro_rope(qv, D, pos_offset + (double)(n - 1), sh->rope_theta, qr);
      double amax = -INFINITY;
      for (int64_t r = 0; r < n; ++r) {
        const int64_t koff = (int64_t)h * sh->k_stride_head + list[r] * sh->k_stride_tok;
        for (int c = 0; c < D; ++c) kv[c] = ro_load(k_cache, koff + c, sh->dtype);
        ro_rope(kv, D, pos_offset + (double)r, sh->rope_theta, kr);
        double dot = 0.0;
        for (int c = 0; c < D; ++c) dot += qr[c] * kr[c];
        a[r] = dot * scale;
        if (a[r] > amax) amax = a[r];
      }
      double z = 0.0;
      for (int64_t r = 0; r < n; ++r) { a[r] = exp(a[r] - amax); z += a[r]; }
      double* o = out + ((int64_t)i * Hq + hq) * D;
      for (int c = 0; c < D; ++c) o[c] = 0.0;
      for (int64_t r = 0; r < n; ++r) {
        const int64_t voff = (int64_t)h * sh->v_stride_head + list[r] * sh->v_stride_tok;
        const double p = a[r] / z;
        for (int c = 0; c < D; ++c) o[c] += p * ro_load(v_cache, voff + c, sh->dtype);
      }
      free(list); free(a); free(x);
    }
  return rc;
}

/* ---- the whole per-layer step, in the paper's order ---------------------- */
/* score -> top-k -> concat -> positional embedding -> self-attention.
 * idx: [n_query][Hkv][k_eff] out; kth: [n_query][Hkv] out (may be NULL);
 * scores_out: [n_query][Hkv][N_mid] out (may be NULL: allocated internally). */
int ro_forward(const ro_shape* sh, int32_t n_query, const void* q, const int64_t* q_tok,
               const void* k_cache, const void* v_cache,
               int32_t* idx, double* kth, double* scores_out, double* out) {
  int64_t s, l, mid, k;
  ro_partition(sh->n_ctx, sh->n_sink, sh->n_local, sh->top_k, &s, &l, &mid, &k);
  const int64_t rows = (int64_t)n_query * sh->n_kv_heads;
  double* sc = scores_out;
  if (!sc) sc = (double*)malloc((size_t)(rows * mid > 0 ? rows * mid : 1) * sizeof *sc);
  if (!sc) return -2;
  int rc = ro_score(sh, n_query, q, k_cache, sc);
  if (!rc) rc = ro_topk(sc, rows, mid, k, s, idx, kth);
  if (!rc) rc = ro_attend(sh, n_query, q, q_tok, k_cache, v_cache, idx, 0.0, out);
  if (!scores_out) free(sc);
  return rc;
}

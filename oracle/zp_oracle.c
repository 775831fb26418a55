/*
 * CPU oracle for the compression step of Compressed PagedAttention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition of what
 * the compression step computes.  It shares no code with the HIP library and
 * the product never calls it; only the tests, the smoke check and the CPU
 * baseline leg of the benchmark do.
 *
 * It follows the paper step by step (Method, "The Compression Process
 * Pipeline"; appendix "Paged Attention Score" with the algorithm "Block
 * Attention Logits Computation"; appendix "KV Cache Compression" with the
 * algorithm of the same name; Method, "Shared Prefix Cache for Compressed
 * PagedAttention"), in fp64 for every floating-point step, with no blocking,
 * fusion or reordering.  bf16 inputs are widened exactly.
 *
 * Memory layout (Background, "Pre-allocated memory"; Method, query cache):
 *   K, V : [L][N_total][b][h_kv][d]
 *   Q    : [L][M][w][h_q][d]
 *
 * Readings taken where the paper is silent, ambiguous or at odds with itself
 * (each is also listed in the design notes of the repository):
 *  R1  The printed causal mask of the logits algorithm hides keys *before* the
 *      query.  A causal mask hides keys *after* it: key position > query
 *      position is masked.  Pinned by the textbook causal-attention case.
 *  R2  The printed mask only touches the last block (it assumes w <= b).  Here
 *      the mask is stated on positions, so it also holds for w > b; for w <= b
 *      it is the printed one (with R1).
 *  R3  Query head hq belongs to kv head hq / G, G = h_q / h_kv (standard GQA).
 *  R4  Order of reductions: softmax over positions, then max over the query
 *      heads of the group, then mean over the w window rows (divisor always w).
 *  R5  Ties in top-k: the lower position wins.  NaN ranks as -inf.
 *  R6  The budget k includes the window (the window gets +inf, then competes).
 *  R7  The top-k tag is called T here; F is the global-score cache only.
 *  R8  With N == N_max nothing is released; block index N_max-1 stays reserved.
 *  R9  The last block is full: T = N * b.
 *  R10 Per-head keep counts k_h (<= budget) and a per-head valid prefix
 *      valid_len (<= (N-1) b).  A head's live sequence is the concatenation
 *      [0, valid_len) ++ [(N-1) b, N b) of logical positions; positions in
 *      between are stale: masked in the softmax, scored -inf, never kept.  The
 *      window is the last w entries of the live sequence and query row u sits
 *      at live index Tv - w + u, Tv = valid_len + b.  With valid_len = (N-1) b
 *      this is the paper's setting.
 *  R11 Target block i (< N_max-1) is a fresh block if source block i is shared
 *      (reference count > 1), otherwise source block i itself.
 *  R12 The reserved block is the first private block at index >= N_max-1.
 *  R13 "Shared" is judged on the reference counts at batch start; decrements
 *      are applied in batch order afterwards; a block is freed when its count
 *      reaches 0.  Freed order: request-major, logical index ascending.
 *  R14 Bytes outside the first k_h rows of the targets are never written.
 *
 * Parity pins (tests/, marker "not gpu"): textbook causal softmax attention
 * for G = 1, single softmax row for w = 1, closed-form cases (orthogonal and
 * identical keys), invariants (row sums, range), block-table permutation
 * invariance, brute-force stable-sort selection, a sequential in-place
 * move without a snapshot for the compaction, and the block counts of the paper's first
 * figure (N_max = 4, b = 4, w = 2).  The paper prints no numeric example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ZO_F32 = 0, ZO_BF16 = 1 };
enum { ZO_OK = 0, ZO_EINVAL = -1, ZO_ENOMEM = -2 };

typedef struct {
    int32_t L, N_total, b, h_kv, h_q, d, M, w, dtype;
} zo_shape;

typedef struct {
    int32_t B, N_max, max_blocks;
    const int32_t *block_table; /* [B][max_blocks] */
    const int32_t *dst_table;   /* [B][N_max-1] or NULL (in place) */
    const int32_t *num_blocks;  /* [B] */
    const int32_t *q_slot;      /* [B] */
    const int32_t *valid_len;   /* [B][L][h_kv] or NULL */
    const int32_t *keep;        /* [B][L][h_kv] or NULL */
} zo_batch;

int zo_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double elem(const void *base, size_t i, int dtype) {
    if (dtype == ZO_F32) return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 -> f32, exact */
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}
static size_t esize(int dtype) { return dtype == ZO_F32 ? 4 : 2; }

/* element offset of row (layer, physical block, slot, head) in K or V */
static size_t kv_row(const zo_shape *s, int l, int blk, int slot, int h) {
    return ((((size_t)l * s->N_total + blk) * s->b + slot) * s->h_kv + h) * (size_t)s->d;
}
static size_t q_row(const zo_shape *s, int l, int slot, int u, int hq) {
    return ((((size_t)l * s->M + slot) * s->w + u) * s->h_q + hq) * (size_t)s->d;
}

static int unit_valid_len(const zo_shape *s, const zo_batch *bt, int n, int l, int h) {
    int N = bt->num_blocks[n];
    if (!bt->valid_len) return (N - 1) * s->b;
    return bt->valid_len[((size_t)n * s->L + l) * s->h_kv + h];
}
static int unit_keep(const zo_shape *s, const zo_batch *bt, int n, int l, int h) {
    if (!bt->keep) return (bt->N_max - 1) * s->b;
    return bt->keep[((size_t)n * s->L + l) * s->h_kv + h];
}

/* live index of logical position t, or -1 if t is stale (reading R10) */
static int live_index(int t, int N, int b, int vl) {
    if (t < vl) return t;
    if (t >= (N - 1) * b) return vl + (t - (N - 1) * b);
    return -1;
}

static int check_batch(const zo_shape *s, const zo_batch *bt) {
    if (s->h_kv <= 0 || s->h_q % s->h_kv) return ZO_EINVAL;
    if (bt->N_max < 2 || s->b <= 0 || s->w <= 0) return ZO_EINVAL;
    for (int n = 0; n < bt->B; n++) {
        int N = bt->num_blocks[n];
        if (N < bt->N_max || N > bt->max_blocks) return ZO_EINVAL;
        if (bt->q_slot && (bt->q_slot[n] < 0 || bt->q_slot[n] >= s->M)) return ZO_EINVAL;
        for (int i = 0; i < N; i++) {
            int p = bt->block_table[(size_t)n * bt->max_blocks + i];
            if (p < 0 || p >= s->N_total) return ZO_EINVAL;
        }
        for (int l = 0; l < s->L; l++)
            for (int h = 0; h < s->h_kv; h++) {
                int vl = unit_valid_len(s, bt, n, l, h);
                if (vl < 0 || vl > (N - 1) * s->b) return ZO_EINVAL;
                if (vl + s->b < s->w) return ZO_EINVAL;
                int k = unit_keep(s, bt, n, l, h);
                int cap = (bt->N_max - 1) * s->b;
                if (vl + s->b < cap) cap = vl + s->b;
                if (k < s->w || k > cap) return ZO_EINVAL;
            }
    }
    return ZO_OK;
}

/*
 * Scores S (Method, compression pipeline; appendix "Paged Attention Score").
 * scores: [B][L][h_kv][max_blocks*b] fp64; entries at stale positions and at
 * positions >= N*b are 0.  No +inf / -inf fill here (that is part of selection).
 */
int zo_score(const zo_shape *s, const zo_batch *bt, const void *K, const void *Q, double *scores) {
    int rc = check_batch(s, bt);
    if (rc) return rc;
    const int G = s->h_q / s->h_kv, b = s->b, w = s->w, d = s->d;
    const size_t Tmax = (size_t)bt->max_blocks * b;
    const long units = (long)bt->B * s->L * s->h_kv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long unit = 0; unit < units; unit++) {
        int h = (int)(unit % s->h_kv), l = (int)((unit / s->h_kv) % s->L);
        int n = (int)(unit / ((long)s->h_kv * s->L));
        int N = bt->num_blocks[n], T = N * b;
        int vl = unit_valid_len(s, bt, n, l, h), Tv = vl + b;
        const int32_t *tbl = bt->block_table + (size_t)n * bt->max_blocks;
        double *S = scores + (size_t)unit * Tmax;
        double *P = (double *)malloc((size_t)G * w * T * sizeof(double));
        if (!P) { failed = 1; continue; }
        const double inv_sqrt_d = 1.0 / sqrt((double)d);
        for (int g = 0; g < G; g++)
            for (int u = 0; u < w; u++) {
                double *a = P + ((size_t)g * w + u) * T;
                size_t qo = q_row(s, l, bt->q_slot[n], u, h * G + g);
                /* logits: scaled dot product of window query u with every key */
                for (int t = 0; t < T; t++) {
                    int j = live_index(t, N, b, vl);
                    if (j < 0 || j > Tv - w + u) { a[t] = -INFINITY; continue; } /* stale, or after the query */
                    size_t ko = kv_row(s, l, tbl[t / b], t % b, h);
                    double acc = 0.0;
                    for (int c = 0; c < d; c++) acc += elem(Q, qo + c, s->dtype) * elem(K, ko + c, s->dtype);
                    a[t] = acc * inv_sqrt_d;
                }
                /* softmax over all T positions */
                double m = -INFINITY, z = 0.0;
                for (int t = 0; t < T; t++) if (a[t] > m) m = a[t];
                for (int t = 0; t < T; t++) z += exp(a[t] - m);
                for (int t = 0; t < T; t++) a[t] = exp(a[t] - m) / z;
            }
        /* max over the group's query heads, then mean over the window rows */
        for (int t = 0; t < T; t++) {
            double acc = 0.0;
            for (int u = 0; u < w; u++) {
                double mx = 0.0; /* probabilities are >= 0 */
                for (int g = 0; g < G; g++) {
                    double p = P[((size_t)g * w + u) * T + t];
                    if (p > mx) mx = p;
                }
                acc += mx;
            }
            S[t] = acc / (double)w;
        }
        for (size_t t = T; t < Tmax; t++) S[t] = 0.0;
        free(P);
    }
    return failed ? ZO_ENOMEM : ZO_OK;
}

/*
 * Score refinements the paper layers on top of the attention score, in its order (appendix "Global Score",
 * "Pooling at the Sequence Dimension", "Redundancy Score of Key states", "Lightning Redundancy", "Combining All
 * These Techniques"):  attention score -> global score (decayed max with the cached history) -> max pooling along
 * the sequence -> S - lambda * R with the lightning (within-block) redundancy R.
 * Readings (also in the design notes):
 *  X1 History exists for the live prefix [0, valid_len) of a request that was compressed before; the last block
 *     holds new tokens without history (the paper's "not the last block" for w <= b, stated on positions).
 *  X2 The cache F holds fp32 values; the value stored is the score after the global update, before pooling and
 *     redundancy (the paper pools "after computing the global score" and applies redundancy "after max pooling").
 *  X3 MaxPool1D: odd kernel m, stride 1, implicit -inf padding (the library default the paper uses), taken along
 *     the live sequence; the paper does not give m, so it is a parameter (1 = off).  The ablation compares pooling at
 *     every compression with pooling at the first one only and recommends the latter: pool_first_only restricts
 *     pooling to the requests of the batch that have no history.
 *  X4 Lightning redundancy: cosine similarity between the live keys of one physical block; diagonal zeroed; in every
 *     column the LAST (highest row, i.e. newest token) entry above the threshold p is zeroed; row sums are divided
 *     by the live sequence length Tv, then a softmax with temperature tau over the live sequence gives R.
 *     A key of zero norm has similarity 0 to everything.  p is a parameter (the paper gives no value).
 */
typedef struct {
    float *F;                  /* [L][N_total][b][h_kv] global-score cache, updated in place; NULL = no global score */
    const int32_t *compressed; /* [B] nonzero: the request was compressed before (history valid); NULL = none was */
    double alpha;              /* decay of the history */
    int32_t pool_kernel;       /* odd >= 1; 1 = no pooling */
    double lambda, tau, p;     /* redundancy weight (0 = off), softmax temperature, similarity threshold */
    int32_t pool_first_only;   /* nonzero: pool only requests without history (the setting the paper recommends) */
} zo_extras;

static size_t f_index(const zo_shape *s, int l, int blk, int slot, int h) {
    return (((size_t)l * s->N_total + blk) * s->b + slot) * s->h_kv + h;
}

/* The refinements applied to scores that are already there (scores: [units][max_blocks*b] fp64, in place). */
int zo_refine(const zo_shape *s, const zo_batch *bt, const void *K, const zo_extras *ex, double *scores) {
    if (!ex) return ZO_OK;
    if (ex->pool_kernel < 1 || !(ex->pool_kernel & 1) || (ex->lambda != 0.0 && !(ex->tau > 0.0))) return ZO_EINVAL;
    const int b = s->b, d = s->d;
    const size_t Tmax = (size_t)bt->max_blocks * b;
    const long units = (long)bt->B * s->L * s->h_kv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long unit = 0; unit < units; unit++) {
        int h = (int)(unit % s->h_kv), l = (int)((unit / s->h_kv) % s->L), n = (int)(unit / ((long)s->h_kv * s->L));
        int N = bt->num_blocks[n], T = N * b, vl = unit_valid_len(s, bt, n, l, h), Tv = vl + b;
        const int32_t *tbl = bt->block_table + (size_t)n * bt->max_blocks;
        double *S = scores + (size_t)unit * Tmax;
        /* live sequence: pos[j] = logical position of live index j */
        int *pos = (int *)malloc((size_t)Tv * sizeof(int));
        double *tmp = (double *)malloc((size_t)Tv * sizeof(double));
        double *Cm = (double *)malloc((size_t)b * b * sizeof(double));
        if (!pos || !tmp || !Cm) { failed = 1; free(pos); free(tmp); free(Cm); continue; }
        for (int t = 0, j = 0; t < T; t++) if (live_index(t, N, b, vl) >= 0) pos[j++] = t;
        /* global score */
        const int has_hist = ex->compressed && ex->compressed[n];
        if (ex->F) {
            for (int j = 0; j < Tv; j++) {
                int t = pos[j];
                size_t fi = f_index(s, l, tbl[t / b], t % b, h);
                double v = S[t];
                if (has_hist && t < vl) {
                    double old = ex->alpha * (double)ex->F[fi];
                    if (old > v) v = old;
                }
                ex->F[fi] = (float)v;
                S[t] = v;
            }
        }
        /* max pooling along the live sequence */
        if (ex->pool_kernel > 1 && !(ex->pool_first_only && has_hist)) {
            int r = ex->pool_kernel / 2;
            for (int j = 0; j < Tv; j++) {
                double m = -INFINITY;
                for (int q = j - r; q <= j + r; q++) if (q >= 0 && q < Tv && S[pos[q]] > m) m = S[pos[q]];
                tmp[j] = m;
            }
            for (int j = 0; j < Tv; j++) S[pos[j]] = tmp[j];
        }
        /* lightning redundancy */
        if (ex->lambda != 0.0) {
            for (int j = 0; j < Tv; j++) tmp[j] = 0.0;   /* row sums per live index */
            for (int i = 0; i < N; i++) {
                /* similarity matrix of block i: rows/cols = slots; stale slots stay zero */
                for (int r = 0; r < b; r++)
                    for (int c = 0; c < b; c++) {
                        double v = 0.0;
                        int tr = i * b + r, tc = i * b + c;
                        if (r != c && live_index(tr, N, b, vl) >= 0 && live_index(tc, N, b, vl) >= 0) {
                            size_t ro = kv_row(s, l, tbl[i], r, h), co = kv_row(s, l, tbl[i], c, h);
                            double dot = 0.0, nr = 0.0, nc = 0.0;
                            for (int e = 0; e < d; e++) {
                                double x = elem(K, ro + e, s->dtype), y = elem(K, co + e, s->dtype);
                                dot += x * y; nr += x * x; nc += y * y;
                            }
                            if (nr > 0.0 && nc > 0.0) v = dot / (sqrt(nr) * sqrt(nc));
                        }
                        Cm[r * b + c] = v;
                    }
                for (int c = 0; c < b; c++)             /* newest similar token is spared: last entry above p in the column */
                    for (int r = b - 1; r >= 0; r--)
                        if (Cm[r * b + c] > ex->p) { Cm[r * b + c] = 0.0; break; }
                for (int r = 0; r < b; r++) {
                    int j = live_index(i * b + r, N, b, vl);
                    if (j < 0) continue;
                    double acc = 0.0;
                    for (int c = 0; c < b; c++) acc += Cm[r * b + c];
                    tmp[j] = acc / (double)Tv;
                }
            }
            double m = -INFINITY, z = 0.0;
            for (int j = 0; j < Tv; j++) if (tmp[j] / ex->tau > m) m = tmp[j] / ex->tau;
            for (int j = 0; j < Tv; j++) z += exp(tmp[j] / ex->tau - m);
            for (int j = 0; j < Tv; j++) S[pos[j]] -= ex->lambda * exp(tmp[j] / ex->tau - m) / z;
        }
        free(pos); free(tmp); free(Cm);
    }
    return failed ? ZO_ENOMEM : ZO_OK;
}

int zo_score_ex(const zo_shape *s, const zo_batch *bt, const void *K, const void *Q, const zo_extras *ex, double *scores) {
    int rc = zo_score(s, bt, K, Q, scores);
    return rc ? rc : zo_refine(s, bt, K, ex, scores);
}

/* The global-score cache moves with the kept entries (appendix "KV Cache Compression", last paragraph): the same
   gather as zo_compact with a row of one fp32 value. */
int zo_compact_global(const zo_shape *s, const zo_batch *bt, float *F, const int32_t *keep_idx, const int32_t *len) {
    const int b = s->b, budget = (bt->N_max - 1) * b;
    const long units = (long)bt->B * s->L * s->h_kv;
    for (long unit = 0; unit < units; unit++) {
        int h = (int)(unit % s->h_kv), l = (int)((unit / s->h_kv) % s->L), n = (int)(unit / ((long)s->h_kv * s->L));
        int k = len[unit];
        if (k < 0 || k > budget) return ZO_EINVAL;
        const int32_t *tbl = bt->block_table + (size_t)n * bt->max_blocks;
        const int32_t *dst = bt->dst_table ? bt->dst_table + (size_t)n * (bt->N_max - 1) : tbl;
        const int32_t *idx = keep_idx + (size_t)unit * budget;
        float *snap = (float *)malloc((size_t)(k ? k : 1) * sizeof(float));
        if (!snap) return ZO_ENOMEM;
        for (int r = 0; r < k; r++) snap[r] = F[f_index(s, l, tbl[idx[r] / b], idx[r] % b, h)];
        for (int r = 0; r < k; r++) F[f_index(s, l, dst[r / b], r % b, h)] = snap[r];
        free(snap);
    }
    return ZO_OK;
}

/* sort record for selection: score descending, then position ascending */
typedef struct { float s; int32_t t; } zo_rec;
static int rec_cmp(const void *pa, const void *pb) {
    const zo_rec *a = (const zo_rec *)pa, *b = (const zo_rec *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->t > b->t) - (a->t < b->t);
}
static int int_cmp(const void *pa, const void *pb) {
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * Selection (Method, compression pipeline: window gets +inf, keep the top k).
 * The decision is taken on fp32 scores (the precision the device kernel scores
 * in).  scores: [B][L][h_kv][T_max] fp32.  keep_idx: [B][L][h_kv][budget],
 * ascending positions, padded with -1.  len_out: [B][L][h_kv] = k_h.
 */
int zo_select(const zo_shape *s, const zo_batch *bt, const float *scores, int32_t T_max,
              int32_t *keep_idx, int32_t *len_out) {
    int rc = check_batch(s, bt);
    if (rc) return rc;
    if (T_max < bt->max_blocks * s->b) return ZO_EINVAL;
    const int b = s->b, w = s->w, budget = (bt->N_max - 1) * b;
    const long units = (long)bt->B * s->L * s->h_kv;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long unit = 0; unit < units; unit++) {
        int h = (int)(unit % s->h_kv), l = (int)((unit / s->h_kv) % s->L);
        int n = (int)(unit / ((long)s->h_kv * s->L));
        int N = bt->num_blocks[n], T = N * b;
        int vl = unit_valid_len(s, bt, n, l, h), Tv = vl + b, k = unit_keep(s, bt, n, l, h);
        const float *S = scores + (size_t)unit * T_max;
        zo_rec *r = (zo_rec *)malloc((size_t)T * sizeof(zo_rec));
        if (!r) { failed = 1; continue; }
        for (int t = 0; t < T; t++) {
            int j = live_index(t, N, b, vl);
            float v = S[t];
            if (v != v) v = -INFINITY;          /* NaN ranks lowest */
            if (j < 0) v = -INFINITY;            /* stale */
            else if (j >= Tv - w) v = INFINITY;  /* observation window */
            r[t].s = v; r[t].t = t;
        }
        qsort(r, (size_t)T, sizeof(zo_rec), rec_cmp); /* total order: no two records compare equal */
        int32_t *out = keep_idx + (size_t)unit * budget;
        for (int i = 0; i < k; i++) out[i] = r[i].t;
        qsort(out, (size_t)k, sizeof(int32_t), int_cmp);
        for (int i = k; i < budget; i++) out[i] = -1;
        len_out[unit] = k;
        free(r);
    }
    return failed ? ZO_ENOMEM : ZO_OK;
}

/*
 * Compaction (appendix "KV Cache Compression"), written as its definition:
 * row r of the targets receives the pre-state row keep_idx[r], for K and V.
 * All source rows of a unit are snapshotted before any row is written.
 */
int zo_compact(const zo_shape *s, const zo_batch *bt, void *K, void *V,
               const int32_t *keep_idx, const int32_t *len) {
    const int b = s->b, budget = (bt->N_max - 1) * b;
    const size_t rowb = (size_t)s->d * esize(s->dtype);
    const long units = (long)bt->B * s->L * s->h_kv;
    for (long unit = 0; unit < units; unit++) {
        int n = (int)(unit / ((long)s->h_kv * s->L));
        int N = bt->num_blocks[n];
        if (N < bt->N_max || N > bt->max_blocks) return ZO_EINVAL;
        int k = len[unit];
        if (k < 0 || k > budget) return ZO_EINVAL;
        const int32_t *idx = keep_idx + (size_t)unit * budget;
        for (int r = 0; r < k; r++)
            if (idx[r] < 0 || idx[r] >= N * b || (r && idx[r] <= idx[r - 1])) return ZO_EINVAL;
    }
    int failed = 0;
    /* units of one request touch disjoint rows (different layer or head) and
       requests in a batch own disjoint target blocks, so units are independent */
#pragma omp parallel for schedule(dynamic, 1)
    for (long unit = 0; unit < units; unit++) {
        int h = (int)(unit % s->h_kv), l = (int)((unit / s->h_kv) % s->L);
        int n = (int)(unit / ((long)s->h_kv * s->L));
        int k = len[unit];
        const int32_t *tbl = bt->block_table + (size_t)n * bt->max_blocks;
        const int32_t *dst = bt->dst_table ? bt->dst_table + (size_t)n * (bt->N_max - 1) : tbl;
        const int32_t *idx = keep_idx + (size_t)unit * budget;
        char *snapK = (char *)malloc((size_t)(k ? k : 1) * rowb), *snapV = (char *)malloc((size_t)(k ? k : 1) * rowb);
        if (!snapK || !snapV) { failed = 1; free(snapK); free(snapV); continue; }
        for (int r = 0; r < k; r++) {
            size_t so = kv_row(s, l, tbl[idx[r] / b], idx[r] % b, h) * esize(s->dtype);
            memcpy(snapK + (size_t)r * rowb, (char *)K + so, rowb);
            memcpy(snapV + (size_t)r * rowb, (char *)V + so, rowb);
        }
        for (int r = 0; r < k; r++) {
            size_t to = kv_row(s, l, dst[r / b], r % b, h) * esize(s->dtype);
            memcpy((char *)K + to, snapK + (size_t)r * rowb, rowb);
            memcpy((char *)V + to, snapV + (size_t)r * rowb, rowb);
        }
        free(snapK); free(snapV);
    }
    return failed ? ZO_ENOMEM : ZO_OK;
}

/*
 * Block bookkeeping (Method, "Compressed PagedAttention" second rule; "Shared
 * Prefix Cache for Compressed PagedAttention"), readings R8, R11-R13.
 * All arrays are host arrays.  refcnt is updated in place on success only.
 * free_in is consumed front to back; n_free_used reports how many were taken.
 */
int zo_plan(int32_t B, int32_t N_max, int32_t max_blocks, int32_t N_total,
            const int32_t *block_table, const int32_t *num_blocks, int32_t *refcnt,
            const int32_t *free_in, int32_t n_free_in, int32_t *n_free_used,
            int32_t *dst_table, int32_t *new_table, int32_t *freed, int32_t *n_freed) {
    if (N_max < 2) return ZO_EINVAL;
    int32_t *cnt = (int32_t *)malloc((size_t)N_total * sizeof(int32_t));
    if (!cnt) return ZO_ENOMEM;
    memcpy(cnt, refcnt, (size_t)N_total * sizeof(int32_t));
    int used = 0, nf = 0, rc = ZO_OK;
    for (int n = 0; n < B && !rc; n++) {
        const int32_t *tbl = block_table + (size_t)n * max_blocks;
        int N = num_blocks[n];
        if (N < N_max || N > max_blocks) { rc = ZO_EINVAL; break; }
        for (int i = 0; i < N; i++)
            if (tbl[i] < 0 || tbl[i] >= N_total || refcnt[tbl[i]] < 1) { rc = ZO_EINVAL; break; }
        if (rc) break;
        /* targets: shared (at batch start) -> fresh block, private -> itself */
        for (int i = 0; i < N_max - 1; i++) {
            if (refcnt[tbl[i]] > 1) {
                if (used >= n_free_in) { rc = ZO_ENOMEM; break; }
                int f = free_in[used++];
                if (f < 0 || f >= N_total || cnt[f] != 0) { rc = ZO_EINVAL; break; }
                cnt[f] = 1;
                dst_table[(size_t)n * (N_max - 1) + i] = f;
            } else {
                dst_table[(size_t)n * (N_max - 1) + i] = tbl[i];
            }
        }
        if (rc) break;
        /* reserved: first private block at index >= N_max-1 */
        int res = -1;
        for (int i = N_max - 1; i < N; i++)
            if (refcnt[tbl[i]] == 1) { res = i; break; }
        if (res < 0) { rc = ZO_EINVAL; break; }
        for (int i = 0; i < N_max - 1; i++) new_table[(size_t)n * N_max + i] = dst_table[(size_t)n * (N_max - 1) + i];
        new_table[(size_t)n * N_max + N_max - 1] = tbl[res];
        /* release */
        for (int i = 0; i < N; i++) {
            int p = tbl[i];
            if (refcnt[p] > 1) {               /* shared at batch start: drop this request's reference */
                if (cnt[p] < 1) { rc = ZO_EINVAL; break; }
                if (--cnt[p] == 0) freed[nf++] = p;
            } else if (i >= N_max - 1 && i != res) {
                cnt[p] = 0;
                freed[nf++] = p;
            }
        }
    }
    if (!rc) {
        memcpy(refcnt, cnt, (size_t)N_total * sizeof(int32_t));
        *n_free_used = used;
        *n_freed = nf;
    }
    free(cnt);
    return rc;
}

/*
 * Check-only paged decode attention over a (compacted) cache: one query per
 * (request, layer, query head), keys/values = the first len[n][l][h] rows of
 * the request's table for kv head h = hq / G.  Textbook softmax(q K^T / sqrt d) V.
 * q: [B][L][h_q][d] (same dtype as the pools); out: [B][L][h_q][d] fp64.
 */
int zo_decode_attention(const zo_shape *s, int32_t B, int32_t table_stride, const int32_t *table,
                        const int32_t *len, const void *K, const void *V, const void *q, double *out) {
    const int G = s->h_q / s->h_kv, b = s->b, d = s->d;
    const long items = (long)B * s->L * s->h_q;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long it = 0; it < items; it++) {
        int hq = (int)(it % s->h_q), l = (int)((it / s->h_q) % s->L), n = (int)(it / ((long)s->h_q * s->L));
        int h = hq / G, len_h = len[((size_t)n * s->L + l) * s->h_kv + h];
        const int32_t *tbl = table + (size_t)n * table_stride;
        double *a = (double *)malloc((size_t)(len_h ? len_h : 1) * sizeof(double));
        if (!a) { failed = 1; continue; }
        size_t qo = (size_t)it * d;
        double m = -INFINITY, z = 0.0;
        for (int t = 0; t < len_h; t++) {
            size_t ko = kv_row(s, l, tbl[t / b], t % b, h);
            double acc = 0.0;
            for (int c = 0; c < d; c++) acc += elem(q, qo + c, s->dtype) * elem(K, ko + c, s->dtype);
            a[t] = acc / sqrt((double)d);
            if (a[t] > m) m = a[t];
        }
        for (int t = 0; t < len_h; t++) { a[t] = exp(a[t] - m); z += a[t]; }
        for (int c = 0; c < d; c++) {
            double acc = 0.0;
            for (int t = 0; t < len_h; t++)
                acc += a[t] / z * elem(V, kv_row(s, l, tbl[t / b], t % b, h) + c, s->dtype);
            out[(size_t)it * d + c] = acc;
        }
        free(a);
    }
    return failed ? ZO_ENOMEM : ZO_OK;
}

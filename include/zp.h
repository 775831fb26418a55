/*
 * zp.h - C ABI of the compression step of Compressed PagedAttention on MI355X (gfx950).
 *
 * For every request whose paged KV cache has reached N_max blocks the step
 *   (1) scores each cached token per (layer, kv head) from the attention of the
 *       last w window queries           (paper: Method, "The Compression Process
 *       Pipeline"; appendix "Paged Attention Score"),
 *   (2) keeps the k_h best tokens per head, the window always among them
 *       (same section: +inf for the observation window, then top-k),
 *   (3) moves the kept K/V rows, order preserved, into the request's first
 *       N_max-1 target blocks            (appendix "KV Cache Compression"),
 *   (4) tells the block manager which blocks are targets, which one stays
 *       reserved for decoding and which are released (Method, "Compressed
 *       PagedAttention"; "Shared Prefix Cache for Compressed PagedAttention").
 *
 * Conventions
 *  - Plain C, no exceptions.  Every call returns a zp_status; zp_last_error()
 *    gives the text for the last failure on that context.
 *  - DEVICE pointers are marked [dev], HOST pointers [host].  The caller owns
 *    every tensor; the library never frees or reallocates them.
 *  - Calls that take a stream are asynchronous on it (stream is a hipStream_t
 *    passed as void*; NULL is the default stream).  No implicit synchronisation.
 *  - Scalar arguments are validated on the host before any launch.  Table
 *    contents live on the device: kernels bounds-check them, skip a unit whose
 *    metadata is inconsistent, write len_out = -1 for it and raise a flag that
 *    zp_sync_status() reports.  zp_validate_batch() checks everything up front.
 *  - The library writes only: rows [0, k_h) of the target blocks, the output
 *    arrays named below, and its own status words.
 *
 * Notation (paper): L layers, N_total physical blocks, block size b, h_kv kv
 * heads, h_q query heads (G = h_q / h_kv, query head hq belongs to kv head
 * hq / G), head dimension d, M query slots, window w, block cap N_max, budget
 * k = (N_max-1) b.  A request holds N >= N_max blocks, all full: T = N b
 * logical positions.  A "unit" is one (request, layer, kv head).
 */
#ifndef ZP_H
#define ZP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zp_ctx zp_ctx;

typedef enum {
    ZP_OK = 0,
    ZP_EINVAL = -1,       /* an argument or a table entry violates the contract */
    ZP_ENOMEM = -2,       /* free list exhausted (zp_plan) or allocation failure */
    ZP_EHIP = -3,         /* a HIP runtime call failed (no device, launch error) */
    ZP_EUNSUPPORTED = -4  /* shape outside what the kernels handle (see zp_score) */
} zp_status;

typedef enum { ZP_F32 = 0, ZP_BF16 = 1 } zp_dtype;

/*
 * Paged memory of one layer slab (Background, "Pre-allocated memory"; Method,
 * query cache).  A slab holds L_slab consecutive layers starting at global
 * layer layer0 (the paper compresses l layers at a time: appendix "Cross-Layer
 * Parallel Compression"); layer0 only offsets the layer index of the per-unit
 * arrays of zp_batch.
 */
typedef struct {
    void *k;        /* [dev] [L_slab][N_total][b][h_kv][d] */
    void *v;        /* [dev] same layout as k */
    const void *q;  /* [dev] [L_slab][M][w][h_q][d]; row u of a slot is the query of the
                       token at live index Tv - w + u (oldest first) */
    int32_t layer0, L_slab;
    int32_t N_total, b, h_kv, h_q, d, M, w;
    int32_t dtype;  /* zp_dtype; scores are always fp32 with fp32 accumulation */
} zp_pool;

/*
 * One compression batch.  L below is the total layer count the per-unit arrays
 * are laid out for (>= layer0 + L_slab).  All arrays are [dev] int32.
 */
typedef struct {
    int32_t B, N_max, max_blocks, L;
    const int32_t *block_table; /* [B][max_blocks] logical -> physical block of the source */
    const int32_t *dst_table;   /* [B][N_max-1] target blocks; NULL = in place (first N_max-1 of
                                   block_table).  dst_table[i] must be block_table[i] or a block
                                   that is in no table of the batch. */
    const int32_t *num_blocks;  /* [B] N, N_max <= N <= max_blocks, last block full */
    const int32_t *q_slot;      /* [B] query slot in [0, M) */
    const int32_t *valid_len;   /* [B][L][h_kv] live prefix length within the first N-1 blocks;
                                   NULL = (N-1) b.  The live sequence of a head is positions
                                   [0, valid_len) followed by the last block; positions between
                                   are stale: never scored, never kept. */
    const int32_t *keep;        /* [B][L][h_kv] k_h, window included:
                                   w <= k_h <= min((N_max-1) b, valid_len + b); NULL = (N_max-1) b */
} zp_batch;

/* Context: owns a few device status words and the last error text.  Needs a GPU. */
zp_status zp_create(zp_ctx **out);
void zp_destroy(zp_ctx *ctx);
const char *zp_last_error(const zp_ctx *ctx); /* ctx may be NULL: text of the last failed zp_create/zp_plan */

/* Device scratch zp_score / zp_compress need beyond inputs and outputs for this shape.  The kernels of this build keep
   everything between their steps on chip, so this is 0; it is non-zero only for the switched-off split kernel (see
   ZP_OPT_SPLIT), whose exchange buffers the context would allocate on first use and keep. */
size_t zp_scratch_bytes(const zp_pool *pool, const zp_batch *batch);

/* Tuning / test switches.  ZP_OPT_SPLIT: -1 automatic (default) and 0 = one workgroup per unit (keys swept twice
   from HBM).  1 = several workgroups per unit with LDS-resident key chunks (keys read from HBM once; needs the scratch
   zp_scratch_bytes reports) is SWITCHED OFF in this build and returns ZP_EUNSUPPORTED: the bounded wait between the
   workgroups of a unit has expired intermittently on MI355X and the cause is not established.
   ZP_OPT_SPIN_LIMIT: bound on that wait loop (iterations, > 0).
   ZP_OPT_STREAMS: cap (1..8) on the ticket streams the split path orders its workgroups by.
   ZP_OPT_XCD_MAP: 1 (default) = every XCD works on a contiguous range of units, so that the kv heads of one
   (request, layer), which read the same blocks, run side by side on one XCD; 0 = workgroup i takes unit i. */
typedef enum { ZP_OPT_SPLIT = 1, ZP_OPT_SPIN_LIMIT = 2, ZP_OPT_STREAMS = 3, ZP_OPT_XCD_MAP = 4 } zp_option;
zp_status zp_set_option(zp_ctx *ctx, int32_t option, int32_t value);

/*
 * Step (1).  scores: [dev] fp32 [B][L_slab][h_kv][T_max], T_max = max_blocks*b.
 * S[t] = (1/w) sum_u max_g softmax_t(q_{g,u} . k_t / sqrt d), causal within the
 * window, stale positions masked.  Entries at stale positions and at t >= N b
 * are written as 0.  No +inf / -inf fill (that belongs to selection).
 * ZP_EUNSUPPORTED: d*elemsize not a multiple of 16 bytes, h_q not a multiple of
 * h_kv, or T_max too large for the on-chip score array (about 30k positions).
 */
zp_status zp_score(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch, float *scores, void *stream);

/*
 * Step (2).  Reads scores ([dev], row stride T_max >= max_blocks*b), gives the
 * window +inf and stale positions -inf (NaN ranks as -inf), keeps the k_h
 * largest with ties going to the lower position.
 * keep_idx: [dev] int32 [B][L_slab][h_kv][(N_max-1) b], kept positions ascending,
 * padded with -1.  len_out: [dev] int32 [B][L_slab][h_kv] = k_h (-1 for a skipped unit).
 */
zp_status zp_select_topk(zp_ctx *ctx, const float *scores, int32_t T_max, const zp_pool *pool,
                         const zp_batch *batch, int32_t *keep_idx, int32_t *len_out, void *stream);

/*
 * Step (3).  For r in [0, len): row r of the targets <- row keep_idx[r] of the
 * source, for K and V, byte exact, safe when targets alias sources (in place).
 * keep_idx rows must be strictly ascending.  Rows that already sit at their
 * destination are not touched.
 */
zp_status zp_compact_kv(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch, const int32_t *keep_idx,
                        const int32_t *len, void *stream);

/*
 * Steps (1)+(2)+(3) fused: one pass per unit, scores never leave the chip.
 * len_out: [dev] int32 [B][L_slab][h_kv].  scores_dbg / keep_idx_dbg: optional
 * [dev] outputs with the layouts of zp_score / zp_select_topk (NULL to skip);
 * they hold bit for bit what the staged calls produce.
 */
zp_status zp_compress(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch, int32_t *len_out,
                      float *scores_dbg, int32_t *keep_idx_dbg, void *stream);

/*
 * zp_compress for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Such callers cannot call zp_create (it allocates the status words the kernels report skipped
 * units through), so this call takes no context: the status words live in a device array that is part of the
 * library image, 256 bytes on every GPU the library runs on, held until the process ends.  The call allocates and
 * frees nothing, on the host or on the device, and enqueues kernels only (one small fill kernel that clears the
 * status words, then the fused kernel).  Its very first call on a device resolves the array's address and loads
 * the kernels: make that call outside any capture.
 * Same arguments, results and shape limits as zp_compress(ctx, pool, batch, len_out, NULL, NULL, stream); the
 * array's size does not grow with the shape, so no shape is refused on its account.  A skipped unit is visible
 * as len_out = -1 (there is no context to ask); the failure text of a refused call is zp_last_error(NULL).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 * race on the status words.  Their K/V results and len_out do not depend on those words.
 */
zp_status zp_compress_static(const zp_pool *pool, const zp_batch *batch, int32_t *len_out, void *stream);

/*
 * Score refinements layered on the attention score, in the paper's order (appendix "Global Score", "Pooling at
 * the Sequence Dimension", "Lightning Redundancy", "Combining All These Techniques"):
 *   global score   S[t] <- max(alpha * F[t], S[t]) on the live prefix [0, valid_len) of a request that was
 *                  compressed before (compressed[n] != 0), then F[t] <- S[t] for every live position;
 *   max pooling    along the live sequence, odd kernel, stride 1, -inf padding (optionally only for requests
 *                  without history);
 *   redundancy     S <- S - lambda * R, R = softmax over the live sequence, temperature tau, of the row sums
 *                  (divided by the live length) of the cosine similarity between the live keys of one physical
 *                  block, diagonal zeroed and, in every column, the last (newest) entry above p zeroed.
 * All fields by value except the two [dev] arrays.  A zeroed struct with pool_kernel = 1 changes nothing.
 */
typedef struct {
    float *F;                  /* [dev] fp32 [L_slab][N_total][b][h_kv] global-score cache of the slab, updated in
                                  place; NULL = no global score */
    const int32_t *compressed; /* [dev] [B] nonzero: the request has history in F; NULL = no request has */
    float alpha;               /* decay of the history */
    int32_t pool_kernel;       /* odd >= 1; 1 = no pooling */
    float lambda, tau, p;      /* redundancy weight (0 = off), temperature (> 0), similarity threshold */
    int32_t pool_first_only;   /* nonzero: pool only requests without history, i.e. at their first compression
                                  (the setting the paper's ablation recommends) */
} zp_extras;

/* zp_score followed by the refinements.  With F set, F is written at every live source position of every unit
   (blocks shared by several requests of the batch receive the value of whichever sharer writes last). */
zp_status zp_score_ex(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch, const zp_extras *extras, float *scores,
                      void *stream);

/* zp_compact_kv that also moves the cached global scores of the kept entries (appendix "KV Cache Compression",
   last paragraph): F[target row r] <- F[source row keep_idx[r]].  F as in zp_extras; NULL = zp_compact_kv.  With
   source blocks shared inside the batch use zp_compress_ex instead: this call reads the values back from F. */
zp_status zp_compact_kv_ex(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch, float *F, const int32_t *keep_idx,
                           const int32_t *len, void *stream);

/* zp_compress with the refinements; with F set the kept entries' global scores travel to the targets inside the
   kernel (on-chip copy, so shared source blocks are safe).  scores_dbg receives the refined scores. */
zp_status zp_compress_ex(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch, const zp_extras *extras,
                         int32_t *len_out, float *scores_dbg, int32_t *keep_idx_dbg, void *stream);

/* Waits for the stream and reports whether any kernel launched through ctx since the
   last call skipped a unit (ZP_EINVAL, with the first offending unit in the error text). */
zp_status zp_sync_status(zp_ctx *ctx, void *stream);

/*
 * Check-only helper, NOT part of the compression path: paged decode attention over a
 * (compacted) cache with per-head lengths, so that a caller can verify that the compacted cache is usable
 * (textbook softmax(q K^T / sqrt d) V; the paper's engine uses its own attention kernels for decoding).
 * pool: k, v and the shape fields are used (q, M, w ignored).  table: [dev] int32 [B][table_stride] logical ->
 * physical block; len: [dev] int32 [B][L_slab][h_kv] rows to attend to (<= table_stride*b);
 * q: [dev] [B][L_slab][h_q][d] in the pool's dtype; out: [dev] fp32 [B][L_slab][h_q][d] (zeros where len = 0).
 * Bad table entries or lengths are reported through zp_sync_status().
 */
zp_status zp_decode_attention(zp_ctx *ctx, const zp_pool *pool, int32_t B, int32_t table_stride, const int32_t *table,
                              const int32_t *len, const void *q, float *out, void *stream);

/* Synchronous, slow, complete check of a batch: copies the tables to the host and
   verifies every rule stated in zp_batch.  ZP_OK or ZP_EINVAL with a message. */
zp_status zp_validate_batch(zp_ctx *ctx, const zp_pool *pool, const zp_batch *batch);

/*
 * Step (4), host only, deterministic (Method, "Compressed PagedAttention" second
 * rule; "Shared Prefix Cache for Compressed PagedAttention").  All arrays [host].
 * A block is shared if its reference count at entry is > 1.  For request n:
 *   target i (< N_max-1) = a fresh block taken from the front of free_in if source block i
 *   is shared, else source block i;  reserved = first private source block at index >= N_max-1;
 *   new_table[n] = targets ++ [reserved];
 *   released: private blocks that are neither target nor reserved, and shared blocks whose
 *   count reaches 0 once every request of the batch has dropped its reference.
 * refcnt [N_total] is updated in place (fresh blocks get 1).  freed (capacity >= sum of
 * num_blocks) lists released blocks request-major, logical index ascending.
 * On any failure nothing is modified.  ZP_ENOMEM: free list too short.
 */
zp_status zp_plan(int32_t B, int32_t N_max, int32_t max_blocks, int32_t N_total, const int32_t *block_table,
                  const int32_t *num_blocks, int32_t *refcnt, const int32_t *free_in, int32_t n_free_in,
                  int32_t *n_free_used, int32_t *dst_table, int32_t *new_table, int32_t *freed, int32_t *n_freed);

#ifdef __cplusplus
}
#endif
#endif /* ZP_H */

// Kernel-side argument block and launch entry points shared by the HIP sources of libzp.
// Paper sections are cited as in include/zp.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zp {

enum : int {
    STAGE_SCORE = 1,    // compute S from K and the window queries
    STAGE_SELECT = 2,   // fill, top-k_h, ascending list
    STAGE_COMPACT = 4,  // move kept K/V rows
    STAGE_LOAD_SCORES = 8,  // S comes from args.scores_in instead of STAGE_SCORE
    STAGE_LOAD_LIST = 16,   // the kept list comes from args.keep_idx_in / len_in
};

// Score refinements switched on for a launch (appendix "Global Score", "Pooling at the Sequence Dimension",
// "Lightning Redundancy") and how compaction carries the global-score cache along.
enum : int {
    EX_GLOBAL = 1,     // decayed max with the cached history, cache updated
    EX_POOL = 2,       // max pooling along the live sequence
    EX_RED = 4,        // S - lambda * R
    EX_MOVE_F = 8,     // compaction moves F rows read back from global memory (staged call)
    EX_POOL_FIRST = 32,  // pooling only for requests without history
    EX_RED_FUSED = 64,   // redundancy: the similarity tiles of the live prefix come from the key tiles of sweep 2 (row sums at off_R)
    EX_MOVE_F_LDS = 16 // compaction writes the kept entries' values from the on-chip copy made by EX_GLOBAL (fused call)
};

// Reasons a kernel skips a unit (reported through the context's status words).
enum : int {
    BAD_NUM_BLOCKS = 1, BAD_VALID_LEN = 2, BAD_KEEP = 3, BAD_SLOT = 4, BAD_BLOCK_ID = 5, BAD_KEEP_IDX = 6, BAD_SYNC = 7,
};

struct Args {
    // paged memory (Background, "Pre-allocated memory"; Method, query cache)
    char *k, *v;
    const char *q;
    int layer0, L_slab, N_total, b, h_kv, h_q, d, M, w, dtype;
    // batch
    int B, N_max, max_blocks, L;
    const int *block_table, *dst_table, *num_blocks, *q_slot, *valid_len, *keep;
    // derived on the host
    int G, T_max, budget, row_bytes, b_shift;   // b_shift >= 0 iff b is a power of two
    float scale_log2;                          // log2(e) / sqrt(d)
    int stages;
    int xcd_map;                               // 1: contiguous unit ranges per XCD (see unit_of_block)
    // staged inputs / outputs (device pointers, any may be null depending on stages)
    const float *scores_in; int scores_in_stride;
    float *scores_out;                         // [units][T_max]
    const int *keep_idx_in; const int *len_in;
    int *keep_idx_out;                         // [units][budget]
    int *len_out;                              // [units]
    int *status;                               // [8]: flag, first bad unit, reason, drain flag of the split path, 4 words of detail
    // refinements
    int ex;                                    // EX_* flags
    float *F;                                  // [L_slab][N_total][b][h_kv] global-score cache
    const int *compressed;                     // [B]
    float alpha, lambda, inv_tau_log2, p_thr;  // inv_tau_log2 = log2(e) / tau
    int pool_r;                                // pooling radius (kernel - 1) / 2
    int off_G;                                 // LDS: [T_max] copy of the global scores for EX_MOVE_F_LDS
    int off_R;                                 // LDS: [T_max] redundancy row sums + 96 words per wave for EX_RED_FUSED
    // byte offsets into dynamic LDS
    int off_S, off_tbl, off_dst, off_misc, off_union, lds_bytes;
    // MFMA path geometry
    int NB;                                    // 32-row query blocks in use
    // split path: C workgroups share one unit, each keeps a chunk of its keys resident in LDS
    int C, NS, RP, spin_limit;                 // workgroups per unit, ticket streams, padded query rows, bound on the wait loop
    int *sync;                                 // [256: one ticket per 128-byte line][units arrive1][units ready1][units arrive2], zeroed before the launch
    float2 *partial;                           // [units][C][RP] per-chunk (max, sum) of every query row
    float *lse_g;                              // [units][RP] combined log-sum-exp
    float *sbuf;                               // [units][T_max] scores, gathered by the workgroup that finishes the unit
    int off_chunk, off_part;                   // LDS offsets of the split phase (alias the tail's regions)
};

// check-only paged decode attention (zp_check.hip)
struct DecodeArgs {
    const char *k, *v, *q;      // pools [L_slab][N_total][b][h_kv][d]; q [B][L_slab][h_q][d]
    float *out;                 // [B][L_slab][h_q][d]
    const int *table, *len;     // [B][table_stride], [B][L_slab][h_kv]
    int *status;
    int B, L_slab, N_total, b, h_kv, h_q, d, dtype, table_stride, row_bytes;
    float scale_log2;
};
hipError_t launch_decode_attention(const DecodeArgs &a, int items, hipStream_t s);

// launchers (host).  Each returns the hipError_t of the launch.
hipError_t launch_unit_generic(const Args &a, int units, hipStream_t s);
// returns hipErrorInvalidConfiguration when no MFMA instantiation covers (d, G, w)
bool mfma_path_available(const Args &a, int *NW, int *RB);
hipError_t launch_unit_mfma(const Args &a, int units, int NW, int RB, hipStream_t s);
// instantiations by head dimension and workgroup width, one translation unit each (zp_mfma_*.hip)
hipError_t launch_mfma_d64(const Args &a, int units, int NW, int RB, hipStream_t s);
hipError_t launch_mfma_d64_wide(const Args &a, int units, int NW, int RB, hipStream_t s);
hipError_t launch_mfma_d128(const Args &a, int units, int NW, int RB, hipStream_t s);
hipError_t launch_mfma_d128_wide(const Args &a, int units, int NW, int RB, hipStream_t s);
constexpr int KT = 64;                          // keys per LDS tile of the matrix-core kernel
size_t mfma_union_bytes(int d, int NW, int NB);
// split path (zp_split.hip)
constexpr int SPLIT_SUBS = 8;                  // 32-key subtiles a workgroup keeps in LDS
hipError_t launch_unit_split(const Args &a, int units, int NW, int RB, hipStream_t s);
hipError_t launch_zero_words(int *p, int n, hipStream_t s);
hipError_t launch_split_d64(const Args &a, int units, int NW, int RB, hipStream_t s);
hipError_t launch_split_d128(const Args &a, int units, int NW, int RB, hipStream_t s);

}  // namespace zp

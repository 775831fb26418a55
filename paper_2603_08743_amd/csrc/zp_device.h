// Device-side building blocks shared by the unit kernels: per-unit metadata checks, the
// order-preserving score key, radix top-k with the lower-position tie-break, and the
// alias-safe row mover.  One workgroup processes one unit = (request, layer, kv head).
#pragma once
#include "zp_kernels.h"

#ifndef ZP_COMPACT_U
#define ZP_COMPACT_U 8
#endif

namespace zp {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

struct Misc {            // small LDS block at Args::off_misc
    int hist[256];
    unsigned scan[16];
    int sel_digit, sel_gt, bad, pad;
};

struct Unit {
    int unit, n, ls, h;  // request, layer inside the slab, kv head
    int N, T;            // blocks held, logical positions N*b
    int vl, Tv;          // live prefix length, live sequence length vl + b
    int k;               // keep count
    int slot;            // query slot
};

__device__ __forceinline__ int div_b(const Args &a, int t) { return a.b_shift >= 0 ? (t >> a.b_shift) : (t / a.b); }

// live index -> logical position: the live sequence is [0, vl) followed by the last block
__device__ __forceinline__ int live_to_pos(const Unit &u, const Args &a, int j) {
    return j < u.vl ? j : j + (u.N - 1) * a.b - u.vl;
}

__device__ __forceinline__ size_t row_off(const Args &a, int ls, int blk, int slot, int h) {
    return ((((size_t)ls * a.N_total + blk) * a.b + slot) * a.h_kv + h) * (size_t)a.row_bytes;
}

__device__ __forceinline__ void report_bad(const Args &a, int unit, int reason) {
    if (a.len_out) a.len_out[unit] = -1;
    if (atomicCAS(&a.status[0], 0, 1) == 0) {
        a.status[1] = unit;
        a.status[2] = reason;
    }
}

// Decode the unit and check its scalar metadata (identical for every thread and every workgroup
// that looks at the unit).  Returns 0 or the reason the unit must be skipped.
__device__ inline int unit_scalars(const Args &a, int unit, Unit &u) {
    u.unit = unit;
    u.h = unit % a.h_kv;
    u.ls = (unit / a.h_kv) % a.L_slab;
    u.n = unit / (a.h_kv * a.L_slab);
    u.N = a.num_blocks[u.n];
    u.T = u.N * a.b;
    u.slot = 0;
    u.k = a.budget;
    u.vl = (u.N - 1) * a.b;
    u.Tv = u.vl + a.b;
    if (u.N < a.N_max || u.N > a.max_blocks) return BAD_NUM_BLOCKS;
    const int idx = (u.n * a.L + a.layer0 + u.ls) * a.h_kv + u.h;
    if (a.valid_len) {
        u.vl = a.valid_len[idx];
        if (u.vl < 0 || u.vl > (u.N - 1) * a.b) return BAD_VALID_LEN;
    }
    u.Tv = u.vl + a.b;
    if (u.Tv < a.w) return BAD_VALID_LEN;
    if (a.stages & STAGE_LOAD_LIST) {
        u.k = a.len_in[unit];
        if (u.k > a.budget) return BAD_KEEP;
    } else {
        if (a.keep) u.k = a.keep[idx];
        const int cap = a.budget < u.Tv ? a.budget : u.Tv;
        if (u.k < a.w || u.k > cap) return BAD_KEEP;
    }
    if (a.stages & STAGE_SCORE) {
        u.slot = a.q_slot[u.n];
        if (u.slot < 0 || u.slot >= a.M) return BAD_SLOT;
    }
    return 0;
}

// Decode the unit, check its metadata, stage both block tables in LDS.
// Returns false (for every thread alike) when the unit must be skipped.
__device__ inline bool unit_setup(const Args &a, int unit, Unit &u, int *tbl, int *dst, Misc *misc) {
    const int tid = threadIdx.x, nt = blockDim.x;
    int bad = unit_scalars(a, unit, u);
    if (tid == 0) misc->bad = bad;
    __syncthreads();
    if (!bad) {
        const int *src = a.block_table + (size_t)u.n * a.max_blocks;
        for (int i = tid; i < u.N; i += nt) {
            int p = src[i];
            if (p < 0 || p >= a.N_total) { misc->bad = BAD_BLOCK_ID; p = 0; }
            tbl[i] = p;
        }
        const int *d = a.dst_table ? a.dst_table + (size_t)u.n * (a.N_max - 1) : src;
        for (int i = tid; i < a.N_max - 1; i += nt) {
            int p = d[i];
            if (p < 0 || p >= a.N_total) { misc->bad = BAD_BLOCK_ID; p = 0; }
            dst[i] = p;
        }
    }
    __syncthreads();
    bad = misc->bad;
    if (bad || u.k < 0) {           // k < 0: a unit an earlier stage already skipped
        if (bad && tid == 0) report_bad(a, unit, bad);
        return false;
    }
    return true;
}

// fp32 score -> unsigned key with the same order; NaN ranks with -inf, -0 equals +0.
__device__ __forceinline__ unsigned score_key(float f) {
    unsigned v = __float_as_uint(f);
    if ((v & 0x7fffffffu) > 0x7f800000u) v = 0xff800000u;
    if (v == 0x80000000u) v = 0u;
    return (v & 0x80000000u) ? ~v : (v | 0x80000000u);
}
#define ZP_KEY_NEG_INF 0x007fffffu
#define ZP_KEY_POS_INF 0xff800000u

__device__ __forceinline__ unsigned wave_incl_scan(unsigned x, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        unsigned y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    return x;
}

// Selection (Method, compression pipeline): window +inf, stale -inf, keep the k largest, ties to the
// lower position.  keys: LDS, holds fp32 scores on entry, destroyed.  list: LDS, receives the k kept
// positions in ascending order.  Exact integer work: radix select on the key, then one packed scan.
__device__ inline void select_unit(const Args &a, const Unit &u, unsigned *keys, int *list, Misc *misc) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wv = tid >> 6;
    const int T = u.T, k = u.k;
    const int stale_lo = u.vl, stale_hi = (u.N - 1) * a.b;       // [vl, (N-1) b) is stale
    const int win_lo_live = u.Tv - a.w;                          // live indices >= this are the window
    for (int t = tid; t < T; t += nt) {
        unsigned key;
        if (t >= stale_lo && t < stale_hi) key = ZP_KEY_NEG_INF;
        else {
            const int j = t < stale_lo ? t : t - stale_hi + u.vl;
            key = j >= win_lo_live ? ZP_KEY_POS_INF : score_key(__uint_as_float(keys[t]));
        }
        keys[t] = key;
    }
    unsigned prefix = 0;
    int remaining = k;
#pragma unroll 1
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = tid; i < 256; i += nt) misc->hist[i] = 0;
        __syncthreads();
        for (int t = tid; t < T; t += nt) {
            const unsigned key = keys[t];
            if (shift == 24 || (key >> (shift + 8)) == prefix) atomicAdd(&misc->hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid < 64) {                                          // digit with: count(above) < remaining <= count(at or above)
            const int c0 = misc->hist[4 * lane], c1 = misc->hist[4 * lane + 1], c2 = misc->hist[4 * lane + 2], c3 = misc->hist[4 * lane + 3];
            const int c = c0 + c1 + c2 + c3;
            int x = c;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                int y = __shfl_down(x, off);
                if (lane + off < 64) x += y;
            }
            int run = x - c;                                     // entries in higher lanes' bins
            if (run < remaining && remaining <= x) {
                int dsel = 4 * lane + 3;
                if (run + c3 < remaining) { run += c3; dsel--;
                    if (run + c2 < remaining) { run += c2; dsel--;
                        if (run + c1 < remaining) { run += c1; dsel--; } } }
                misc->sel_digit = dsel;
                misc->sel_gt = run;
            }
        }
        __syncthreads();
        prefix = (prefix << 8) | (unsigned)misc->sel_digit;
        remaining -= misc->sel_gt;
        __syncthreads();
    }
    // prefix = key of the k-th largest; `remaining` of the entries equal to it are kept, lowest positions first
    const unsigned tau = prefix;
    const int E = (T + nt - 1) / nt;
    const int t0 = tid * E, t1 = (t0 + E < T) ? t0 + E : T;
    unsigned local = 0;                                          // low 16: keys > tau, high 16: keys == tau
    for (int t = t0; t < t1; t++) {
        const unsigned key = keys[t];
        local += (key > tau ? 1u : 0u) + (key == tau ? 0x10000u : 0u);
    }
    const unsigned incl = wave_incl_scan(local, lane);
    if (lane == 63) misc->scan[wv] = incl;
    __syncthreads();
    unsigned base = incl - local;
    for (int i = 0; i < wv; i++) base += misc->scan[i];
    int gt = base & 0xffffu, eq = base >> 16;
    for (int t = t0; t < t1; t++) {
        const unsigned key = keys[t];
        if (key > tau) { list[gt + (eq < remaining ? eq : remaining)] = t; gt++; }
        else if (key == tau) { if (eq < remaining) list[gt + eq] = t; eq++; }
    }
    __syncthreads();
}

// Compaction (appendix "KV Cache Compression"): row r of the targets <- source row list[r], K and V.
// Safe in place: kept positions ascend, so list[r] >= r; ranks are taken in ascending chunks, every
// row of a chunk is in registers (loads complete) before the barrier that precedes the chunk's
// stores, and a later chunk only reads positions at or beyond its own ranks, so its loads may be in
// flight while the previous chunk is being stored (two register sets, loads and stores overlap).
template <int U> struct RowSet {
    u32x4 kk[U], vv[U];
    size_t dof[U];
    bool mv[U];
};

template <int U>
__device__ __forceinline__ void rows_load(const Args &a, const Unit &u, const int *tbl, const int *dst, const int *list, int k,
                                          int r0, int rpp, int rsub, int ch, bool active, RowSet<U> &s) {
#pragma unroll
    for (int i = 0; i < U; i++) {
        const int r = r0 + i * rpp + rsub;
        s.mv[i] = false;
        if (active && r < k) {
            const int t = list[r];
            const int sb = div_b(a, t), db = div_b(a, r);
            const size_t so = row_off(a, u.ls, tbl[sb], t - sb * a.b, u.h) + ch;
            s.dof[i] = row_off(a, u.ls, dst[db], r - db * a.b, u.h) + ch;
            if (so != s.dof[i]) {
                s.mv[i] = true;
                s.kk[i] = *(const u32x4 *)(a.k + so);
                s.vv[i] = *(const u32x4 *)(a.v + so);
            }
        }
    }
}

template <int U>
__device__ __forceinline__ void rows_store(const Args &a, const RowSet<U> &s) {
#pragma unroll
    for (int i = 0; i < U; i++) {
        if (s.mv[i]) {
            *(u32x4 *)(a.k + s.dof[i]) = s.kk[i];
            *(u32x4 *)(a.v + s.dof[i]) = s.vv[i];
        }
    }
}

__device__ inline void compact_unit(const Args &a, const Unit &u, const int *tbl, const int *dst, const int *list, int k) {
    const int tid = threadIdx.x;
    const int cpr = a.row_bytes >> 4;                            // 16-byte pieces per row
    const int rpp = blockDim.x / cpr;                            // rows per pass
    const int rsub = tid / cpr, ch = (tid - rsub * cpr) << 4;
    const bool active = rsub < rpp;
    constexpr int U = ZP_COMPACT_U;
    const int CH = U * rpp;                                      // rows per chunk
    RowSet<U> A, B;
    if (k > 0) rows_load<U>(a, u, tbl, dst, list, k, 0, rpp, rsub, ch, active, A);
#pragma unroll 1
    for (int r0 = 0; r0 < k; r0 += 2 * CH) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (r0 + CH < k) rows_load<U>(a, u, tbl, dst, list, k, r0 + CH, rpp, rsub, ch, active, B);
        rows_store<U>(a, A);
        if (r0 + CH >= k) break;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (r0 + 2 * CH < k) rows_load<U>(a, u, tbl, dst, list, k, r0 + 2 * CH, rpp, rsub, ch, active, A);
        rows_store<U>(a, B);
    }
}

// Everything after S sits in LDS: optional score output, selection, optional list output, compaction.
__device__ inline void unit_tail(const Args &a, const Unit &u, char *smem, const int *tbl, const int *dst, Misc *misc) {
    const int tid = threadIdx.x, nt = blockDim.x;
    float *S = (float *)(smem + a.off_S);
    int *list = (int *)(smem + a.off_union);
    if (a.stages & STAGE_LOAD_SCORES) {
        const float *src = a.scores_in + (size_t)u.unit * a.scores_in_stride;
        for (int t = tid; t < u.T; t += nt) S[t] = src[t];
        __syncthreads();
    }
    if (a.scores_out) {
        float *o = a.scores_out + (size_t)u.unit * a.T_max;
        for (int t = tid; t < a.T_max; t += nt) o[t] = t < u.T ? S[t] : 0.f;
        __syncthreads();
    }
    if (a.stages & STAGE_SELECT) {
        select_unit(a, u, (unsigned *)S, list, misc);
        if (a.keep_idx_out) {
            int *o = a.keep_idx_out + (size_t)u.unit * a.budget;
            for (int r = tid; r < a.budget; r += nt) o[r] = r < u.k ? list[r] : -1;
        }
        if (a.len_out && tid == 0) a.len_out[u.unit] = u.k;
    }
    if (a.stages & STAGE_LOAD_LIST) {
        const int *src = a.keep_idx_in + (size_t)u.unit * a.budget;
        for (int r = tid; r < u.k; r += nt) {
            const int t = src[r];
            const int prev = r ? src[r - 1] : -1;
            if (t <= prev || t >= u.T) misc->bad = BAD_KEEP_IDX;
            list[r] = t;
        }
        __syncthreads();
        if (misc->bad) {
            if (tid == 0) report_bad(a, u.unit, misc->bad);
            return;
        }
    }
    if (a.stages & STAGE_COMPACT) compact_unit(a, u, tbl, dst, list, u.k);
}

}  // namespace zp

// Device-side building blocks shared by the unit kernels: per-unit metadata checks, the
// order-preserving score key, radix top-k with the lower-position tie-break, and the
// alias-safe row mover.  One workgroup processes one unit = (request, layer, kv head).
#pragma once
#include "zp_kernels.h"

#include <type_traits>

#ifndef ZP_COMPACT_U
#define ZP_COMPACT_U 4
#endif

namespace zp {

// A workgroup may use the whole 160 KB of LDS; the runtime wants to be told once per kernel.
template <class K> static hipError_t allow_big_lds(K kernel) {
    static hipError_t state = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return state;
}

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float flog2(float x) { return __builtin_amdgcn_logf(x); }


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

// logical position -> live index, -1 for a stale position
__device__ __forceinline__ int pos_to_live(const Unit &u, const Args &a, int t) {
    const int lb = (u.N - 1) * a.b;
    return t < u.vl ? t : (t >= lb ? t - lb + u.vl : -1);
}

// element index into the global-score cache F [L_slab][N_total][b][h_kv] (host-checked to fit 32 bits)
__device__ __forceinline__ unsigned f_off(const Args &a, int ls, int blk, int slot, int h) {
    return (((unsigned)ls * (unsigned)a.N_total + (unsigned)blk) * (unsigned)a.b + (unsigned)slot) * (unsigned)a.h_kv + (unsigned)h;
}

__device__ __forceinline__ void report_bad(const Args &a, int unit, int reason) {
    if (a.len_out) a.len_out[unit] = -1;
    if (atomicCAS(&a.status[0], 0, 1) == 0) {
        a.status[1] = unit;
        a.status[2] = reason;
    }
}

// Workgroup -> unit.  The hardware deals consecutive workgroups to the 8 XCDs in turn (workgroup i runs on XCD
// i mod 8, each with its own L2 and address-translation cache).  Neighbouring units are the kv heads of one
// (request, layer): they walk the same physical blocks, 256 bytes apart inside every 2 KiB token row.  The map below
// gives every XCD a contiguous range of units, so that those neighbours run side by side on one XCD.
__device__ __forceinline__ int unit_of_block(int bid, int n, int mode) {
    if (mode == 0 || n < 16) return bid;
    const int q = n >> 3, r = n & 7, x = bid & 7, i = bid >> 3;
    return x < r ? x * (q + 1) + i : r * (q + 1) + (x - r) * q + i;
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
// stores, and a later chunk only reads positions at or beyond its own ranks, so its loads may be
// issued while the previous chunk's stores are still on their way.  One register set: what makes this
// phase fast is the number of waves per CU that issue memory operations, not the rows a thread holds
// (a second, alternating set cost registers, i.e. resident waves, and was slower).
// Moved rows are touched once: they are loaded and stored with the non-temporal hint, so that they do not push the
// keys of the first sweep, which the second sweep reads again, out of L2 / Infinity Cache (config 2: 15.2 -> 14.7 ms).
#define ZP_NT_LOAD(p) __builtin_nontemporal_load(p)
#define ZP_NT_STORE(v, p) __builtin_nontemporal_store(v, p)

// A row is addressed by its token index `block * b + slot` inside the unit's (layer, head) plane: one 32-bit multiply-add
// per row (host-checked to fit), then one 64-bit multiply-add to the byte address.  Sixteen lanes share a row, so this
// arithmetic is replicated sixteen times per row: it is kept to a dozen instructions.
template <int U, int FM> struct RowSet {   // FM: 0 K/V only, 1 F read back from global memory, 2 F from the on-chip copy
    u32x4 kk[U], vv[U];
    unsigned dtok[U];
    bool mv[U];
    float fv[FM ? U : 1];
};

struct RowBase {
    size_t byte_base;      // byte offset of (layer, block 0, slot 0, head) plus this lane's 16-byte piece
    unsigned tok_bytes;    // bytes between consecutive tokens
    unsigned f_base, f_tok;  // the same for the global-score cache, in elements
};

// KV_APART: a chunk's K rows are all requested before its V rows (small workgroups), instead of K and V row by row.
// The two pools are separate allocations addressed by the same offsets; which order the memory system prefers depends
// on how many waves issue the requests (measured: the paper's own geometry with two-wave workgroups runs 41.8-43.3 ms per
// launch row by row and 35.2-36.8 ms apart; the 8B-like shape with eight-wave workgroups 14.55 ms against 15.16 ms).
template <int U, int FM, bool POW2, bool KV_APART>
__device__ __forceinline__ void rows_load(const Args &a, const RowBase &rb, const int *tbl, const int *dst, const int *list, const float *Sg, int k,
                                          int r0, int rpp, int rsub, bool lead, bool active, RowSet<U, FM> &s) {
    size_t vo[KV_APART ? U : 1];
#pragma unroll
    for (int i = 0; i < U; i++) {
        const int r = r0 + i * rpp + rsub;
        s.mv[i] = false;
        if (active && r < k) {
            const int t = list[r];
            unsigned st, dt;
            if (POW2) {
                st = ((unsigned)tbl[t >> a.b_shift] << a.b_shift) + (unsigned)(t & (a.b - 1));
                dt = ((unsigned)dst[r >> a.b_shift] << a.b_shift) + (unsigned)(r & (a.b - 1));
            } else {
                const int sb = t / a.b, db = r / a.b;
                st = (unsigned)tbl[sb] * (unsigned)a.b + (unsigned)(t - sb * a.b);
                dt = (unsigned)dst[db] * (unsigned)a.b + (unsigned)(r - db * a.b);
            }
            s.dtok[i] = dt;
            if (st != dt) {
                s.mv[i] = true;
                const size_t so = rb.byte_base + (size_t)st * rb.tok_bytes;
                s.kk[i] = ZP_NT_LOAD((const u32x4 *)(a.k + so));
                if (KV_APART) vo[i] = so;
                else s.vv[i] = ZP_NT_LOAD((const u32x4 *)(a.v + so));
                if (FM && lead) s.fv[i] = FM == 2 ? Sg[t] : a.F[rb.f_base + st * rb.f_tok];   // one lane per row carries the cached global score
            }
        }
    }
    if (KV_APART) {
#pragma unroll
        for (int i = 0; i < U; i++)
            if (s.mv[i]) s.vv[i] = ZP_NT_LOAD((const u32x4 *)(a.v + vo[KV_APART ? i : 0]));
    }
}

template <int U, int FM>
__device__ __forceinline__ void rows_store(const Args &a, const RowBase &rb, bool lead, const RowSet<U, FM> &s) {
#pragma unroll
    for (int i = 0; i < U; i++) {
        if (s.mv[i]) {
            const size_t dof = rb.byte_base + (size_t)s.dtok[i] * rb.tok_bytes;
            ZP_NT_STORE(s.kk[i], (u32x4 *)(a.k + dof));
            ZP_NT_STORE(s.vv[i], (u32x4 *)(a.v + dof));
            if (FM && lead) a.F[rb.f_base + s.dtok[i] * rb.f_tok] = s.fv[i];
        }
    }
}

template <int FM, bool POW2, bool KV_APART>
__device__ __forceinline__ void compact_rows(const Args &a, const Unit &u, const int *tbl, const int *dst, const int *list, const float *Sg, int k) {
    const int tid = threadIdx.x;
    const int cpr = a.row_bytes >> 4;                            // 16-byte pieces per row
    const int rpp = blockDim.x / cpr;                            // rows per pass
    const int rsub = tid / cpr, ch = (tid - rsub * cpr) << 4;
    const bool active = rsub < rpp;
    constexpr int U = ZP_COMPACT_U;
    const int CH = U * rpp;                                      // rows per chunk
    RowBase rb;
    rb.tok_bytes = (unsigned)a.h_kv * (unsigned)a.row_bytes;
    rb.byte_base = ((size_t)u.ls * a.N_total * a.b * a.h_kv + u.h) * (size_t)a.row_bytes + ch;
    rb.f_tok = (unsigned)a.h_kv;
    rb.f_base = (unsigned)u.ls * (unsigned)a.N_total * (unsigned)a.b * (unsigned)a.h_kv + (unsigned)u.h;
    RowSet<U, FM> A;
#pragma unroll 1
    for (int r0 = 0; r0 < k; r0 += CH) {
        rows_load<U, FM, POW2, KV_APART>(a, rb, tbl, dst, list, Sg, k, r0, rpp, rsub, ch == 0, active, A);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        rows_store<U, FM>(a, rb, ch == 0, A);
    }
}

template <int FM>
__device__ inline void compact_unit(const Args &a, const Unit &u, const int *tbl, const int *dst, const int *list, const float *Sg, int k) {
    if (a.b_shift < 0) compact_rows<FM, false, false>(a, u, tbl, dst, list, Sg, k);
    else if (blockDim.x <= 128) compact_rows<FM, true, true>(a, u, tbl, dst, list, Sg, k);
    else compact_rows<FM, true, false>(a, u, tbl, dst, list, Sg, k);
}

// ------------------------------------------------------------------ score refinements
//
// Applied to S (LDS, indexed by logical position) right after scoring, in the paper's order (appendix
// "Combining All These Techniques"): global score -> max pooling -> S - lambda * R.

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// workgroup-wide max and sum of per-thread values, same result in every thread, fixed order
__device__ inline float block_reduce(float v, bool is_max, Misc *misc) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, nw = blockDim.x >> 6;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float o = __shfl_xor(v, off);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    float *sc = (float *)misc->scan;
    __syncthreads();
    if (lane == 0) sc[wv] = v;
    __syncthreads();
    v = sc[0];
    for (int i = 1; i < nw; i++) v = is_max ? fmaxf(v, sc[i]) : v + sc[i];
    return v;
}

// Lightning redundancy, any element type and block size (appendix "Lightning Redundancy"): one thread per
// live key computes its row of the within-block cosine-similarity matrix on the vector ALUs.  The matrix is
// symmetric, so the row of key r is also column r: the thread finds the last entry above p of its column
// there and publishes (row, value); row sums are corrected after a barrier.  rs[j] receives the row sum / Tv.
template <int DT>
__device__ inline void redundancy_valu(const Args &a, const Unit &u, const int *tbl, float *rs, float *inv, int *zl, float *zv) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const int n_el = a.d;
    for (int j = tid; j < u.Tv; j += nt) {
        const int t = live_to_pos(u, a, j), blk = div_b(a, t);
        const char *kr = a.k + row_off(a, u.ls, tbl[blk], t - blk * a.b, u.h);
        float n2 = 0.f;
        for (int e = 0; e < n_el; e++) {
            const float x = DT ? __uint_as_float((unsigned)((const unsigned short *)kr)[e] << 16) : ((const float *)kr)[e];
            n2 = fmaf(x, x, n2);
        }
        inv[j] = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
    }
    __syncthreads();
    for (int j = tid; j < u.Tv; j += nt) {
        const int t = live_to_pos(u, a, j), blk = div_b(a, t), r = t - blk * a.b;
        const char *kb = a.k + row_off(a, u.ls, tbl[blk], 0, u.h);
        const size_t slot_bytes = (size_t)a.h_kv * a.row_bytes;
        const char *kr = kb + r * slot_bytes;
        const float ir = inv[j];
        float acc = 0.f, lastv = 0.f;
        int last = -1;
        for (int c = 0; c < a.b; c++) {
            const int jc = pos_to_live(u, a, blk * a.b + c);
            float val = 0.f;
            if (c != r && jc >= 0) {
                const float ic = inv[jc];
                if (ir != 0.f && ic != 0.f) {
                    const char *kc = kb + c * slot_bytes;
                    float dot = 0.f;
                    for (int e = 0; e < n_el; e++) {
                        const float x = DT ? __uint_as_float((unsigned)((const unsigned short *)kr)[e] << 16) : ((const float *)kr)[e];
                        const float y = DT ? __uint_as_float((unsigned)((const unsigned short *)kc)[e] << 16) : ((const float *)kc)[e];
                        dot = fmaf(x, y, dot);
                    }
                    val = dot * (ir * ic);
                }
            }
            acc += val;
            if (val > a.p_thr) { last = c; lastv = val; }
        }
        rs[j] = acc;
        zl[j] = last;
        zv[j] = lastv;
    }
    __syncthreads();
    const float inv_len = 1.0f / (float)u.Tv;
    for (int j = tid; j < u.Tv; j += nt) {
        const int t = live_to_pos(u, a, j), blk = div_b(a, t), r = t - blk * a.b;
        float corr = 0.f;
        for (int c = 0; c < a.b; c++) {
            const int jc = pos_to_live(u, a, blk * a.b + c);
            if (jc >= 0 && zl[jc] == r) corr += zv[jc];
        }
        rs[j] = (rs[j] - corr) * inv_len;
    }
    __syncthreads();
}

// The same for bf16 keys with a block size that divides 32: K_g K_g^T of 32 consecutive logical positions
// (32/b whole blocks) is one 32x32 tile of the matrix cores, both operands being the same register fragments.
// Lane L, register i holds the entry (row 8*(i/4) + 4*(L/32) + i%4, column L%32); only entries whose row and
// column lie in the same block are used.  A wave owns a group; its 96 words of LDS hold the inverse norms and
// the (row, value) of the entry zeroed in every column.
// last_only: only the rows of the last block are produced (the live prefix was done from the key tiles of sweep 2).
template <int D>
__device__ inline void redundancy_mfma(const Args &a, const Unit &u, const int *tbl, float *rs, float *wave_scratch, bool last_only) {
    constexpr int KK = D / 16;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, nw = blockDim.x >> 6, l32 = lane & 31, hf = lane >> 5;
    float *inv = wave_scratch + wv * 96, *zv = inv + 64;
    int *zr = (int *)(inv + 32);
    const int ngroups = (u.T + 31) >> 5;
    const int stale_hi = (u.N - 1) * a.b;
    const float inv_len = 1.0f / (float)u.Tv;
    const int cblk = l32 >> a.b_shift;                              // block of this lane's column inside the group
    const int dgi = ((l32 >> 3) << 2) | (l32 & 3);              // register that holds the diagonal entry ...
    const bool dg_mine = hf == ((l32 >> 2) & 1);                // ... in this half of the wave
    // groups of this wave in ascending order, wholly stale ones skipped; the fragments of the next group are
    // requested before the current one is worked on
    auto next_group = [&](int g) {
        while (g < ngroups && g * 32 + 32 <= stale_hi && (last_only || g * 32 >= u.vl)) g += nw;
        return g;
    };
    auto live_of = [&](int g) {
        const int p = g * 32 + l32;
        if (p >= u.T || (last_only && p < stale_hi)) return -1;
        return pos_to_live(u, a, p);
    };
    auto load_group = [&](int g, bf16x8 (&kf)[KK]) {
        const int pc = live_of(g) >= 0 ? g * 32 + l32 : u.T - 1;  // rows that are not live read a valid row and are masked
        const int blk = div_b(a, pc);
        const char *kp = a.k + row_off(a, u.ls, tbl[blk], pc - blk * a.b, u.h) + hf * 16;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) kf[kk] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(kp + kk * 32));
    };
    bf16x8 kf[KK], kn[KK];
    int g = next_group(wv);
    if (g < ngroups) load_group(g, kf);
#pragma unroll 1
    while (g < ngroups) {
        const int gn = next_group(g + nw);
        if (gn < ngroups) load_group(gn, kn);
        const int jl = live_of(g);
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; i++) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], kf[kk], acc, 0, 0, 0);
        float dg = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i++) dg = i == dgi ? acc[i] : dg;
        if (dg_mine) inv[l32] = (jl >= 0 && dg > 0.f) ? 1.0f / sqrtf(dg) : 0.f;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // LDS serves a wave's accesses in order
        const float ic = inv[l32];
        float csum = 0.f, lastv = 0.f;
        int last = -1;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int row = 8 * (i >> 2) + 4 * hf + (i & 3);
            const float ir = inv[row];
            const bool in_blk = (row >> a.b_shift) == cblk;
            float val = 0.f;
            if (in_blk && row != l32 && ir != 0.f && ic != 0.f) val = acc[i] * (ir * ic);
            csum += val;
            if (in_blk && val > a.p_thr) { last = row; lastv = val; }   // rows ascend with i
        }
        const int o_last = __shfl_xor(last, 32);
        const float o_lastv = __shfl_xor(lastv, 32), o_csum = __shfl_xor(csum, 32);
        const float colsum = hf ? o_csum + csum : csum + o_csum;  // same bits in both halves
        if (hf == 0) {
            zr[l32] = last > o_last ? last : o_last;
            zv[l32] = last > o_last ? lastv : o_lastv;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // symmetric matrix: the sum of row r before zeroing is the sum of column r; take off what was zeroed in row r
        if (hf == 0 && jl >= 0) {
            float corr = 0.f;
            const int c0 = cblk * a.b;
            for (int c = c0; c < c0 + a.b; c++)
                if (zr[c] == l32) corr += zv[c];
            rs[jl] = (colsum - corr) * inv_len;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the next group reuses the wave's scratch
#pragma unroll
        for (int kk = 0; kk < KK; kk++) kf[kk] = kn[kk];
        g = gn;
    }
    __syncthreads();
}

// Block size 16, live prefix: the similarity matrix of one block from the key tile that sweep 2 holds in LDS anyway
// (rows `rows`, ROWB bytes apart, 16 keys of one block).  K_blk K_blk^T is one 16x16 tile of the matrix cores
// (v_mfma_f32_16x16x32_bf16, both operands the same fragments: lane L supplies key L%16, elements 8*(L/16).. of every
// 32-wide step; register i of lane L holds entry (row 4*(L/16) + i, column L%16)).  j_first: live index of the
// block's first key; rows at or beyond the live prefix are not live.  Everything after the products stays in
// registers: norms and the column rule travel by lane permutes, the row sums by adds across the 16 lanes of a row group
// (this step sits inside the tile loop of sweep 2, where every wait on LDS holds up the whole workgroup's barrier).
// It comes in two parts so that the caller can take the products while the key rows are in LDS and finish later.
typedef __attribute__((ext_vector_type(4))) float f32x4;

// sum over the 16 lanes that share lane/16, the same bits in all of them (a + b and b + a at every step)
__device__ __forceinline__ float row16_sum(float v) {
    auto dpp = [](float x, auto ctrl) { return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, true)); };
    v += dpp(v, std::integral_constant<int, 0xB1>());      // lane ^ 1 inside every quad
    v += dpp(v, std::integral_constant<int, 0x4E>());      // lane ^ 2
    v += dpp(v, std::integral_constant<int, 0x141>());     // mirror inside every half row: the other quad's sum
    v += dpp(v, std::integral_constant<int, 0x140>());     // mirror inside the row: the other half's sum
    return v;
}

// the products: needs the key rows in LDS only here
template <int D, int ROWB>
__device__ __forceinline__ f32x4 block_gram(const char *rows, int lane) {
    const int c = lane & 15, g = lane >> 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const char *kp = rows + c * ROWB + g * 16;
#pragma unroll
    for (int kk = 0; kk < D / 32; kk++) {
        const bf16x8 f = *(const bf16x8 *)(kp + kk * 64);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f, f, acc, 0, 0, 0);
    }
    return acc;
}

// from the products to the row sums of the block's live keys: rs[j] = (row sum with the column rule applied) / Tv
__device__ __forceinline__ void block_row_sums(const Args &a, const Unit &u, const f32x4 acc, int j_first, float inv_len, float *rs, int lane) {
    const int c = lane & 15, g = lane >> 4;
    // inverse norm of key c from the diagonal entry (c, c), which sits in lane (column c, group c/4), register c%4
    float dg = acc[0];
#pragma unroll
    for (int i = 1; i < 4; i++) dg = i == (c & 3) ? acc[i] : dg;
    const float own = (j_first + c < u.vl && dg > 0.f) ? 1.0f / sqrtf(dg) : 0.f;    // meaningful in the diagonal lanes only
    const float ic = __shfl(own, (c >> 2) * 16 + c);
    float val[4];
    int last = -1;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int row = 4 * g + i;
        const float ir = __shfl(ic, g * 16 + row);              // the lane of column `row` in this group holds its inverse norm
        float v = 0.f;
        if (row != c && ir != 0.f && ic != 0.f) v = acc[i] * (ir * ic);
        val[i] = v;
        if (v > a.p_thr) last = row;                            // rows ascend with i
    }
    // the four lanes of a column (rows 0-3, 4-7, 8-11, 12-15) agree on the last entry above p ...
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const int ol = __shfl_xor(last, off);
        last = ol > last ? ol : last;
    }
    // ... it is zeroed where it lives, and every row is summed over the 16 columns
    float mine = 0.f;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const float s = row16_sum(4 * g + i == last ? 0.f : val[i]);
        mine = i == c ? s : mine;
    }
    if (c < 4 && j_first + 4 * g + c < u.vl) rs[j_first + 4 * g + c] = mine * inv_len;
}

// D > 0: called from the matrix-core kernel for head dimension D (bf16); D = 0: generic kernel, element type DT.
template <int D, int DT>
__device__ inline void refine_unit(const Args &a, const Unit &u, char *smem, const int *tbl, Misc *misc) {
    const int tid = threadIdx.x, nt = blockDim.x;
    float *S = (float *)(smem + a.off_S);
    float *tmp = (float *)(smem + a.off_union);
    const bool hist = a.compressed && a.compressed[u.n] != 0;
    if (a.ex & EX_GLOBAL) {
        float *Sg = (float *)(smem + a.off_G);
        for (int j = tid; j < u.Tv; j += nt) {
            const int t = live_to_pos(u, a, j), blk = div_b(a, t);
            const unsigned fi = f_off(a, u.ls, tbl[blk], t - blk * a.b, u.h);
            float v = S[t];
            if (hist && t < u.vl) {                              // the last block holds new tokens: no history
                const float old = a.alpha * a.F[fi];
                if (old > v) v = old;
            }
            a.F[fi] = v;
            S[t] = v;
            if (a.ex & EX_MOVE_F_LDS) Sg[t] = v;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // compaction may write the same cache entries later
        __syncthreads();
    }
    if ((a.ex & EX_POOL) && !((a.ex & EX_POOL_FIRST) && hist)) {
        const int r = a.pool_r;
        for (int j = tid; j < u.Tv; j += nt) {
            const int lo = j - r < 0 ? 0 : j - r, hi = j + r > u.Tv - 1 ? u.Tv - 1 : j + r;
            float m = -INFINITY;
            for (int q = lo; q <= hi; q++) {
                const float x = S[live_to_pos(u, a, q)];
                if (x > m) m = x;
            }
            tmp[j] = m;
        }
        __syncthreads();
        for (int j = tid; j < u.Tv; j += nt) S[live_to_pos(u, a, j)] = tmp[j];
        __syncthreads();
    }
    if (a.ex & EX_RED) {
        const bool mf = D > 0 && 32 % a.b == 0;
        if (a.ex & EX_RED_FUSED) {                               // the live prefix was done from the key tiles of sweep 2
            tmp = (float *)(smem + a.off_R);
            if constexpr (D > 0) redundancy_mfma<D>(a, u, tbl, tmp, tmp + a.T_max, true);
        } else if (mf) {
            if constexpr (D > 0) redundancy_mfma<D>(a, u, tbl, tmp, tmp + a.T_max, false);
        } else {
            redundancy_valu<DT>(a, u, tbl, tmp, tmp + a.T_max, (int *)(tmp + 2 * (size_t)a.T_max), tmp + 3 * (size_t)a.T_max);
        }
        // R = softmax over the live sequence of (row sum / Tv) / tau, in base 2
        float m = -INFINITY;
        for (int j = tid; j < u.Tv; j += nt) m = fmaxf(m, tmp[j] * a.inv_tau_log2);
        m = block_reduce(m, true, misc);
        float z = 0.f;
        for (int j = tid; j < u.Tv; j += nt) {
            const float e = __builtin_amdgcn_exp2f(tmp[j] * a.inv_tau_log2 - m);
            tmp[j] = e;
            z += e;
        }
        z = block_reduce(z, false, misc);
        const float f = a.lambda / z;
        for (int j = tid; j < u.Tv; j += nt) S[live_to_pos(u, a, j)] -= f * tmp[j];
        __syncthreads();
    }
}

// Everything after S sits in LDS: refinements, optional score output, selection, optional list output, compaction.
template <int D, int DT>
__device__ inline void unit_tail(const Args &a, const Unit &u, char *smem, const int *tbl, const int *dst, Misc *misc) {
    const int tid = threadIdx.x, nt = blockDim.x;
    float *S = (float *)(smem + a.off_S);
    int *list = (int *)(smem + a.off_union);
    if (a.stages & STAGE_LOAD_SCORES) {
        const float *src = a.scores_in + (size_t)u.unit * a.scores_in_stride;
        for (int t = tid; t < u.T; t += nt) S[t] = src[t];
        __syncthreads();
    }
    if ((a.stages & STAGE_SCORE) && (a.ex & (EX_GLOBAL | EX_POOL | EX_RED))) refine_unit<D, DT>(a, u, smem, tbl, misc);
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
    if (a.stages & STAGE_COMPACT) {
        if (a.ex & EX_MOVE_F_LDS) compact_unit<2>(a, u, tbl, dst, list, (const float *)(smem + a.off_G), u.k);
        else if (a.ex & EX_MOVE_F) compact_unit<1>(a, u, tbl, dst, list, nullptr, u.k);
        else compact_unit<0>(a, u, tbl, dst, list, nullptr, u.k);
    }
}

}  // namespace zp

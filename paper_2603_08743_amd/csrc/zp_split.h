// Split-unit kernel of libzp (bf16 pools), kernel and launcher templates; instantiated in zp_split*.hip.
// Split-unit kernel: C workgroups share one unit (request, layer, kv head).
//
// Why: the max over the query heads of a group needs every row's final softmax normaliser, so the
// keys must be swept twice (appendix "Paged Attention Score").  A unit's keys (1 MiB for 4112
// positions) fit neither LDS nor the L2 share of a workgroup, and a second sweep from HBM costs
// 28 % extra traffic.  Here every workgroup keeps a chunk of at most 256 keys resident in LDS
// (64 KiB, XOR-swizzled rows), runs sweep 1 on it, publishes the chunk's per-row (max, sum), waits
// until the last of the C workgroups has combined them into the unit's log-sum-exp, runs sweep 2
// from the same LDS chunk and writes its slice of S.  The workgroup that finishes a unit last
// gathers S and does selection and compaction for the whole unit (nobody waits for that).
//
// The one wait is made safe the way decoupled look-back scans do it: workgroups draw their logical
// id from an atomic ticket when they START, so the peers a workgroup waits for have lower tickets
// (already running) or belong to the single partly started unit of its ticket stream, which the
// GPU can always finish admitting because at most (streams x (C-1)) workgroups can be waiting.
// The wait loop is bounded; on expiry the unit is reported (BAD_SYNC), a drain flag is raised and every
// workgroup that sees it exits.
#pragma once
#include "zp_device.h"

namespace zp {

// Data exchanged between the workgroups of a unit is written and read with relaxed device-scope atomic
// accesses (they bypass the non-coherent cache levels), and a workgroup raises its arrival counter only after
// s_waitcnt vmcnt(0) + barrier, i.e. once every one of its stores has completed.  Device-scope fences are
// avoided on purpose: each one writes back / invalidates a whole L2 and they made this kernel 10x slower.
__device__ __forceinline__ void xstore(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float xload(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void xstore2(float2 *p, float x, float y) {
    const unsigned long long bits = ((unsigned long long)__float_as_uint(y) << 32) | __float_as_uint(x);
    __hip_atomic_store((unsigned long long *)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 xload2(const float2 *p) {
    const unsigned long long bits = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)bits), __uint_as_float((unsigned)(bits >> 32)));
}
__device__ __forceinline__ void stores_done_barrier() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

__device__ __forceinline__ float sexp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float slog2(float x) { return __builtin_amdgcn_logf(x); }

// padded query row (block gb, row m32 of the 32x32 tile) -> window row uu and head g; false for zero rows.
// One half-wave of a tile owns 16 accumulator slots per key column: slot i = ul*G + g.
__device__ __forceinline__ bool split_row(int gb, int m32, int G, int UL, int w, int &uu, int &g) {
    const int mh = (m32 >> 2) & 1, i = ((m32 >> 3) << 2) | (m32 & 3);
    const int ul = i / G;
    g = i - ul * G;
    uu = (gb * 2 + mh) * UL + ul;
    return ul < UL && uu < w;
}

template <int D, int RB, int NW, int GT>
__global__ void __launch_bounds__(NW * 64) unit_split(const Args a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    Misc *misc = (Misc *)(smem + a.off_misc);
    constexpr int NT = NW * 64, KK = D / 16, CPR = D * 2 / 16, ROWB = D * 2, SUBS = SPLIT_SUBS;
    constexpr int LPT = SUBS * 32 * CPR / NT;
    static_assert(SUBS * 32 * CPR % NT == 0, "chunk pieces must divide evenly among the threads");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hf = lane >> 5;
    const int units = a.B * a.L_slab * a.h_kv;
    int *arrive1 = a.sync + 256, *ready1 = arrive1 + units, *arrive2 = ready1 + units;   // tickets: one 128-byte line per stream

    // An earlier wait expired: drain the grid.  One thread reads the flag and the whole workgroup takes the same
    // exit (a per-thread test could let thread 0 leave before it has drawn the ticket the others then wait for).
    if (tid == 0) misc->bad = __hip_atomic_load(&a.status[3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (misc->bad) return;
    // logical id in start order
    const int xs = a.NS > 1 ? (int)(blockIdx.x % (unsigned)a.NS) : 0;
    if (tid == 0) misc->sel_digit = atomicAdd(&a.sync[xs * 32], 1);
    __syncthreads();
    const int ticket = misc->sel_digit;
    const int cl = ticket / a.C, c = ticket - cl * a.C;
    const int unit = xs + a.NS * cl;
    if (unit >= units) return;

    Unit u;
    const int bad = unit_scalars(a, unit, u);
    if (bad) {                                               // every workgroup of the unit takes this exit
        if (c == 0 && tid == 0) report_bad(a, unit, bad);
        return;
    }
    const int G = GT ? GT : a.G, UL = 16 / G, w = a.w;
    const float sc = a.scale_log2;
    char *chunk = smem + a.off_chunk;
    float *part = (float *)(smem + a.off_part);              // [NW][SUBS*32]

    // this workgroup's keys: 32-key subtiles [s_lo, s_hi) of the live sequence
    const int nsub = (u.Tv + 31) >> 5;
    const int s_lo = (int)(((long long)c * nsub) / a.C), s_hi = (int)(((long long)(c + 1) * nsub) / a.C);
    const int ns = s_hi - s_lo, j_lo = s_lo * 32, nrows = ns * 32;

    // key chunk HBM -> registers -> LDS (row r, 16-byte piece p stored at piece p ^ (r mod CPR))
    {
        u32x4 stage[LPT];
        const int *tblg = a.block_table + (size_t)u.n * a.max_blocks;
#pragma unroll
        for (int i = 0; i < LPT; i++) {
            const int idx = tid + i * NT, row = idx / CPR, ch = idx - row * CPR;
            if (row < nrows) {
                int j = j_lo + row;
                j = j < u.Tv ? j : u.Tv - 1;                 // rows past the end repeat the last key (masked later)
                const int t = live_to_pos(u, a, j), blk = div_b(a, t);
                int p = tblg[blk];
                if (p < 0 || p >= a.N_total) p = 0;          // the finishing workgroup re-checks the table and reports
                stage[i] = *(const u32x4 *)(a.k + row_off(a, u.ls, p, t - blk * a.b, u.h) + ch * 16);
            }
        }
#pragma unroll
        for (int i = 0; i < LPT; i++) {
            const int idx = tid + i * NT, row = idx / CPR, ch = idx - row * CPR;
            if (row < nrows) *(u32x4 *)(chunk + row * ROWB + ((ch ^ (row & (CPR - 1))) << 4)) = stage[i];
        }
    }

    // query fragments of this wave's RB blocks (registers), as in the row layout described above
    bf16x8 qf[RB][KK];
    int u_col[RB];
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
        const int gb = wv * RB + rb;
        int uu, g;
        const bool ok = split_row(gb, l32, G, UL, w, uu, g);
        u_col[rb] = ok ? uu : -1;
        const char *qp = a.q + ((((size_t)u.ls * a.M + u.slot) * w + (ok ? uu : 0)) * a.h_q + u.h * G + g) * (size_t)ROWB + hf * 16;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (ok) raw = *(const u32x4 *)(qp + kk * 32);
            qf[rb][kk] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    __syncthreads();

    const int sw = l32 & (CPR - 1);
    const char *krow = chunk + l32 * ROWB;                   // + s*32*ROWB + ((kk*2+hf) ^ sw)*16

    // ---------------- sweep 1: running (max, sum of exp2) of every query row over this chunk
    float rm[RB], rl[RB];
#pragma unroll
    for (int rb = 0; rb < RB; rb++) { rm[rb] = -1e30f; rl[rb] = 0.f; }
#pragma unroll 1
    for (int s = 0; s < ns; s++) {
        f32x16 acc[RB];
#pragma unroll
        for (int rb = 0; rb < RB; rb++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[rb][i] = 0.f;
        const char *kp = krow + s * 32 * ROWB;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
            const bf16x8 kf = *(const bf16x8 *)(kp + (((kk * 2 + hf) ^ sw) << 4));
#pragma unroll
            for (int rb = 0; rb < RB; rb++) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][kk], acc[rb], 0, 0, 0);
        }
        const int j0 = j_lo + s * 32;
        const bool edge = j0 + 32 > u.Tv - w;
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {
            if (edge) {
                const int lim = u_col[rb] >= 0 ? u.Tv - w + u_col[rb] : u.Tv - 1;
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int j = j0 + 4 * hf + 8 * (i >> 2) + (i & 3);
                    if (j > lim) acc[rb][i] = -INFINITY;
                }
            }
            float tm = acc[rb][0];
#pragma unroll
            for (int i = 1; i < 16; i++) tm = fmaxf(tm, acc[rb][i]);
            const float mn = fmaxf(rm[rb], tm * sc);
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; i++) sum += sexp2(fmaf(acc[rb][i], sc, -mn));
            rl[rb] = rl[rb] * sexp2(rm[rb] - mn) + sum;
            rm[rb] = mn;
        }
    }
    {
        float2 *mine = a.partial + ((size_t)unit * a.C + c) * a.RP;
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {                    // the two half-waves hold the same row, different keys
            const float mo = __shfl_xor(rm[rb], 32), lo = __shfl_xor(rl[rb], 32);
            const float mm = fmaxf(rm[rb], mo);
            const float ll = rl[rb] * sexp2(rm[rb] - mm) + lo * sexp2(mo - mm);
            if (hf == 0) xstore2(&mine[(wv * RB + rb) * 32 + l32], mm, ll);
        }
    }

    // ---------------- rendezvous: the last workgroup to arrive combines the chunks (fixed order: deterministic)
    stores_done_barrier();
    if (tid == 0) misc->sel_gt = (__hip_atomic_fetch_add(&arrive1[unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.C - 1);
    __syncthreads();
    if (misc->sel_gt) {
        for (int r = tid; r < a.RP; r += NT) {
            int uu, g;
            float lse = INFINITY;                            // zero rows: exp2(x - inf) = 0 in sweep 2
            if (split_row(r >> 5, r & 31, G, UL, w, uu, g)) {
                float m = -1e30f, l = 0.f;
                const float2 *pr = a.partial + (size_t)unit * a.C * a.RP + r;
                for (int c0 = 0; c0 < a.C; c0 += 16) {          // 16 independent loads in flight, then a fixed-order combine
                    float2 pl[16];
#pragma unroll
                    for (int q = 0; q < 16; q++) pl[q] = xload2(pr + (size_t)(c0 + q < a.C ? c0 + q : a.C - 1) * a.RP);
#pragma unroll
                    for (int q = 0; q < 16; q++) {
                        if (c0 + q < a.C) {
                            const float mm = fmaxf(m, pl[q].x);
                            l = l * sexp2(m - mm) + pl[q].y * sexp2(pl[q].x - mm);
                            m = mm;
                        }
                    }
                }
                lse = m + slog2(l);
            }
            xstore(&a.lse_g[(size_t)unit * a.RP + r], lse);
        }
        stores_done_barrier();
        if (tid == 0) __hip_atomic_store(&ready1[unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        if (tid == 0) {
            int it = 0, ok = 1;
            while (__hip_atomic_load(&ready1[unit], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
                __builtin_amdgcn_s_sleep(16);
                if (++it > a.spin_limit || __hip_atomic_load(&a.status[3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                    __hip_atomic_store(&a.status[3], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = 0;
                    break;
                }
            }
            misc->bad = ok ? 0 : BAD_SYNC;
        }
        __syncthreads();
        if (misc->bad) {
            if (tid == 0) {                                      // first reporter also leaves what it saw for the error text
                if (a.len_out) a.len_out[unit] = -1;
                if (atomicCAS(&a.status[0], 0, 1) == 0) {
                    a.status[1] = unit;
                    a.status[2] = BAD_SYNC;
                    a.status[4] = __hip_atomic_load(&arrive1[unit], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    a.status[5] = __hip_atomic_load(&a.sync[xs * 32], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    a.status[6] = ticket;
                    a.status[7] = (int)blockIdx.x;
                }
            }
            return;
        }
    }

    // ---------------- sweep 2: S[t] = (1/w) sum_u max_g exp2(x - lse), from the same LDS chunk
    float lr[RB][16];
    int ub[RB];
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
        const int gb = wv * RB + rb;
        ub[rb] = (gb * 2 + hf) * UL;
        const float *lp = a.lse_g + (size_t)unit * a.RP + gb * 32 + 4 * hf;
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
            const float2 v0 = xload2((const float2 *)(lp + 8 * q4)), v1 = xload2((const float2 *)(lp + 8 * q4 + 2));
            lr[rb][4 * q4 + 0] = v0.x; lr[rb][4 * q4 + 1] = v0.y; lr[rb][4 * q4 + 2] = v1.x; lr[rb][4 * q4 + 3] = v1.y;
        }
    }
#pragma unroll 1
    for (int s = 0; s < ns; s++) {
        f32x16 acc[RB];
#pragma unroll
        for (int rb = 0; rb < RB; rb++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[rb][i] = 0.f;
        const char *kp = krow + s * 32 * ROWB;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
            const bf16x8 kf = *(const bf16x8 *)(kp + (((kk * 2 + hf) ^ sw) << 4));
#pragma unroll
            for (int rb = 0; rb < RB; rb++) acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][kk], kf, acc[rb], 0, 0, 0);
        }
        const int j0 = j_lo + s * 32, j = j0 + l32;
        const bool edge = j0 + 32 > u.Tv - w;
        const int thr = j - (u.Tv - w);                      // window rows u < thr come before key j: hidden
        float ps = 0.f;
#pragma unroll
        for (int rb = 0; rb < RB; rb++) {
            float p[16];
#pragma unroll
            for (int i = 0; i < 16; i++) p[i] = sexp2(fmaf(acc[rb][i], sc, -lr[rb][i]));
            if (GT) {
#pragma unroll
                for (int ul = 0; ul < (GT ? 16 / GT : 1); ul++) {
                    float mx = p[ul * GT];
#pragma unroll
                    for (int g = 1; g < GT; g++) mx = fmaxf(mx, p[ul * GT + g]);
                    if (edge && ub[rb] + ul < thr) mx = 0.f;
                    ps += mx;
                }
            } else {
                float mx = 0.f;
                int g = 0, ul = 0;
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const float v = (edge && ub[rb] + ul < thr) ? 0.f : p[i];
                    mx = fmaxf(mx, v);
                    if (++g == G) { ps += mx; mx = 0.f; g = 0; ul++; }
                }
            }
        }
        ps += __shfl_xor(ps, 32);
        if (hf == 0) part[wv * (SUBS * 32) + s * 32 + l32] = ps;
    }
    __syncthreads();
    {
        float *so = a.sbuf + (size_t)unit * a.T_max;
        for (int r = tid; r < nrows; r += NT) {
            const int jj = j_lo + r;
            if (jj < u.Tv) {
                float s = 0.f;
#pragma unroll
                for (int v = 0; v < NW; v++) s += part[v * (SUBS * 32) + r];   // fixed order over the waves
                xstore(&so[live_to_pos(u, a, jj)], s / (float)w);
            }
        }
    }

    // ---------------- the workgroup that completes the unit finishes it
    stores_done_barrier();
    if (tid == 0) misc->sel_gt = (__hip_atomic_fetch_add(&arrive2[unit], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.C - 1);
    __syncthreads();
    if (!misc->sel_gt) return;
    int *tbl = (int *)(smem + a.off_tbl), *dst = (int *)(smem + a.off_dst);
    if (!unit_setup(a, unit, u, tbl, dst, misc)) return;
    float *S = (float *)(smem + a.off_S);
    {
        const float *si = a.sbuf + (size_t)unit * a.T_max;
        const int stale_hi = (u.N - 1) * a.b;
        for (int t = tid; t < u.T; t += NT) S[t] = (t < u.vl || t >= stale_hi) ? xload(&si[t]) : 0.f;
    }
    __syncthreads();
    unit_tail<0, 1>(a, u, smem, tbl, dst, misc);
}

template <class K> static hipError_t allow_big_lds_split(K kernel) {
    static hipError_t state = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return state;
}

template <int D, int RB, int NW>
static hipError_t launch_g(const Args &a, int units, hipStream_t s) {
    const dim3 grid((unsigned)((size_t)units * a.C)), block(NW * 64);
#define ZP_LAUNCH(GT)                                                                        \
    {                                                                                        \
        hipError_t e = allow_big_lds_split(unit_split<D, RB, NW, GT>);                       \
        if (e != hipSuccess) return e;                                                       \
        hipLaunchKernelGGL((unit_split<D, RB, NW, GT>), grid, block, a.lds_bytes, s, a);     \
    }                                                                                        \
    break;
    switch (a.G) {
        case 4: ZP_LAUNCH(4)
        case 5: ZP_LAUNCH(5)
        case 7: ZP_LAUNCH(7)
        case 8: ZP_LAUNCH(8)
        default: ZP_LAUNCH(0)
    }
#undef ZP_LAUNCH
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const Args &a, int units, int NW, int RB, hipStream_t s) {
    if (RB == 1 && NW == 1) return launch_g<D, 1, 1>(a, units, s);
    if (RB == 1 && NW == 2) return launch_g<D, 1, 2>(a, units, s);
    if (RB == 1 && NW == 4) return launch_g<D, 1, 4>(a, units, s);
    if (RB == 2 && NW == 4) return launch_g<D, 2, 4>(a, units, s);
    if (RB == 2 && NW == 8) return launch_g<D, 2, 8>(a, units, s);
    if (RB == 3 && NW == 8) return launch_g<D, 3, 8>(a, units, s);
    if (RB == 4 && NW == 8) return launch_g<D, 4, 8>(a, units, s);
    return hipErrorInvalidConfiguration;
}

}  // namespace zp

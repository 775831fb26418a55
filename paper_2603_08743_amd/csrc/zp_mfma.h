// Matrix-core unit kernel of libzp (bf16 pools) and its launcher templates.  The instantiations are spread over
// several translation units (zp_mfma_*.hip) so that they compile in parallel.
#pragma once
#include "zp_device.h"

#include <type_traits>

namespace zp {

// Key tiles: the first sweep loads them normally (the second sweep, which runs the other way, finds the most recent
// ones in L2 / Infinity Cache); the second sweep is their last use by this workgroup and loads them non-temporally.
// Measured on the 8B-like shape: non-temporal in sweep 1 costs 0.5 ms per launch, in sweep 2 it gains 0.1-0.3 ms.
#define ZP_NT1 std::false_type
#define ZP_NT2 std::true_type

// Waves per SIMD the register allocation aims at.  One query block per wave (RB = 1) fits 128 registers: eight such
// waves per workgroup and two workgroups per CU put four waves on every SIMD, which overlaps the matrix-core and
// vector-ALU phases of different waves and gives the row-moving phase sixteen waves per CU to issue memory operations
// from (measured on the 8B-like shape: 15.0 ms per launch against 17.0 ms with four waves of two blocks each).
#define ZP_WPE(NW, RB) ((NW) == 8 && (RB) == 1 ? 4 : ((NW) >= 4 ? 2 : 1))

// ------------------------------------------------------------------ MFMA path (bf16)
//
// Query rows are laid out so that both reductions of sweep 2 stay inside a lane.  A 32x32 MFMA
// tile gives lane L, register i the element (row 4*(L/32) + 8*(i/4) + i%4, column L%32).  With
// the query block as the row operand, one half-wave (hf = L/32) owns 16 rows of the block per
// key column; those 16 slots hold UL = 16/G window rows u with their G query heads side by side
// (slot i = ul*G + g; left-over slots are zero rows).  Block gb, half hf, slot i therefore is
// window row u = (gb*2 + hf)*UL + i/G, head g = i%G.  NW waves split the NB blocks (RB each) and
// share every key tile through LDS.  In sweep 1 the operands swap, so a lane owns one query row
// and 16 keys per tile and the running (max, sum) of a row never leaves its lane.

template <int D> struct KTile {
    static constexpr int ROW = D * 2 + 16;        // padded row stride in bytes: conflict-free 16-byte fragment reads
    static constexpr int BYTES = KT * ROW;
    static constexpr int CPR = D * 2 / 16;        // 16-byte pieces per key row
};

// RED: the launch computes the lightning redundancy with block size 16 and takes the similarity tiles of the live
// prefix from the key tiles of sweep 2 (instantiated for RB = 1 only; otherwise the keys are read a third time in the tail).
template <int D, int RB, int NW, int GT, bool RED>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(ZP_WPE(NW, RB)))) unit_mfma(const Args a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *tbl = (int *)(smem + a.off_tbl), *dst = (int *)(smem + a.off_dst);
    Misc *misc = (Misc *)(smem + a.off_misc);
    Unit u;
    if (!unit_setup(a, unit_of_block((int)blockIdx.x, (int)gridDim.x, a.xcd_map), u, tbl, dst, misc)) return;

    using KTl = KTile<D>;
    constexpr int NT = NW * 64, KK = D / 16, LPT = KT * KTl::CPR / NT;
    static_assert(KT * KTl::CPR % NT == 0, "tile pieces must divide evenly among the threads");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hf = lane >> 5;
    const int G = GT ? GT : a.G, UL = 16 / G, w = a.w;
    float *S = (float *)(smem + a.off_S);
    char *kbuf = smem + a.off_union;
    float *part = (float *)(kbuf + 2 * KTl::BYTES);          // [2][NW][KT] partial sums of sweep 2
    float *lse = part + 2 * NW * KT;                         // [NB*32] per padded query row
    const float c = a.scale_log2;

    for (int t = tid; t < u.T; t += NT) S[t] = 0.f;          // stale positions stay 0

    // query fragments: this lane supplies padded row l32 of each of its blocks, 8 elements per 16-wide k step
    bf16x8 qf[RB][KK];
    int u_col[RB];                                           // window row this lane owns in sweep 1 (-1: zero row)
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
        const int gb = wv * RB + rb;
        const int mh = (l32 >> 2) & 1, i = ((l32 >> 3) << 2) | (l32 & 3);
        const int ul = i / G, g = i - ul * G, uu = (gb * 2 + mh) * UL + ul;
        const bool ok = ul < UL && uu < w;
        u_col[rb] = ok ? uu : -1;
        const char *qp = a.q + ((((size_t)u.ls * a.M + u.slot) * w + (ok ? uu : 0)) * a.h_q + u.h * G + g) * (size_t)(D * 2) + hf * 16;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (ok) raw = *(const u32x4 *)(qp + kk * 32);
            qf[rb][kk] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    const int ntiles = (u.Tv + KT - 1) / KT;
    // Key tiles travel HBM -> registers -> LDS.  Two register sets alternate so that a tile is requested two
    // iterations before it is needed (one tile of compute is shorter than the HBM latency).
    u32x4 stA[LPT], stB[LPT];
    // a thread always fetches the same 16-byte piece of rows r0, r0 + RSTEP, ...: one 64-bit base, then
    // base + token * (bytes between consecutive tokens) with token = block * b + slot (fits 32 bits, host-checked)
    constexpr int RSTEP = NT / KTl::CPR;
    const int r0 = tid / KTl::CPR;
    const char *kbase = a.k + ((size_t)u.ls * a.N_total * a.b * a.h_kv + u.h) * (size_t)(D * 2) + (tid - r0 * KTl::CPR) * 16;
    const unsigned tok_bytes = (unsigned)a.h_kv * (D * 2);
    const int gap = (u.N - 1) * a.b - u.vl;                   // stale positions between the live prefix and the last block
    auto gload = [&](int tile, u32x4 (&st)[LPT], auto nt_tag) {   // rows past the end repeat the last key (masked later)
        // Tiles that lie wholly in the live prefix (all but the last one or two) need none of the edge handling when
        // the block size is a power of two: position = live index.  (Eight-wave workgroups only: with fewer waves a
        // thread loads eight or sixteen pieces per tile and the second copy of that code costs registers.)
        if (NW == 8 && a.b_shift >= 0 && (tile + 1) * KT <= u.vl) {
#pragma unroll
            for (int i = 0; i < LPT; i++) {
                const int j = tile * KT + i * RSTEP + r0;
                const unsigned tok = ((unsigned)tbl[j >> a.b_shift] << a.b_shift) + (unsigned)(j & (a.b - 1));
                if (decltype(nt_tag)::value) st[i] = __builtin_nontemporal_load((const u32x4 *)(kbase + (size_t)tok * tok_bytes));
                else st[i] = *(const u32x4 *)(kbase + (size_t)tok * tok_bytes);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; i++) {
            int j = tile * KT + r0 + i * RSTEP;
            j = j < u.Tv ? j : u.Tv - 1;
            const int t = j < u.vl ? j : j + gap;
            unsigned tok;
            if (a.b_shift >= 0) {
                const int blk = t >> a.b_shift;
                tok = ((unsigned)tbl[blk] << a.b_shift) + (unsigned)(t & (a.b - 1));
            } else {
                const int blk = t / a.b;
                tok = (unsigned)tbl[blk] * (unsigned)a.b + (unsigned)(t - blk * a.b);
            }
            if (decltype(nt_tag)::value) st[i] = __builtin_nontemporal_load((const u32x4 *)(kbase + (size_t)tok * tok_bytes));
            else st[i] = *(const u32x4 *)(kbase + (size_t)tok * tok_bytes);
        }
    };
    const int lds_st = r0 * KTl::ROW + (tid - r0 * KTl::CPR) * 16;
    auto lstore = [&](char *buf, const u32x4 (&st)[LPT]) {
#pragma unroll
        for (int i = 0; i < LPT; i++) *(u32x4 *)(buf + lds_st + i * RSTEP * KTl::ROW) = st[i];
    };
    char *buf0 = kbuf, *buf1 = kbuf + KTl::BYTES;
    f32x16 zero16;
#pragma unroll
    for (int i = 0; i < 16; i++) zero16[i] = 0.f;

    // ---------------- sweep 1: per query row, running max and sum of exp2 over the keys it may see
    float rm[RB], rl[RB];
#pragma unroll
    for (int rb = 0; rb < RB; rb++) { rm[rb] = -1e30f; rl[rb] = 0.f; }
    // The sum of exp2(x - ref) is kept against a per-row reference `rm` that only moves when the sum leaves the
    // safe range (first subtile, or logits that jump by more than ~2^100): then the subtile is redone with the
    // proper maximum.  This keeps the common path free of the max reduction: fma, exp2, add per logit.
    auto sweep1_body = [&](const char *buf, int j0, auto edge_tag) {
        constexpr bool edge = decltype(edge_tag)::value;
#pragma unroll
        for (int sub = 0; sub < KT / 32; sub++) {
            f32x16 acc[RB];
            const char *kp = buf + (sub * 32 + l32) * KTl::ROW + hf * 16;
#pragma unroll
            for (int kk = 0; kk < KK; kk++) {
                const bf16x8 kf = *(const bf16x8 *)(kp + kk * 32);
#pragma unroll
                for (int rb = 0; rb < RB; rb++)
                    acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][kk], kk ? acc[rb] : zero16, 0, 0, 0);
            }
            // acc[rb][i]: key j0 + sub*32 + 4*hf + 8*(i/4) + i%4, query row = this lane's column
#pragma unroll
            for (int rb = 0; rb < RB; rb++) {
                if (edge) {
                    const int lim = u_col[rb] >= 0 ? u.Tv - w + u_col[rb] : u.Tv - 1;
#pragma unroll
                    for (int i = 0; i < 16; i++) {
                        const int j = j0 + sub * 32 + 4 * hf + 8 * (i >> 2) + (i & 3);
                        if (j > lim) acc[rb][i] = -INFINITY;
                    }
                }
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; i++) sum += fexp2(fmaf(acc[rb][i], c, -rm[rb]));
                const float ln = rl[rb] + sum;
                if (__builtin_expect(__any(!(ln < 1e30f)), 0)) {        // wave-uniform, rare
                    float tm = acc[rb][0];
#pragma unroll
                    for (int i = 1; i < 16; i++) tm = fmaxf(tm, acc[rb][i]);
                    const float mn = fmaxf(rm[rb], tm * c);
                    sum = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; i++) sum += fexp2(fmaf(acc[rb][i], c, -mn));
                    rl[rb] = rl[rb] * fexp2(rm[rb] - mn) + sum;
                    rm[rb] = mn;
                } else {
                    rl[rb] = ln;
                }
            }
        }
    };
    auto sweep1_tile = [&](const char *buf, int j0) {
        if (j0 + KT > u.Tv - w) sweep1_body(buf, j0, std::true_type());
        else sweep1_body(buf, j0, std::false_type());
    };
    gload(0, stA, ZP_NT1());
    lstore(buf0, stA);
    if (ntiles > 1) gload(1, stA, ZP_NT1());
    __syncthreads();
#pragma unroll 1
    for (int it = 0; it < ntiles; it += 2) {
        if (it + 2 < ntiles) gload(it + 2, stB, ZP_NT1());
        sweep1_tile(buf0, it * KT);
        if (it + 1 < ntiles) lstore(buf1, stA);
        __syncthreads();
        if (it + 1 >= ntiles) break;
        if (it + 3 < ntiles) gload(it + 3, stA, ZP_NT1());
        sweep1_tile(buf1, (it + 1) * KT);
        if (it + 2 < ntiles) lstore(buf0, stB);
        __syncthreads();
    }
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {                         // the two half-waves hold the same row, different keys
        const float mo = __shfl_xor(rm[rb], 32), lo = __shfl_xor(rl[rb], 32);
        const float mm = fmaxf(rm[rb], mo);
        const float ll = rl[rb] * fexp2(rm[rb] - mm) + lo * fexp2(mo - mm);
        if (hf == 0) lse[(wv * RB + rb) * 32 + l32] = u_col[rb] >= 0 ? mm + flog2(ll) : INFINITY;
    }
    __syncthreads();

    // ---------------- sweep 2: S[t] = (1/w) sum_u max_g exp2(x - lse)
    // The products start from -lse / c instead of zero (the accumulator input of the first matrix instruction), so the
    // matrix cores deliver x - lse / c, the logit minus the row's normaliser in units of 1 / c: nothing is left to
    // subtract per logit.  Zero rows have lse = +inf, i.e. start and stay at -inf.
    f32x16 lrn[RB];
    int ub[RB];                                               // first window row of this half-wave's 16 slots
    const float inv_c = 1.0f / c;
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
        const int gb = wv * RB + rb;
        ub[rb] = (gb * 2 + hf) * UL;
#pragma unroll
        for (int i = 0; i < 16; i++) lrn[rb][i] = -lse[gb * 32 + 4 * hf + 8 * (i >> 2) + (i & 3)] * inv_c;
    }
    // max_g exp2(x_g - lse_g) = exp2(c max_g (x_g - lse_g) / c): the maximum over the group is taken before the
    // exponential (c > 0), so a window row costs one multiply and one exp2 instead of G of each.
    auto sweep2_body = [&](const char *buf, float *pt, int j0, auto edge_tag) {
        constexpr bool edge = decltype(edge_tag)::value;
#pragma unroll
        for (int sub = 0; sub < KT / 32; sub++) {
            f32x16 acc[RB];
            const char *kp = buf + (sub * 32 + l32) * KTl::ROW + hf * 16;
#pragma unroll
            for (int kk = 0; kk < KK; kk++) {
                const bf16x8 kf = *(const bf16x8 *)(kp + kk * 32);
#pragma unroll
                for (int rb = 0; rb < RB; rb++)
                    acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][kk], kf, kk ? acc[rb] : lrn[rb], 0, 0, 0);
            }
            // acc[rb][i]: slot i of this half-wave, key j = j0 + sub*32 + l32
            const int j = j0 + sub * 32 + l32;
            const int thr = j - (u.Tv - w);                   // window rows u < thr come before key j: hidden
            float ps = 0.f;
#pragma unroll
            for (int rb = 0; rb < RB; rb++) {
                const f32x16 &y = acc[rb];                    // (x - lse) / c in base 2; zero rows: -inf
                if (GT) {
#pragma unroll
                    for (int ul = 0; ul < (GT ? 16 / GT : 1); ul++) {
                        float mx = y[ul * GT];
#pragma unroll
                        for (int g = 1; g < GT; g++) mx = fmaxf(mx, y[ul * GT + g]);
                        if (edge && ub[rb] + ul < thr) mx = -INFINITY;
                        ps += fexp2(mx * c);
                    }
                } else {                                      // group size known only at run time
                    float mx = -INFINITY;
                    int g = 0, ul = 0;
#pragma unroll
                    for (int i = 0; i < 16; i++) {
                        const float v = (edge && ub[rb] + ul < thr) ? -INFINITY : y[i];
                        mx = fmaxf(mx, v);
                        if (++g == G) { ps += fexp2(mx * c); mx = -INFINITY; g = 0; ul++; }
                    }
                }
            }
            ps += __shfl_xor(ps, 32);
            if (hf == 0) pt[wv * KT + sub * 32 + l32] = ps;
        }
    };
    // Redundancy (RED, b = 16): a tile holds four blocks of the live prefix, one similarity tile each.  Turning a tile
    // of products into row sums is a chain of dependent lane exchanges which the whole workgroup waits for at the tile
    // barrier, so it runs once per PAIR of tiles, all eight blocks of the pair on the eight waves at once (fewer waves
    // take several blocks in turn).  The first tile of a pair is overwritten while the second is worked on, so the
    // waves that take its blocks compute the products (four registers per block) while it is still theirs to read and
    // hold them across the barrier.  The last block, off the 16-grid of the live sequence, is done in the tail.
    float *rs_red = (float *)(smem + a.off_R);
    const float inv_len = 1.0f / (float)u.Tv;
    constexpr int PER = KT / 16, HOLD = (PER + NW - 1) / NW;  // blocks per tile; first-tile blocks one wave takes
    f32x4 gacc[HOLD];
    auto gram_first = [&](const char *buf, int j0) {
#pragma unroll
        for (int h = 0; h < HOLD; h++) {
            const int q = wv + h * NW;
            if (q < PER && j0 + 16 * q < u.vl) gacc[h] = block_gram<D, KTl::ROW>(buf + 16 * q * KTl::ROW, lane);
        }
    };
    // jA: live index of the first tile (products held in gacc); bufB / jB: the second tile, jB < 0 if there is none
    auto gram_finish = [&](int jA, const char *bufB, int jB) {
#pragma unroll
        for (int h = 0; h < HOLD; h++) {
            const int q = wv + h * NW;
            if (q < PER && jA + 16 * q < u.vl) block_row_sums(a, u, gacc[h], jA + 16 * q, inv_len, rs_red, lane);
        }
        if (jB >= 0) {
            for (int q = wv; q < 2 * PER; q += NW) {
                const int qq = q - PER;
                if (qq >= 0 && jB + 16 * qq < u.vl)
                    block_row_sums(a, u, block_gram<D, KTl::ROW>(bufB + 16 * qq * KTl::ROW, lane), jB + 16 * qq, inv_len, rs_red, lane);
            }
        }
    };
    auto sweep2_tile = [&](const char *buf, float *pt, int j0) {
        if (j0 + KT > u.Tv - w) sweep2_body(buf, pt, j0, std::true_type());
        else sweep2_body(buf, pt, j0, std::false_type());
    };
    auto reduce_tile = [&](const float *pt, int j0) {         // fixed-order sum over the waves: deterministic
        if (tid < KT) {
            const int jj = j0 + tid;
            if (jj < u.Tv) {
                float s = 0.f;
#pragma unroll
                for (int v = 0; v < NW; v++) s += pt[v * KT + tid];
                S[live_to_pos(u, a, jj)] = s / (float)w;
            }
        }
    };
    float *pt0 = part, *pt1 = part + NW * KT;
    // tiles are taken in DESCENDING order (tile number rt = ntiles-1-it): the keys sweep 1 read last are the ones
    // most likely to be still in L2 / Infinity Cache
    gload(ntiles - 1, stA, ZP_NT2());
    lstore(buf0, stA);
    if (ntiles > 1) gload(ntiles - 2, stA, ZP_NT2());
    __syncthreads();
#pragma unroll 1
    for (int it = 0; it < ntiles; it += 2) {
        const int rt = ntiles - 1 - it;
        if (it + 2 < ntiles) gload(rt - 2, stB, ZP_NT2());
        sweep2_tile(buf0, pt0, rt * KT);
        if (RED) {
            gram_first(buf0, rt * KT);
            if (it + 1 >= ntiles) gram_finish(rt * KT, nullptr, -1);
        }
        if (it + 1 < ntiles) lstore(buf1, stA);
        __syncthreads();
        reduce_tile(pt0, rt * KT);
        if (it + 1 >= ntiles) break;
        if (it + 3 < ntiles) gload(rt - 3, stA, ZP_NT2());
        sweep2_tile(buf1, pt1, (rt - 1) * KT);
        if (RED) gram_finish(rt * KT, buf1, (rt - 1) * KT);
        if (it + 2 < ntiles) lstore(buf0, stB);
        __syncthreads();
        reduce_tile(pt1, (rt - 1) * KT);
    }
    __syncthreads();
    unit_tail<D, 1>(a, u, smem, tbl, dst, misc);
}

template <int D, int RB, int NW>
static hipError_t launch_g(const Args &a, int units, hipStream_t s) {
    const dim3 grid(units), block(NW * 64);
#define ZP_LAUNCH(GT)                                                                                  \
    {                                                                                                  \
        if constexpr (RB == 1) {                                                                       \
            if (a.ex & EX_RED_FUSED) {                                                                 \
                hipError_t e = allow_big_lds(unit_mfma<D, RB, NW, GT, true>);                          \
                if (e != hipSuccess) return e;                                                         \
                hipLaunchKernelGGL((unit_mfma<D, RB, NW, GT, true>), grid, block, a.lds_bytes, s, a);  \
                break;                                                                                 \
            }                                                                                          \
        }                                                                                              \
        hipError_t e = allow_big_lds(unit_mfma<D, RB, NW, GT, false>);                                 \
        if (e != hipSuccess) return e;                                                                 \
        hipLaunchKernelGGL((unit_mfma<D, RB, NW, GT, false>), grid, block, a.lds_bytes, s, a);         \
    }                                                                                                  \
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

// the (RB, NW) geometries of one head dimension: WIDE = 0 up to four waves, WIDE = 1 eight waves
template <int D, int WIDE>
static hipError_t launch_d(const Args &a, int units, int NW, int RB, hipStream_t s) {
    if constexpr (!WIDE) {
        if (RB == 1 && NW == 1) return launch_g<D, 1, 1>(a, units, s);
        if (RB == 1 && NW == 2) return launch_g<D, 1, 2>(a, units, s);
        if (RB == 1 && NW == 4) return launch_g<D, 1, 4>(a, units, s);
    } else {
        if (RB == 1 && NW == 8) return launch_g<D, 1, 8>(a, units, s);
        if (RB == 2 && NW == 8) return launch_g<D, 2, 8>(a, units, s);
        if (RB == 3 && NW == 8) return launch_g<D, 3, 8>(a, units, s);
        if (RB == 4 && NW == 8) return launch_g<D, 4, 8>(a, units, s);
    }
    return hipErrorInvalidConfiguration;
}

}  // namespace zp

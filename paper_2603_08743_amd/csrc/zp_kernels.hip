// Unit kernels of libzp: one workgroup per (request, layer, kv head).
//
//  * unit_generic: scoring on the vector ALUs for any element type / group size / head
//    dimension (fp32 pools, odd shapes), and the staged select-only / compact-only passes.
//  * unit_mfma: bf16 pools.  The (G*w) x T logits are a dense contraction over d, so they run
//    on the matrix cores (v_mfma_f32_32x32x16_bf16) from LDS-staged key tiles.
//
// Scores follow the appendix "Paged Attention Score": softmax over positions per window
// query, max over the query heads of the group, mean over the window.  The max over heads
// needs the final normaliser of every row, and the (G*w) x T logits do not fit on chip, so
// the keys are swept twice: sweep 1 reduces each row to its log-sum-exp, sweep 2 recomputes
// the logits and reduces them to S[t] = (1/w) sum_u max_g exp(a[g,u,t] - lse[g,u]).
#include "zp_device.h"

namespace zp {

// ------------------------------------------------------------------ generic path

template <int DT> __device__ __forceinline__ float ld_elem(const char *p, int i);
template <> __device__ __forceinline__ float ld_elem<0>(const char *p, int i) { return ((const float *)p)[i]; }
template <> __device__ __forceinline__ float ld_elem<1>(const char *p, int i) {
    return __uint_as_float((unsigned)((const unsigned short *)p)[i] << 16);
}

template <int DT> __device__ __forceinline__ float dot_row(const char *q, const char *k, int d) {
    float acc = 0.f;
    for (int c = 0; c < d; c++) acc = fmaf(ld_elem<DT>(q, c), ld_elem<DT>(k, c), acc);
    return acc;
}

template <int DT>
__device__ void score_generic(const Args &a, const Unit &u, char *smem, const int *tbl) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wv = tid >> 6, nw = nt >> 6;
    float *S = (float *)(smem + a.off_S);
    float *lse = (float *)(smem + a.off_union);
    const int G = a.G, w = a.w, rows = G * w;
    const size_t qbase = (((size_t)u.ls * a.M + u.slot) * w) * a.h_q;   // in rows of d elements
    for (int t = tid; t < u.T; t += nt) S[t] = 0.f;
    // sweep 1: log-sum-exp (base 2) of every window row over the keys it may see
    for (int r = wv; r < rows; r += nw) {
        const int g = r / w, uu = r - g * w;
        const char *q = a.q + (qbase + (size_t)uu * a.h_q + u.h * G + g) * a.row_bytes;
        const int jmax = u.Tv - w + uu;                               // causal: keys after the query are hidden
        float m = -1e30f, l = 0.f;
        for (int j = lane; j <= jmax; j += 64) {
            const int t = live_to_pos(u, a, j), blk = div_b(a, t);
            const float x = dot_row<DT>(q, a.k + row_off(a, u.ls, tbl[blk], t - blk * a.b, u.h), a.d) * a.scale_log2;
            if (x > m) { l = l * fexp2(m - x) + 1.f; m = x; }
            else l += fexp2(x - m);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
            const float mm = fmaxf(m, mo);
            l = l * fexp2(m - mm) + lo * fexp2(mo - mm);
            m = mm;
        }
        if (lane == 0) lse[r] = m + flog2(l);
    }
    __syncthreads();
    // sweep 2: S[t] = (1/w) sum_u max_g exp2(x - lse)
    for (int j = tid; j < u.Tv; j += nt) {
        const int t = live_to_pos(u, a, j), blk = div_b(a, t);
        const char *kr = a.k + row_off(a, u.ls, tbl[blk], t - blk * a.b, u.h);
        float acc = 0.f;
        for (int uu = 0; uu < w; uu++) {
            if (j > u.Tv - w + uu) continue;
            float mx = 0.f;
            for (int g = 0; g < G; g++) {
                const char *q = a.q + (qbase + (size_t)uu * a.h_q + u.h * G + g) * a.row_bytes;
                const float x = dot_row<DT>(q, kr, a.d) * a.scale_log2;
                mx = fmaxf(mx, fexp2(x - lse[g * w + uu]));
            }
            acc += mx;
        }
        S[t] = acc / (float)w;
    }
    __syncthreads();
}

template <int DT>
__global__ void __launch_bounds__(256) unit_generic(const Args a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *tbl = (int *)(smem + a.off_tbl), *dst = (int *)(smem + a.off_dst);
    Misc *misc = (Misc *)(smem + a.off_misc);
    Unit u;
    if (!unit_setup(a, unit_of_block((int)blockIdx.x, (int)gridDim.x, a.xcd_map), u, tbl, dst, misc)) return;
    if (a.stages & STAGE_SCORE) score_generic<DT>(a, u, smem, tbl);
    unit_tail<0, DT>(a, u, smem, tbl, dst, misc);
}

hipError_t launch_unit_generic(const Args &a, int units, hipStream_t s) {
    if (units <= 0) return hipSuccess;
    hipError_t e = a.dtype == 0 ? allow_big_lds(unit_generic<0>) : allow_big_lds(unit_generic<1>);
    if (e != hipSuccess) return e;
    if (a.dtype == 0) hipLaunchKernelGGL(unit_generic<0>, dim3(units), dim3(256), a.lds_bytes, s, a);
    else hipLaunchKernelGGL(unit_generic<1>, dim3(units), dim3(256), a.lds_bytes, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ MFMA path (bf16): geometry and dispatch

size_t mfma_union_bytes(int d, int NW, int NB) {
    const size_t tile = (size_t)KT * (d * 2 + 16);
    return 2 * tile + 2 * (size_t)NW * KT * 4 + (size_t)NB * 32 * 4;
}

// (RB, NW) by the number of 32-row query blocks: small windows use fewer waves, large ones more rows per wave
static void pick_geometry(int NB, int *NW, int *RB) {
    if (NB <= 1) { *NW = 1; *RB = 1; }
    else if (NB <= 2) { *NW = 2; *RB = 1; }
    else if (NB <= 4) { *NW = 4; *RB = 1; }
    else if (NB <= 8) { *NW = 8; *RB = 1; }
    else if (NB <= 16) { *NW = 8; *RB = 2; }
    else if (NB <= 24) { *NW = 8; *RB = 3; }
    else { *NW = 8; *RB = 4; }
}

bool mfma_path_available(const Args &a, int *NW, int *RB) {
    if (a.dtype != 1 || (a.d != 128 && a.d != 64)) return false;
    if (a.G < 1 || a.G > 16) return false;
    const int UL = 16 / a.G, NB = (a.w + 2 * UL - 1) / (2 * UL);
    if (NB > 32) return false;
    pick_geometry(NB, NW, RB);
    return true;
}

hipError_t launch_unit_mfma(const Args &a, int units, int NW, int RB, hipStream_t s) {
    if (units <= 0) return hipSuccess;
    if (a.d == 128) return NW <= 4 ? launch_mfma_d128(a, units, NW, RB, s) : launch_mfma_d128_wide(a, units, NW, RB, s);
    if (a.d == 64) return NW <= 4 ? launch_mfma_d64(a, units, NW, RB, s) : launch_mfma_d64_wide(a, units, NW, RB, s);
    return hipErrorInvalidConfiguration;
}

}  // namespace zp

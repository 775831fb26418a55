// Check-only paged decode attention (not part of the compression path): one query per (request, layer,
// query head) attends to the first len[n][l][h] rows of the request's table, h = hq / G.  It exists so that
// a compacted cache with per-head lengths can be verified end to end, and as a decode-shaped load to run beside the
// compression; vector-ALU code.
#include "zp_kernels.h"

namespace zp {

template <int DT> __device__ __forceinline__ float ck_elem(const char *p, int i);
template <> __device__ __forceinline__ float ck_elem<0>(const char *p, int i) { return ((const float *)p)[i]; }
template <> __device__ __forceinline__ float ck_elem<1>(const char *p, int i) {
    return __uint_as_float((unsigned)((const unsigned short *)p)[i] << 16);
}

// grid: B * L_slab * h_q workgroups of 256 threads.  Keys are taken 256 at a time: thread t scores key t, the
// tile's probabilities go through LDS, then thread c accumulates output dimension c (coalesced over V rows).
template <int DT>
__global__ void __launch_bounds__(256) decode_attention(DecodeArgs a) {
    __shared__ float p_s[256];
    __shared__ float red[8];
    __shared__ int bad_s;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int item = blockIdx.x, hq = item % a.h_q, l = (item / a.h_q) % a.L_slab, n = item / (a.h_q * a.L_slab);
    const int G = a.h_q / a.h_kv, h = hq / G;
    const int len = a.len[((size_t)n * a.L_slab + l) * a.h_kv + h];
    float *out = a.out + (size_t)item * a.d;
    if (tid == 0) bad_s = 0;
    __syncthreads();
    if (len < 0 || len > a.table_stride * a.b) {
        if (tid == 0 && atomicCAS(&a.status[0], 0, 1) == 0) { a.status[1] = item; a.status[2] = BAD_KEEP; }
        return;
    }
    const int *tbl = a.table + (size_t)n * a.table_stride;
    const char *q = a.q + (size_t)item * a.row_bytes;
    const float scale = a.scale_log2;
    float m = -1e30f, lsum = 0.f, acc = 0.f;                      // acc: output dimension tid (if tid < d)
    for (int t0 = 0; t0 < len; t0 += 256) {
        const int t = t0 + tid;
        float x = -INFINITY;
        size_t roff = 0;
        if (t < len) {
            const int blk = t / a.b, p = tbl[blk];
            if (p < 0 || p >= a.N_total) bad_s = BAD_BLOCK_ID;
            else {
                roff = ((((size_t)l * a.N_total + p) * a.b + (t - blk * a.b)) * a.h_kv + h) * (size_t)a.row_bytes;
                float dot = 0.f;
                for (int c = 0; c < a.d; c++) dot = fmaf(ck_elem<DT>(q, c), ck_elem<DT>(a.k + roff, c), dot);
                x = dot * scale;
            }
        }
        // tile maximum
        float tm = x;
        for (int off = 32; off >= 1; off >>= 1) tm = fmaxf(tm, __shfl_xor(tm, off));
        if (lane == 0) red[wv] = tm;
        __syncthreads();
        if (bad_s) break;
        tm = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float mn = fmaxf(m, tm);
        const float p = __builtin_amdgcn_exp2f(x - mn);
        p_s[tid] = p;
        float ts = p;
        for (int off = 32; off >= 1; off >>= 1) ts += __shfl_xor(ts, off);
        if (lane == 0) red[4 + wv] = ts;
        __syncthreads();
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        lsum = lsum * corr + (red[4] + red[5] + red[6] + red[7]);
        m = mn;
        if (tid < a.d) {
            acc *= corr;
            const int nk = len - t0 < 256 ? len - t0 : 256;
            for (int kk = 0; kk < nk; kk++) {
                const int tt = t0 + kk, blk = tt / a.b;
                const size_t vo = ((((size_t)l * a.N_total + tbl[blk]) * a.b + (tt - blk * a.b)) * a.h_kv + h) * (size_t)a.row_bytes;
                acc = fmaf(p_s[kk], ck_elem<DT>(a.v + vo, tid), acc);
            }
        }
        __syncthreads();
    }
    if (bad_s) {
        if (tid == 0 && atomicCAS(&a.status[0], 0, 1) == 0) { a.status[1] = item; a.status[2] = bad_s; }
        return;
    }
    if (tid < a.d) out[tid] = len > 0 ? acc / lsum : 0.f;
}

// bf16, d = 64 or 128, up to 8 query heads per kv head: one workgroup per (request, layer, kv head) reads every K and V
// row once for the whole group (16-byte pieces, a row per 8 or 16 lanes), each lane keeps a running softmax of its rows
// for the G heads and its 8 output dimensions; row groups, then waves, are merged at the end.  This is the shape of a
// decode step's attention and serves as the load for measuring compression beside decoding.
typedef __attribute__((ext_vector_type(4))) unsigned int ck_u32x4;

template <int G, int D>
__global__ void __launch_bounds__(256) decode_attention_gqa(DecodeArgs a) {
    constexpr int CPR = D * 2 / 16, RPW = 64 / CPR, NW = 4, E = 8;
    __shared__ float s_m[NW][G], s_l[NW][G];
    __shared__ float s_acc[NW][G][D];
    __shared__ int bad_s;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, c = lane % CPR, rg = lane / CPR;
    const int item = blockIdx.x, h = item % a.h_kv, l = (item / a.h_kv) % a.L_slab, n = item / (a.h_kv * a.L_slab);
    const int len = a.len[((size_t)n * a.L_slab + l) * a.h_kv + h];
    if (tid == 0) bad_s = 0;
    __syncthreads();
    if (len < 0 || len > a.table_stride * a.b) {
        if (tid == 0 && atomicCAS(&a.status[0], 0, 1) == 0) { a.status[1] = item; a.status[2] = BAD_KEEP; }
        return;
    }
    const int *tbl = a.table + (size_t)n * a.table_stride;
    const size_t q0 = (((size_t)n * a.L_slab + l) * a.h_q + (size_t)h * G);
    auto unpack = [](const ck_u32x4 &w, float (&f)[E]) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    };
    float qf[G][E], m[G], ls[G], acc[G][E];
#pragma unroll
    for (int g = 0; g < G; g++) {
        unpack(*(const ck_u32x4 *)(a.q + (q0 + g) * (size_t)(D * 2) + c * 16), qf[g]);
        m[g] = -1e30f;
        ls[g] = 0.f;
#pragma unroll
        for (int e = 0; e < E; e++) { qf[g][e] *= a.scale_log2; acc[g][e] = 0.f; }
    }
    for (int t = wv * RPW + rg; t < len; t += NW * RPW) {
        const int blk = t / a.b;
        int p = tbl[blk];
        if (p < 0 || p >= a.N_total) { bad_s = BAD_BLOCK_ID; p = 0; }
        const size_t roff = ((((size_t)l * a.N_total + p) * a.b + (t - blk * a.b)) * a.h_kv + h) * (size_t)(D * 2) + c * 16;
        float kf[E], vf[E];
        unpack(*(const ck_u32x4 *)(a.k + roff), kf);
        unpack(*(const ck_u32x4 *)(a.v + roff), vf);
#pragma unroll
        for (int g = 0; g < G; g++) {
            float x = 0.f;
#pragma unroll
            for (int e = 0; e < E; e++) x = fmaf(qf[g][e], kf[e], x);
#pragma unroll
            for (int off = 1; off < CPR; off <<= 1) x += __shfl_xor(x, off);   // the lanes of a row are active together
            const float mn = fmaxf(m[g], x), corr = __builtin_amdgcn_exp2f(m[g] - mn), pr = __builtin_amdgcn_exp2f(x - mn);
            ls[g] = ls[g] * corr + pr;
            m[g] = mn;
#pragma unroll
            for (int e = 0; e < E; e++) acc[g][e] = fmaf(pr, vf[e], acc[g][e] * corr);
        }
    }
    // merge the row groups of a wave, then the waves
#pragma unroll
    for (int off = CPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; g++) {
            const float mo = __shfl_xor(m[g], off), lo = __shfl_xor(ls[g], off);
            const float mn = fmaxf(m[g], mo), cs = __builtin_amdgcn_exp2f(m[g] - mn), co = __builtin_amdgcn_exp2f(mo - mn);
            ls[g] = ls[g] * cs + lo * co;
#pragma unroll
            for (int e = 0; e < E; e++) acc[g][e] = acc[g][e] * cs + __shfl_xor(acc[g][e], off) * co;
            m[g] = mn;
        }
    }
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < G; g++) {
            if (c == 0) { s_m[wv][g] = m[g]; s_l[wv][g] = ls[g]; }
#pragma unroll
            for (int e = 0; e < E; e++) s_acc[wv][g][c * E + e] = acc[g][e];
        }
    }
    __syncthreads();
    if (bad_s) {
        if (tid == 0 && atomicCAS(&a.status[0], 0, 1) == 0) { a.status[1] = item; a.status[2] = bad_s; }
        return;
    }
    for (int i = tid; i < G * D; i += 256) {
        const int g = i / D, dim = i - g * D;
        float mm = s_m[0][g];
#pragma unroll
        for (int v = 1; v < NW; v++) mm = fmaxf(mm, s_m[v][g]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int v = 0; v < NW; v++) {
            const float sc = __builtin_amdgcn_exp2f(s_m[v][g] - mm);
            num += s_acc[v][g][dim] * sc;
            den += s_l[v][g] * sc;
        }
        a.out[(q0 + g) * (size_t)D + dim] = len > 0 ? num / den : 0.f;
    }
}

template <int D>
static bool launch_gqa(const DecodeArgs &a, int G, int groups, hipStream_t s) {
    switch (G) {
        case 1: hipLaunchKernelGGL((decode_attention_gqa<1, D>), dim3(groups), dim3(256), 0, s, a); return true;
        case 2: hipLaunchKernelGGL((decode_attention_gqa<2, D>), dim3(groups), dim3(256), 0, s, a); return true;
        case 4: hipLaunchKernelGGL((decode_attention_gqa<4, D>), dim3(groups), dim3(256), 0, s, a); return true;
        case 5: hipLaunchKernelGGL((decode_attention_gqa<5, D>), dim3(groups), dim3(256), 0, s, a); return true;
        case 7: hipLaunchKernelGGL((decode_attention_gqa<7, D>), dim3(groups), dim3(256), 0, s, a); return true;
        case 8: hipLaunchKernelGGL((decode_attention_gqa<8, D>), dim3(groups), dim3(256), 0, s, a); return true;
        default: return false;
    }
}

hipError_t launch_decode_attention(const DecodeArgs &a, int items, hipStream_t s) {
    if (items <= 0) return hipSuccess;
    const int G = a.h_q / a.h_kv, groups = items / G;
    bool done = false;
    if (a.dtype == 1 && a.d == 128) done = launch_gqa<128>(a, G, groups, s);
    else if (a.dtype == 1 && a.d == 64) done = launch_gqa<64>(a, G, groups, s);
    if (!done) {                                                  // any other shape: one workgroup per query head
        if (a.dtype == 0) hipLaunchKernelGGL(decode_attention<0>, dim3(items), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(decode_attention<1>, dim3(items), dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace zp

// Check-only paged decode attention (not part of the compression path): one query per (request, layer,
// query head) attends to the first len[n][l][h] rows of the request's table, h = hq / G.  It exists so that
// a compacted cache with per-head lengths can be verified end to end; plain vector-ALU code, not tuned.
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

hipError_t launch_decode_attention(const DecodeArgs &a, int items, hipStream_t s) {
    if (items <= 0) return hipSuccess;
    if (a.dtype == 0) hipLaunchKernelGGL(decode_attention<0>, dim3(items), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(decode_attention<1>, dim3(items), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace zp

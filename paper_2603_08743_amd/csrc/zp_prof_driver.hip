// Stand-alone driver for hardware-counter runs of the fused compression kernel (no Python, no torch):
//   rocprofv3 --pmc FETCH_SIZE -- ./zp_prof_driver [B] [L_slab] [config] [reps] [stages] [split] [streams] [extras] [xcd_map]
// stages = 1 also times the staged calls (zp_score, zp_select_topk, zp_compact_kv) one by one.
// extras: bit mask of score refinements to time with zp_compress_ex after the plain run (1 global score, 2 max
// pooling with kernel 7, 4 lightning redundancy); every set of bits from 1 up to the mask that is a subset of it is run.
// It builds one layer slab of a benchmark-shaped workload with an on-device integer-hash fill
// (approximately N(0,1) values, 5 % of the key positions scaled x3, shuffled block tables, per-head
// keep counts for config 2), runs a plain copy kernel of known size first (the calibration dispatch
// for the byte counters), then zp_compress through the C ABI, and prints the event-timed duration.
#include "../../include/zp.h"
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <numeric>
#include <random>
#include <vector>

#define CK(x)                                                                                  \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } \
    } while (0)

__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ unsigned short f2bf(float f) {
    unsigned u = __float_as_uint(f);
    return (unsigned short)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// element i <- sum of four 16-bit uniforms, centred and scaled to unit variance; x3 on heavy rows
__global__ void fill_bf16(unsigned short *out, size_t n, unsigned long long seed, int row_elems, int rows_per_layer, int heavy) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const unsigned long long h = mix64(seed ^ (i * 0x9E3779B97F4A7C15ull));
        const int s = (int)(h & 0xffff) + (int)((h >> 16) & 0xffff) + (int)((h >> 32) & 0xffff) + (int)(h >> 48);
        float z = (float)(s - 131070) * (1.0f / 37837.0f);
        if (heavy) {
            const size_t row = (i / row_elems) % rows_per_layer;               // (block, slot): same for every layer and head
            if ((mix64(seed * 31 + row) & 0xffff) < 3277) z *= 3.0f;
        }
        out[i] = f2bf(z);
    }
}

__global__ void plain_copy(const uint4 *src, uint4 *dst, size_t n16) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

int main(int argc, char **argv) {
    const int B = argc > 1 ? atoi(argv[1]) : 256;
    const int Ls = argc > 2 ? atoi(argv[2]) : 8;
    const int cfg = argc > 3 ? atoi(argv[3]) : 2;
    const int reps = argc > 4 ? atoi(argv[4]) : 1;
    const int staged = argc > 5 ? atoi(argv[5]) : 0;
    const int split = argc > 6 ? atoi(argv[6]) : -1;
    const int streams = argc > 7 ? atoi(argv[7]) : 8;
    const int extras = argc > 8 ? atoi(argv[8]) : 0;
    const int xcd_map = argc > 9 ? atoi(argv[9]) : 1;
    int h_kv = 8, h_q = 32, d = 128, b = 16, N_max = 257, w = 64;
    bool per_head_keep = true;
    if (cfg == 1) { h_kv = 4; h_q = 28; N_max = 129; w = 32; per_head_keep = false; }
    if (cfg == 4) { h_q = 40; N_max = 513; w = 128; }
    const int N_total = B * N_max + 64, budget = (N_max - 1) * b;
    const size_t kv_elems = (size_t)Ls * N_total * b * h_kv * d, q_elems = (size_t)Ls * B * w * h_q * d;
    unsigned short *K, *V, *Q, *K0, *V0;
    CK(hipMalloc((void **)&K, kv_elems * 2));
    CK(hipMalloc((void **)&V, kv_elems * 2));
    CK(hipMalloc((void **)&K0, kv_elems * 2));
    CK(hipMalloc((void **)&V0, kv_elems * 2));
    CK(hipMalloc((void **)&Q, q_elems * 2));
    hipLaunchKernelGGL(fill_bf16, dim3(8192), dim3(256), 0, 0, K0, kv_elems, 11ull, h_kv * d, N_total * b, 1);
    hipLaunchKernelGGL(fill_bf16, dim3(8192), dim3(256), 0, 0, V0, kv_elems, 12ull, h_kv * d, N_total * b, 0);
    hipLaunchKernelGGL(fill_bf16, dim3(8192), dim3(256), 0, 0, Q, q_elems, 13ull, h_q * d, 1, 0);
    CK(hipDeviceSynchronize());

    std::mt19937 rng(20260308 + cfg);
    std::vector<int> perm(N_total), tbl((size_t)B * N_max), nb(B, N_max), slot(B), keep((size_t)B * Ls * h_kv, budget);
    std::iota(perm.begin(), perm.end(), 0);
    std::shuffle(perm.begin(), perm.end(), rng);
    std::copy(perm.begin(), perm.begin() + (size_t)B * N_max, tbl.begin());
    std::iota(slot.begin(), slot.end(), 0);
    if (per_head_keep) {
        std::uniform_int_distribution<int> u(budget / 4, budget);
        for (auto &x : keep) x = u(rng);
    }
    int *d_tbl, *d_nb, *d_slot, *d_keep, *d_len;
    CK(hipMalloc((void **)&d_tbl, tbl.size() * 4));
    CK(hipMalloc((void **)&d_nb, nb.size() * 4));
    CK(hipMalloc((void **)&d_slot, slot.size() * 4));
    CK(hipMalloc((void **)&d_keep, keep.size() * 4));
    CK(hipMalloc((void **)&d_len, keep.size() * 4));
    CK(hipMemcpy(d_tbl, tbl.data(), tbl.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_nb, nb.data(), nb.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_slot, slot.data(), slot.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_keep, keep.data(), keep.size() * 4, hipMemcpyHostToDevice));

    zp_ctx *ctx;
    if (zp_create(&ctx) != ZP_OK) { fprintf(stderr, "%s\n", zp_last_error(nullptr)); return 1; }
    zp_set_option(ctx, ZP_OPT_SPLIT, split);
    zp_set_option(ctx, ZP_OPT_STREAMS, streams);
    zp_set_option(ctx, ZP_OPT_XCD_MAP, xcd_map);
    zp_pool pool = {K, V, Q, 0, Ls, N_total, b, h_kv, h_q, d, B, w, ZP_BF16};
    zp_batch batch = {B, N_max, N_max, Ls, d_tbl, nullptr, d_nb, d_slot, nullptr, d_keep};
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const size_t n16 = kv_elems * 2 / 16;
    double total_ms = 0;
    for (int r = 0; r < reps; r++) {
        // calibration + restore: plain copies of kv_elems*2 bytes each (read n, write n)
        hipLaunchKernelGGL(plain_copy, dim3(16384), dim3(256), 0, 0, (const uint4 *)K0, (uint4 *)K, n16);
        hipLaunchKernelGGL(plain_copy, dim3(16384), dim3(256), 0, 0, (const uint4 *)V0, (uint4 *)V, n16);
        CK(hipEventRecord(e0, 0));
        if (zp_compress(ctx, &pool, &batch, d_len, nullptr, nullptr, nullptr) != ZP_OK) { fprintf(stderr, "%s\n", zp_last_error(ctx)); return 1; }
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        total_ms += ms;
    }
    if (zp_sync_status(ctx, nullptr) != ZP_OK) { fprintf(stderr, "%s\n", zp_last_error(ctx)); return 1; }
    if (staged) {
        const size_t units = (size_t)B * Ls * h_kv;
        float *scores;
        int *kidx;
        CK(hipMalloc((void **)&scores, units * N_max * b * 4));
        CK(hipMalloc((void **)&kidx, units * budget * 4));
        float t[3] = {0, 0, 0};
        for (int r = 0; r < reps; r++) {
            hipLaunchKernelGGL(plain_copy, dim3(16384), dim3(256), 0, 0, (const uint4 *)K0, (uint4 *)K, n16);
            hipLaunchKernelGGL(plain_copy, dim3(16384), dim3(256), 0, 0, (const uint4 *)V0, (uint4 *)V, n16);
            for (int st = 0; st < 3; st++) {
                CK(hipEventRecord(e0, 0));
                zp_status rc = st == 0 ? zp_score(ctx, &pool, &batch, scores, nullptr)
                             : st == 1 ? zp_select_topk(ctx, scores, N_max * b, &pool, &batch, kidx, d_len, nullptr)
                                       : zp_compact_kv(ctx, &pool, &batch, kidx, d_len, nullptr);
                if (rc != ZP_OK) { fprintf(stderr, "%s\n", zp_last_error(ctx)); return 1; }
                CK(hipEventRecord(e1, 0));
                CK(hipEventSynchronize(e1));
                float ms;
                CK(hipEventElapsedTime(&ms, e0, e1));
                t[st] += ms;
            }
        }
        printf("staged: zp_score %.3f ms, zp_select_topk %.3f ms, zp_compact_kv %.3f ms per launch\n", t[0] / reps, t[1] / reps, t[2] / reps);
    }
    if (extras) {
        float *F;
        int *comp;
        const size_t f_elems = (size_t)Ls * N_total * b * h_kv;
        CK(hipMalloc((void **)&F, f_elems * 4));
        CK(hipMalloc((void **)&comp, B * 4));
        CK(hipMemset(F, 0, f_elems * 4));
        std::vector<int> hc(B);
        for (int n = 0; n < B; n++) hc[n] = n & 1;                 // every other request has history
        CK(hipMemcpy(comp, hc.data(), B * 4, hipMemcpyHostToDevice));
        for (int m = 1; m <= extras; m++) {
            if ((m & extras) != m) continue;
            zp_extras ex = {(m & 1) ? F : nullptr, comp, 0.8f, (m & 2) ? 7 : 1, (m & 4) ? 0.3f : 0.f, 2e-4f, 0.4f, 0};
            double ms_sum = 0;
            for (int r = 0; r < reps; r++) {
                hipLaunchKernelGGL(plain_copy, dim3(16384), dim3(256), 0, 0, (const uint4 *)K0, (uint4 *)K, n16);
                hipLaunchKernelGGL(plain_copy, dim3(16384), dim3(256), 0, 0, (const uint4 *)V0, (uint4 *)V, n16);
                CK(hipEventRecord(e0, 0));
                if (zp_compress_ex(ctx, &pool, &batch, &ex, d_len, nullptr, nullptr, nullptr) != ZP_OK) { fprintf(stderr, "%s\n", zp_last_error(ctx)); return 1; }
                CK(hipEventRecord(e1, 0));
                CK(hipEventSynchronize(e1));
                float ms;
                CK(hipEventElapsedTime(&ms, e0, e1));
                ms_sum += ms;
            }
            if (zp_sync_status(ctx, nullptr) != ZP_OK) { fprintf(stderr, "%s\n", zp_last_error(ctx)); return 1; }
            printf("zp_compress_ex%s%s%s: %.3f ms/launch\n", (m & 1) ? " +global" : "", (m & 2) ? " +pool7" : "", (m & 4) ? " +redundancy" : "", ms_sum / reps);
        }
    }
    long long kept = 0;
    for (int x : keep) kept += x;
    printf("cfg %d split=%d streams=%d: B=%d L_slab=%d units=%d  zp_compress %.3f ms/launch over %d launch(es); plain_copy moves %zu bytes each way; kept rows %lld\n",
           cfg, split, streams, B, Ls, B * Ls * h_kv, total_ms / reps, reps, kv_elems * 2, kept);
    zp_destroy(ctx);
    return 0;
}

/*
 * The outer step through the C ABI from a plain C program (no Python, no torch):
 * device memory with hipMalloc, inputs from a small integer hash, one outer step
 * with libsparseloco.so, the same step with the CPU oracle (liboracle.so), and a
 * comparison: pairs and levels byte for byte, buffers and parameters as numbers.
 * Built by __graft_entry__.build() into tests/c_abi_check; run by
 * tests/test_gpu_c_abi.py.  Exit status 0 = match.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sparseloco.h"

int oracle_compress(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, float beta, int quant_mode,
                    const float* theta_outer, const float* theta_local, const float* delta_f32,
                    const uint16_t* delta_bf16, float* ef, uint16_t* pairs_out, float* scales_out, float* values_out);
int oracle_aggregate(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, int quant_mode,
                     int n_replicas, const uint16_t* const* pairs, const float* const* scales,
                     const float* const* values, float* delta_bar_out);
int oracle_outer_update(int64_t numel, float* theta_outer, const float* delta_bar, float outer_lr);

#define N_TENSORS 3
#define R 3
#define KAPPA 32
#define HIPCHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define SPLCHECK(x) do { int rc_ = (x); if (rc_ != SPLC_OK) { fprintf(stderr, "%s failed: %s\n", #x, sparseloco_strerror(rc_)); return 3; } } while (0)

static float hash_unit(uint32_t i, uint32_t seed) {          /* in [-1, 1) */
    uint32_t h = i * 2654435761u + seed * 40503u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
    return (float)(h & 0xFFFFFF) / 8388608.0f - 1.0f;
}

static float* to_device(const float* h, size_t n) {
    float* d = NULL;
    if (hipMalloc((void**)&d, n * sizeof(float)) != hipSuccess) return NULL;
    if (hipMemcpy(d, h, n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return d;
}

int main(void) {
    const int64_t numel[N_TENSORS] = {4096 * 7 + 33, 2047, 4096};
    int64_t n_chunks = 0, chunk0[N_TENSORS];
    for (int t = 0; t < N_TENSORS; ++t) { chunk0[t] = n_chunks; n_chunks += (numel[t] + 4095) / 4096; }

    float *h_to[N_TENSORS], *h_tl[R][N_TENSORS], *h_ef[R][N_TENSORS], *h_db[N_TENSORS];
    float *d_to[N_TENSORS], *d_tl[R][N_TENSORS], *d_ef[R][N_TENSORS], *d_db[N_TENSORS];
    for (int t = 0; t < N_TENSORS; ++t) {
        size_t n = (size_t)numel[t];
        h_to[t] = malloc(n * 4); h_db[t] = malloc(n * 4);
        for (size_t i = 0; i < n; ++i) h_to[t][i] = 0.02f * hash_unit((uint32_t)i, 100 + t);
        d_to[t] = to_device(h_to[t], n);
        HIPCHECK(hipMalloc((void**)&d_db[t], n * 4));
        for (int r = 0; r < R; ++r) {
            h_tl[r][t] = malloc(n * 4); h_ef[r][t] = malloc(n * 4);
            for (size_t i = 0; i < n; ++i) {
                float u = hash_unit((uint32_t)i, 1000 * (r + 1) + t);
                h_tl[r][t][i] = h_to[t][i] - 1e-3f * u * u * u * 8.0f;     /* heavy-ish tails */
                h_ef[r][t][i] = 1e-4f * hash_unit((uint32_t)i, 5000 * (r + 1) + t);
            }
            d_tl[r][t] = to_device(h_tl[r][t], n);
            d_ef[r][t] = to_device(h_ef[r][t], n);
            if (!d_to[t] || !d_tl[r][t] || !d_ef[r][t]) { fprintf(stderr, "device allocation failed\n"); return 2; }
        }
    }
    /* GPU path */
    sparseloco_plan* plan = NULL;
    SPLCHECK(sparseloco_plan_create(&plan, N_TENSORS, numel, SPLC_CHUNK, KAPPA, SPLC_QUANT_2BIT, NULL));
    if (sparseloco_plan_num_chunks(plan) != n_chunks) { fprintf(stderr, "chunk count mismatch\n"); return 4; }
    uint16_t* d_pairs[R]; float* d_scales[R];
    for (int r = 0; r < R; ++r) {
        HIPCHECK(hipMalloc((void**)&d_pairs[r], (size_t)n_chunks * KAPPA * 2));
        HIPCHECK(hipMalloc((void**)&d_scales[r], (size_t)n_chunks * 2 * 4));
    }
    /* bind the tensor lists once: the shared parameters and the mean as single sets, the replicas' local
       parameters and error-feedback buffers as R sets each, the R messages */
    sparseloco_tensors *b_to = NULL, *b_db = NULL, *b_tl = NULL, *b_ef = NULL;
    sparseloco_messages* b_msg = NULL;
    SPLCHECK(sparseloco_tensors_bind(&b_to, plan, 1, (const void* const*)d_to, SPLC_F32, NULL));
    SPLCHECK(sparseloco_tensors_bind(&b_db, plan, 1, (const void* const*)d_db, SPLC_F32, NULL));
    SPLCHECK(sparseloco_tensors_bind(&b_tl, plan, R, (const void* const*)&d_tl[0][0], SPLC_F32, NULL));
    SPLCHECK(sparseloco_tensors_bind(&b_ef, plan, R, (const void* const*)&d_ef[0][0], SPLC_F32, NULL));
    SPLCHECK(sparseloco_messages_bind(&b_msg, plan, R, d_pairs, d_scales, NULL));
    for (int r = 0; r < R; ++r)
        SPLCHECK(sparseloco_compress(plan, SPLC_DELTA_FROM_PARAMS, b_to, b_tl, b_ef, r, 0.95f, d_pairs[r], d_scales[r],
                                     NULL));
    SPLCHECK(sparseloco_aggregate(plan, b_msg, b_db, NULL));
    SPLCHECK(sparseloco_outer_update(plan, b_to, b_db, 1.0f, NULL));
    HIPCHECK(hipDeviceSynchronize());

    /* oracle */
    uint16_t* o_pairs[R]; float* o_scales[R];
    for (int r = 0; r < R; ++r) {
        o_pairs[r] = malloc((size_t)n_chunks * KAPPA * 2);
        o_scales[r] = malloc((size_t)n_chunks * 2 * 4);
        for (int t = 0; t < N_TENSORS; ++t)
            if (oracle_compress(1, numel[t], 4096, 0, KAPPA, 0.95f, 1, h_to[t], h_tl[r][t], NULL, NULL, h_ef[r][t],
                                o_pairs[r] + chunk0[t] * KAPPA, o_scales[r] + chunk0[t] * 2, NULL) != 0) return 5;
    }
    for (int t = 0; t < N_TENSORS; ++t) {
        const uint16_t* pp[R]; const float* ss[R];
        for (int r = 0; r < R; ++r) { pp[r] = o_pairs[r] + chunk0[t] * KAPPA; ss[r] = o_scales[r] + chunk0[t] * 2; }
        if (oracle_aggregate(1, numel[t], 4096, 0, KAPPA, 1, R, pp, ss, NULL, h_db[t]) != 0) return 5;
        if (oracle_outer_update(numel[t], h_to[t], h_db[t], 1.0f) != 0) return 5;
    }

    /* compare */
    long bad = 0;
    for (int r = 0; r < R; ++r) {
        size_t np = (size_t)n_chunks * KAPPA, ns = (size_t)n_chunks * 2;
        uint16_t* g = malloc(np * 2); float* s = malloc(ns * 4);
        HIPCHECK(hipMemcpy(g, d_pairs[r], np * 2, hipMemcpyDeviceToHost));
        HIPCHECK(hipMemcpy(s, d_scales[r], ns * 4, hipMemcpyDeviceToHost));
        if (memcmp(g, o_pairs[r], np * 2) != 0) { fprintf(stderr, "replica %d: pairs differ\n", r); ++bad; }
        if (memcmp(s, o_scales[r], ns * 4) != 0) { fprintf(stderr, "replica %d: levels differ\n", r); ++bad; }
        for (int t = 0; t < N_TENSORS; ++t) {
            float* e = malloc((size_t)numel[t] * 4);
            HIPCHECK(hipMemcpy(e, d_ef[r][t], (size_t)numel[t] * 4, hipMemcpyDeviceToHost));
            for (int64_t i = 0; i < numel[t]; ++i) if (e[i] != h_ef[r][t][i]) ++bad;
            free(e);
        }
        free(g); free(s);
    }
    for (int t = 0; t < N_TENSORS; ++t) {
        float* a = malloc((size_t)numel[t] * 4); float* b = malloc((size_t)numel[t] * 4);
        HIPCHECK(hipMemcpy(a, d_db[t], (size_t)numel[t] * 4, hipMemcpyDeviceToHost));
        HIPCHECK(hipMemcpy(b, d_to[t], (size_t)numel[t] * 4, hipMemcpyDeviceToHost));
        for (int64_t i = 0; i < numel[t]; ++i) { if (a[i] != h_db[t][i]) ++bad; if (b[i] != h_to[t][i]) ++bad; }
        free(a); free(b);
    }
    sparseloco_messages_release(b_msg);
    sparseloco_tensors_release(b_to); sparseloco_tensors_release(b_db);
    sparseloco_tensors_release(b_tl); sparseloco_tensors_release(b_ef);
    sparseloco_plan_destroy(plan);
    if (bad) { fprintf(stderr, "%ld mismatches\n", bad); return 1; }
    printf("c_abi_check: %d tensors, %lld chunks, %d replicas: GPU library and oracle agree\n", N_TENSORS,
           (long long)n_chunks, R);
    return 0;
}

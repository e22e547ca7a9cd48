// Streaming probes: the access patterns of the outer-step kernels with none of their arithmetic, same launch
// shape (one 256-lane workgroup per 4096 floats, lane t of slot s touches floats s * 1024 + 4 t .. + 3, 16-byte
// non-temporal accesses).  They measure what the chip streams for each mix of reads and writes -- the practical
// ceiling beside which the kernels' achieved bandwidths are read.  Not part of the method.
// The shaped entry point varies what a kernel is free to choose -- how much of each array a workgroup covers,
// which XCD takes which chunks, how many workgroups share a compute unit -- to show what those choices are worth.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparseloco.h"

namespace {

typedef float vfloat4 __attribute__((ext_vector_type(4)));
#define SPLC_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ vfloat4 ld(const float* p) { return __builtin_nontemporal_load((const SPLC_GLOBAL vfloat4*)p); }
__device__ __forceinline__ void st(float* p, vfloat4 v) { __builtin_nontemporal_store(v, (SPLC_GLOBAL vfloat4*)p); }

// SLOTS 16-byte accesses per lane and array (a workgroup covers SLOTS * 4 KB of each array).
// run > 0: the chunk a workgroup takes is dealt out so that every XCD (workgroups go to the eight XCDs round-robin
// by number) walks runs of `run` consecutive chunks instead of every eighth chunk.
template <int PATTERN, int SLOTS>
__global__ __launch_bounds__(256) void stream_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                     float* __restrict__ c, float* __restrict__ sink, uint32_t run) {
    uint32_t chunk = blockIdx.x;
    if (run > 0) {
        const uint32_t xcd = chunk & 7u, q = chunk >> 3;
        chunk = ((q / run) * 8u + xcd) * run + q % run;
    }
    const size_t base = (size_t)chunk * (1024 * SLOTS) + (size_t)threadIdx.x * 4;
    vfloat4 va[SLOTS], vb[SLOTS], vc[SLOTS];
    if (PATTERN != SPLC_STREAM_WRITE) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) va[s] = ld(a + base + s * 1024);
    }
    if (PATTERN == SPLC_STREAM_R3W1) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) vb[s] = ld(b + base + s * 1024);
    }
    if (PATTERN == SPLC_STREAM_R2W1 || PATTERN == SPLC_STREAM_R3W1) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) vc[s] = ld(c + base + s * 1024);
    }
    if (PATTERN == SPLC_STREAM_READ) {
        vfloat4 sum = va[0];
#pragma unroll
        for (int s = 1; s < SLOTS; ++s) sum += va[s];
        if (sum.x + sum.y + sum.z + sum.w == 123.456f) sink[0] = sum.x;      // practically never true
        return;
    }
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        vfloat4 v;
        if (PATTERN == SPLC_STREAM_WRITE) v = vfloat4{1.f, 2.f, 3.f, 4.f};
        else if (PATTERN == SPLC_STREAM_COPY) v = va[s];
        else if (PATTERN == SPLC_STREAM_R2W1) v = vc[s] - va[s];
        else v = (va[s] - vb[s]) + vc[s];
        st(c + base + s * 1024, v);
    }
}

constexpr size_t kLdsPerUnit = 160 * 1024;      // LDS of one compute unit

template <int PATTERN, int SLOTS>
int launch(const float* a, const float* b, float* c, float* sink, int64_t n, uint32_t run, int max_groups,
           hipStream_t stream) {
    // A dynamic LDS reservation nobody touches caps the workgroups resident on a compute unit.
    size_t lds = 0;
    if (max_groups > 0) {
        lds = (kLdsPerUnit / (size_t)max_groups) & ~(size_t)1023;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_kernel<PATTERN, SLOTS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerUnit) != hipSuccess)
            return SPLC_EHIP;
    }
    hipLaunchKernelGGL((stream_kernel<PATTERN, SLOTS>), dim3((unsigned)(n / (1024 * SLOTS))), dim3(256), lds, stream, a, b,
                       c, sink, run);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

template <int SLOTS>
int launch_pattern(int pattern, const float* a, const float* b, float* c, float* sink, int64_t n, uint32_t run,
                   int max_groups, hipStream_t st_) {
    switch (pattern) {
        case SPLC_STREAM_READ: return launch<SPLC_STREAM_READ, SLOTS>(a, b, c, sink, n, run, max_groups, st_);
        case SPLC_STREAM_WRITE: return launch<SPLC_STREAM_WRITE, SLOTS>(a, b, c, sink, n, run, max_groups, st_);
        case SPLC_STREAM_COPY: return launch<SPLC_STREAM_COPY, SLOTS>(a, b, c, sink, n, run, max_groups, st_);
        case SPLC_STREAM_R2W1: return launch<SPLC_STREAM_R2W1, SLOTS>(a, b, c, sink, n, run, max_groups, st_);
        default: return launch<SPLC_STREAM_R3W1, SLOTS>(a, b, c, sink, n, run, max_groups, st_);
    }
}

}  // namespace

extern "C" int sparseloco_stream_probe_shaped(int pattern, const float* a, const float* b, float* c, float* sink,
                                              int64_t n, int slots, int run, int max_groups_per_unit, void* stream) {
    if (n < 0 || n % 4096 != 0 || n / 1024 > 0x7FFFFFFF) return SPLC_EINVAL;
    if (slots != 1 && slots != 4) return SPLC_EINVAL;
    if (run < 0 || run > 65536 || max_groups_per_unit < 0 || max_groups_per_unit > 8) return SPLC_EINVAL;
    if (run > 0 && (n / (1024 * slots)) % (8 * (int64_t)run) != 0) return SPLC_EINVAL;     // whole runs on every XCD
    const bool need_a = pattern != SPLC_STREAM_WRITE, need_b = pattern == SPLC_STREAM_R3W1,
               need_c = pattern != SPLC_STREAM_READ;
    if (pattern < SPLC_STREAM_READ || pattern > SPLC_STREAM_R3W1) return SPLC_EINVAL;
    if ((need_a && !a) || (need_b && !b) || (need_c && !c) || (pattern == SPLC_STREAM_READ && !sink)) return SPLC_EINVAL;
    for (const void* p : {(const void*)a, (const void*)b, (const void*)c})
        if (reinterpret_cast<uintptr_t>(p) & 15) return SPLC_EALIGN;
    if (n == 0) return SPLC_OK;
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    return slots == 4 ? launch_pattern<4>(pattern, a, b, c, sink, n, (uint32_t)run, max_groups_per_unit, st_)
                      : launch_pattern<1>(pattern, a, b, c, sink, n, (uint32_t)run, max_groups_per_unit, st_);
}

extern "C" int sparseloco_stream_probe(int pattern, const float* a, const float* b, float* c, float* sink, int64_t n,
                                       void* stream) {
    return sparseloco_stream_probe_shaped(pattern, a, b, c, sink, n, 4, 0, 0, stream);
}

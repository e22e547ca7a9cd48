// Streaming probes: the access patterns of the outer-step kernels with none of their arithmetic, same launch
// shape (one 256-lane workgroup per 4096 floats, lane t of slot s touches floats s * 1024 + 4 t .. + 3, 16-byte
// non-temporal accesses).  They measure what the chip streams for each mix of reads and writes -- the practical
// ceiling beside which the kernels' achieved bandwidths are read.  Not part of the method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparseloco.h"

namespace {

typedef float vfloat4 __attribute__((ext_vector_type(4)));
#define SPLC_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ vfloat4 ld(const float* p) { return __builtin_nontemporal_load((const SPLC_GLOBAL vfloat4*)p); }
__device__ __forceinline__ void st(float* p, vfloat4 v) { __builtin_nontemporal_store(v, (SPLC_GLOBAL vfloat4*)p); }

template <int PATTERN>
__global__ __launch_bounds__(256) void stream_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                     float* __restrict__ c, float* __restrict__ sink) {
    const size_t base = (size_t)blockIdx.x * 4096 + (size_t)threadIdx.x * 4;
    vfloat4 va[4], vb[4], vc[4];
    if (PATTERN != SPLC_STREAM_WRITE) {
#pragma unroll
        for (int s = 0; s < 4; ++s) va[s] = ld(a + base + s * 1024);
    }
    if (PATTERN == SPLC_STREAM_R3W1) {
#pragma unroll
        for (int s = 0; s < 4; ++s) vb[s] = ld(b + base + s * 1024);
    }
    if (PATTERN == SPLC_STREAM_R2W1 || PATTERN == SPLC_STREAM_R3W1) {
#pragma unroll
        for (int s = 0; s < 4; ++s) vc[s] = ld(c + base + s * 1024);
    }
    if (PATTERN == SPLC_STREAM_READ) {
        vfloat4 sum = va[0] + va[1] + va[2] + va[3];
        if (sum.x + sum.y + sum.z + sum.w == 123.456f) sink[0] = sum.x;      // practically never true
        return;
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        vfloat4 v;
        if (PATTERN == SPLC_STREAM_WRITE) v = vfloat4{1.f, 2.f, 3.f, 4.f};
        else if (PATTERN == SPLC_STREAM_COPY) v = va[s];
        else if (PATTERN == SPLC_STREAM_R2W1) v = vc[s] - va[s];
        else v = (va[s] - vb[s]) + vc[s];
        st(c + base + s * 1024, v);
    }
}

}  // namespace

extern "C" int sparseloco_stream_probe(int pattern, const float* a, const float* b, float* c, float* sink, int64_t n,
                                       void* stream) {
    if (n < 0 || n % 4096 != 0 || n / 4096 > 0x7FFFFFFF) return SPLC_EINVAL;
    const bool need_a = pattern != SPLC_STREAM_WRITE, need_b = pattern == SPLC_STREAM_R3W1,
               need_c = pattern != SPLC_STREAM_READ;
    if (pattern < SPLC_STREAM_READ || pattern > SPLC_STREAM_R3W1) return SPLC_EINVAL;
    if ((need_a && !a) || (need_b && !b) || (need_c && !c) || (pattern == SPLC_STREAM_READ && !sink)) return SPLC_EINVAL;
    for (const void* p : {(const void*)a, (const void*)b, (const void*)c})
        if (reinterpret_cast<uintptr_t>(p) & 15) return SPLC_EALIGN;
    if (n == 0) return SPLC_OK;
    const dim3 grid((unsigned)(n / 4096)), block(256);
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    switch (pattern) {
        case SPLC_STREAM_READ: hipLaunchKernelGGL(stream_kernel<SPLC_STREAM_READ>, grid, block, 0, st_, a, b, c, sink); break;
        case SPLC_STREAM_WRITE: hipLaunchKernelGGL(stream_kernel<SPLC_STREAM_WRITE>, grid, block, 0, st_, a, b, c, sink); break;
        case SPLC_STREAM_COPY: hipLaunchKernelGGL(stream_kernel<SPLC_STREAM_COPY>, grid, block, 0, st_, a, b, c, sink); break;
        case SPLC_STREAM_R2W1: hipLaunchKernelGGL(stream_kernel<SPLC_STREAM_R2W1>, grid, block, 0, st_, a, b, c, sink); break;
        default: hipLaunchKernelGGL(stream_kernel<SPLC_STREAM_R3W1>, grid, block, 0, st_, a, b, c, sink); break;
    }
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

// SparseLoCo outer step for gfx950 (MI355X): kernels and C ABI.
//
// The entry points follow the update equations of section 2.1 of the paper:
// compress (pseudo-gradient, error-feedback fold, chunk Top-kappa, Q, residual;
// per replica, or for all replicas of a single-node simulation at once),
// aggregate (mean over replicas), outer_update (outer SGD), and aggregate_update
// (the last two in one pass).  Nothing here is a dense contraction, so no matrix
// cores are used: the kernels stream 16-byte-per-lane non-temporal accesses, keep
// each 4096-element chunk in registers (16 values per lane, 256 lanes) and use
// LDS only for the small hand-offs of the selection and for the dense
// accumulator of the mean.
//
// Element layout of a chunk inside a workgroup: lane `tid` holds, for slot
// s = 0..3 and j = 0..3, local index  s*1024 + tid*4 + j  (one float4 per slot).
// A chunk is addressed as 64 local rows of 64 elements: local index idx sits at
// element  offset + (idx >> 6) * stride + (idx & 63)  of its tensor.  A flat chunk
// has stride 64 (every load instruction of the workgroup then covers 4 KiB
// contiguous); a 64 x 64 tile of a matrix has stride = number of columns (256-byte
// row segments).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <new>
#include <type_traits>
#include <vector>

#include "sparseloco.h"

namespace {

constexpr int kChunk = SPLC_CHUNK;
constexpr int kThreads = 256;            // one workgroup per chunk
constexpr int kCandCap = 256;            // candidates the exact ranking handles (one per lane)
constexpr int kFilterKappaMax = 256;     // the candidate filter needs kappa <= number of lanes

struct ChunkDesc {
    uint32_t tensor;                     // index into the pointer tables
    uint32_t n_c;                        // elements in this chunk (kChunk unless it is an edge chunk)
    uint64_t offset;                     // element offset of local index 0 inside its tensor
    uint32_t stride;                     // elements between local rows: 64 (flat) or the matrix's columns (tile)
    uint8_t h;                           // local rows present (1..64)
    uint8_t w;                           // width of every row but the last
    uint8_t last_w;                      // width of the last row (flat tail), = w for a tile
    uint8_t vec;                         // 4-element vector accesses apply: bit 0 for fp32 arrays (all 4096
                                         // elements present), bit 1 for bf16 arrays (also every row start even)
    uint32_t id;                         // chunk number (position of its message in pairs / scales / values)
    uint32_t reserved;
};
static_assert(sizeof(ChunkDesc) == 32, "chunk table entries are 32 bytes");

// Local index -> present in the chunk?
__device__ __forceinline__ bool present(const ChunkDesc& d, uint32_t idx) {
    const uint32_t lr = idx >> 6, lc = idx & 63u;
    return lr + 1 < d.h ? lc < d.w : (lr + 1 == d.h && lc < d.last_w);
}
// Local index -> element offset from the chunk's origin.
__device__ __forceinline__ uint32_t elem_of(const ChunkDesc& d, uint32_t idx) {
    return (idx >> 6) * d.stride + (idx & 63u);
}
// Address of lane tid's 4-element vector in slot s (local rows 16 s + tid / 16, columns 4 (tid % 16)...).
// The slot part is uniform and stays in scalar registers; the per-lane part is one 32-bit byte
// offset shared by all slots and arrays (a chunk spans less than 4 GiB: stride < 2^24).
template <class T>
__device__ __forceinline__ T* vec_at(T* origin, const ChunkDesc& d, int tid, int s) {
    const uint32_t lane_bytes = ((uint32_t)(tid >> 4) * d.stride + (uint32_t)(tid & 15) * 4u) * (uint32_t)sizeof(T);
    const uint64_t slot_bytes = (uint64_t)((uint32_t)s * 16u * d.stride) * sizeof(T);
    using Byte = typename std::conditional<std::is_const<T>::value, const char, char>::type;
    return reinterpret_cast<T*>(reinterpret_cast<Byte*>(origin) + slot_bytes + lane_bytes);
}
// Bit el of the result: element el of lane tid is present.
__device__ __forceinline__ uint32_t present_mask(const ChunkDesc& d, int tid) {
    if (d.n_c == (uint32_t)kChunk) return 0xFFFFu;
    uint32_t m = 0;
#pragma unroll
    for (int el = 0; el < 16; ++el)
        m |= present(d, (uint32_t)((el >> 2) * 1024 + tid * 4 + (el & 3))) ? (1u << el) : 0u;
    return m;
}

enum { MODE_PARAMS_F32 = 0, MODE_DIRECT_F32 = 1, MODE_DIRECT_BF16 = 2 };

// Streaming accesses: every dense array is touched exactly once per launch, so loads and stores
// carry the non-temporal hint (measured on MI355X: 3 reads + 1 write streams at ~6.0 TB/s with
// the hint against ~5.6 TB/s without).
// The vector types promise only 4-byte alignment: rows of a tile start at any multiple of 4 bytes,
// and global memory accepts dword-aligned multi-dword accesses.
typedef float vfloat4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t vuint2 __attribute__((ext_vector_type(2), aligned(4)));

// Every tensor lives in global memory; saying so lets the compiler emit global_ instead of flat_
// instructions.
#define SPLC_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ float4 stream_load4(const float* p) {
    vfloat4 v = __builtin_nontemporal_load((const SPLC_GLOBAL vfloat4*)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 stream_load4(const uint16_t* p) {       // four bf16
    vuint2 v = __builtin_nontemporal_load((const SPLC_GLOBAL vuint2*)p);
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void stream_store4(float* p, float4 v) {
    vfloat4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (SPLC_GLOBAL vfloat4*)p);
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        uint32_t other = (uint32_t)__shfl_xor((int)v, o);
        v = other > v ? other : v;
    }
    return v;
}

// e' = fl(fl(beta * e) + delta), delta = fl(theta_outer - theta_local) or given (section 2.1, lines 1-2).
__device__ __forceinline__ float fold(float beta, float e, float delta) {
    return __fadd_rn(__fmul_rn(beta, e), delta);
}

template <int MODE>
__device__ __forceinline__ void load_fold_full(const void* __restrict__ a, const void* __restrict__ b,
                                               const float* __restrict__ e, const ChunkDesc& d, int tid,
                                               float beta, float (&x)[16]) {
    const float* pe = e + d.offset;
    float4 ev[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) ev[s] = stream_load4(vec_at(pe, d, tid, s));
    if (MODE == MODE_PARAMS_F32) {
        const float* po = static_cast<const float*>(a) + d.offset;
        const float* pl = static_cast<const float*>(b) + d.offset;
        float4 ov[4], lv[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) ov[s] = stream_load4(vec_at(po, d, tid, s));
#pragma unroll
        for (int s = 0; s < 4; ++s) lv[s] = stream_load4(vec_at(pl, d, tid, s));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            x[4 * s + 0] = fold(beta, ev[s].x, __fsub_rn(ov[s].x, lv[s].x));
            x[4 * s + 1] = fold(beta, ev[s].y, __fsub_rn(ov[s].y, lv[s].y));
            x[4 * s + 2] = fold(beta, ev[s].z, __fsub_rn(ov[s].z, lv[s].z));
            x[4 * s + 3] = fold(beta, ev[s].w, __fsub_rn(ov[s].w, lv[s].w));
        }
    } else if (MODE == MODE_DIRECT_F32) {
        const float* pd = static_cast<const float*>(a) + d.offset;
        float4 dv[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) dv[s] = stream_load4(vec_at(pd, d, tid, s));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            x[4 * s + 0] = fold(beta, ev[s].x, dv[s].x);
            x[4 * s + 1] = fold(beta, ev[s].y, dv[s].y);
            x[4 * s + 2] = fold(beta, ev[s].z, dv[s].z);
            x[4 * s + 3] = fold(beta, ev[s].w, dv[s].w);
        }
    } else {
        // bf16 -> fp32 is the exact widening: the 16 bits become the upper half of the word
        const uint16_t* pd = static_cast<const uint16_t*>(a) + d.offset;
        uint2 dv[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) dv[s] = stream_load4(vec_at(pd, d, tid, s));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            x[4 * s + 0] = fold(beta, ev[s].x, __uint_as_float(dv[s].x << 16));
            x[4 * s + 1] = fold(beta, ev[s].y, __uint_as_float(dv[s].x & 0xFFFF0000u));
            x[4 * s + 2] = fold(beta, ev[s].z, __uint_as_float(dv[s].y << 16));
            x[4 * s + 3] = fold(beta, ev[s].w, __uint_as_float(dv[s].y & 0xFFFF0000u));
        }
    }
}

// Edge chunks and rows that do not allow vector accesses: element by element, absent elements = +0.
template <int MODE>
__device__ __forceinline__ void load_fold_scalar(const void* __restrict__ a, const void* __restrict__ b,
                                                 const float* __restrict__ e, const ChunkDesc& d, int tid,
                                                 float beta, uint32_t pmask, float (&x)[16]) {
#pragma unroll
    for (int el = 0; el < 16; ++el) {
        const uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
        float v = 0.f;
        if (pmask & (1u << el)) {
            const uint64_t at = d.offset + elem_of(d, idx);
            float dl;
            if (MODE == MODE_PARAMS_F32)
                dl = __fsub_rn(static_cast<const float*>(a)[at], static_cast<const float*>(b)[at]);
            else if (MODE == MODE_DIRECT_F32)
                dl = static_cast<const float*>(a)[at];
            else
                dl = __uint_as_float((uint32_t) static_cast<const uint16_t*>(a)[at] << 16);
            v = fold(beta, e[at], dl);
        }
        x[el] = v;
    }
}

// Shared state of one chunk's selection.
struct SelectShared {
    uint64_t cand[kCandCap + 2];         // (key << 12 | 4095 - idx) of the candidates, zero padded
    uint32_t hist[256];                  // radix select digit histogram
    uint32_t bucket[16];                 // selected entries per 256-element bucket (bucket = idx >> 8)
    uint32_t t0[4];                      // per-wave lower bounds of the threshold
    uint32_t wmax[4];                    // per-wave maxima of the keys (largest selected magnitude)
    uint64_t thr;                        // composite of the kappa_c-th entry in (key desc, idx asc) order
    uint32_t ncand;
    uint32_t digit;
    uint32_t need;
};

// Exact kappa_c-th largest composite by most-significant-digit radix select over
// the 43-bit composites (31 key bits, 12 inverted index bits).  Composites of
// present elements are distinct, so the result identifies one element: the last
// one kept.  Works for any set of present elements (bit el of pmask = element el of this lane is
// present), any kappa_c in 1..n_c, any tie pattern.
__device__ void radix_select(SelectShared& sh, const float (&x)[16], int tid, uint32_t pmask, uint32_t kappa_c) {
    const int lane = tid & 63;
    const int wave = tid >> 6;
    uint64_t prefix = 0;
    uint32_t need = kappa_c;
    int hi_bit = 43;
    // The filter path may already have published counts for this chunk (when another group of the workgroup
    // forced the general path): start from zero.  The first barrier of the loop below orders this.
    if (tid < 16) sh.bucket[tid] = 0;
    if (tid < 4) sh.wmax[tid] = 0;
#pragma unroll 1
    for (int pass = 0; pass < 6; ++pass) {
        const int width = pass < 5 ? 8 : 3;
        const int shift = hi_bit - width;
        sh.hist[tid] = 0;
        __syncthreads();
#pragma unroll
        for (int el = 0; el < 16; ++el) {
            uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
            // The composite is rebuilt in every pass: kept across the passes, the sixteen 64-bit values
            // of this rarely taken path would set the register count of the whole kernel.
            uint32_t bits = __float_as_uint(x[el]);
            asm volatile("" : "+v"(bits));
            uint64_t comp = ((uint64_t)(bits & 0x7FFFFFFFu) << 12) | (uint64_t)(4095u - idx);
            if ((pmask & (1u << el)) && (comp >> hi_bit) == prefix)
                atomicAdd(&sh.hist[(uint32_t)(comp >> shift) & ((1u << width) - 1u)], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane owns bins 4*lane .. 4*lane+3; find the bin where the count from the top reaches `need`
            uint32_t h0 = sh.hist[4 * lane], h1 = sh.hist[4 * lane + 1], h2 = sh.hist[4 * lane + 2],
                     h3 = sh.hist[4 * lane + 3];
            uint32_t own = h0 + h1 + h2 + h3;
            uint32_t suffix = own;               // inclusive sum over lanes >= this one
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t v = (uint32_t)__shfl_down((int)suffix, o);
                if (lane + o < 64) suffix += v;
            }
            uint32_t above = suffix - own;
            if (above < need && need <= suffix) {
                uint32_t bin;
                if (above + h3 >= need) bin = 3;
                else { above += h3;
                    if (above + h2 >= need) bin = 2;
                    else { above += h2;
                        if (above + h1 >= need) bin = 1;
                        else { above += h1; bin = 0; } } }
                sh.digit = 4 * lane + bin;
                sh.need = need - above;
            }
        }
        __syncthreads();
        prefix = (prefix << width) | (uint64_t)sh.digit;
        need = sh.need;
        hi_bit = shift;
    }
    // publish the threshold, the largest key and the selected count of every 256-element bucket
    uint32_t tmax = 0;
#pragma unroll
    for (int el = 0; el < 16; ++el) {
        uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
        uint32_t key = __float_as_uint(x[el]) & 0x7FFFFFFFu;
        uint64_t comp = ((uint64_t)key << 12) | (uint64_t)(4095u - idx);
        if (pmask & (1u << el)) {
            tmax = key > tmax ? key : tmax;
            if (comp >= prefix) atomicAdd(&sh.bucket[idx >> 8], 1u);
        }
    }
    tmax = wave_max_u32(tmax);
    if (lane == 0) sh.wmax[wave] = tmax;
    if (tid == 0) sh.thr = prefix;
    __syncthreads();
}

// Top-kappa selection of the chunk held in x[16] (already folded): finds the composite of the last kept entry
// in (key descending, index ascending) order and publishes it in sh.thr, with the largest key (sh.wmax) and the
// number of kept entries per 256-element bucket (sh.bucket).  Only the magnitudes of x are used, and only at the
// start: a caller that can fetch its values again afterwards need not keep them in registers meanwhile.
// All 256 lanes (of the group) must call it; it ends behind a workgroup barrier.
// group_ok: four flags in LDS when four 256-lane groups of one workgroup each select a chunk of their own side
// by side (tid, lane, wave are then group-local and `sh` is the group's own).  Workgroup barriers must be
// reached by all groups alike, so the groups agree on the path: if one needs the radix select, all take it.
// lds_chunk: if not null, the chunk sits in LDS in local index order and is read from there (x is ignored): once
// for the keys, and again by the (rare) radix select, so that nothing but the keys stays in registers.
__device__ __forceinline__ void find_threshold(SelectShared& sh, const float (&x)[16], int tid, int lane, int wave,
                                               uint32_t kappa_c, uint32_t kappa, uint32_t pmask, int force_radix,
                                               uint32_t* radix_counter, const float* lds_chunk = nullptr,
                                               uint32_t* group_ok = nullptr, int group = 0) {
    sh.cand[tid] = 0;
    if (tid < 2) sh.cand[kCandCap + tid] = 0;
    if (tid < 16) sh.bucket[tid] = 0;
    if (tid < 4) sh.wmax[tid] = 0;
    if (tid == 0) sh.ncand = 0;

    bool selected_by_filter = false;
    if (kappa <= (uint32_t)kFilterKappaMax && !force_radix) {
        // ---- candidate filter: a lower bound T0 of the threshold from the lane maxima ----
        uint32_t key[16];
        if (lds_chunk) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float4 v = *reinterpret_cast<const float4*>(lds_chunk + s * 1024 + tid * 4);
                key[4 * s] = __float_as_uint(v.x) & 0x7FFFFFFFu;
                key[4 * s + 1] = __float_as_uint(v.y) & 0x7FFFFFFFu;
                key[4 * s + 2] = __float_as_uint(v.z) & 0x7FFFFFFFu;
                key[4 * s + 3] = __float_as_uint(v.w) & 0x7FFFFFFFu;
            }
        } else {
#pragma unroll
            for (int el = 0; el < 16; ++el) key[el] = __float_as_uint(x[el]) & 0x7FFFFFFFu;
        }
        uint32_t tmax = 0;
#pragma unroll
        for (int el = 0; el < 16; ++el) tmax = ((pmask >> el) & 1u) && key[el] > tmax ? key[el] : tmax;
        // Largest X (low 10 bits zero) with at least m lanes of this wave that hold a present element
        // >= X.  Those elements are distinct, so over four waves at least 4*m >= kappa_c elements are
        // >= min X: the threshold cannot be below it.  A wave with fewer than m non-empty lanes (edge
        // chunks) leaves X = 0, which makes every present element a candidate.
        const uint32_t m = (kappa_c + 3) >> 2;
        uint32_t X = 0;
#pragma unroll
        for (int b = 30; b >= 10; --b) {
            uint32_t t = X | (1u << b);
            uint32_t cnt = (uint32_t)__popcll(__ballot(pmask != 0 && tmax >= t));
            X = cnt >= m ? t : X;
        }
        if (lane == 0) sh.t0[wave] = X;
        __syncthreads();
        uint32_t T0 = sh.t0[0];
        T0 = sh.t0[1] < T0 ? sh.t0[1] : T0;
        T0 = sh.t0[2] < T0 ? sh.t0[2] : T0;
        T0 = sh.t0[3] < T0 ? sh.t0[3] : T0;

        // ---- compact the candidates (present, key >= T0) into LDS, wave by wave ----
        uint64_t msk[16];
        uint32_t cnt = 0;
#pragma unroll
        for (int el = 0; el < 16; ++el) {
            msk[el] = __ballot(((pmask >> el) & 1u) && key[el] >= T0);
            cnt += (uint32_t)__popcll(msk[el]);
        }
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&sh.ncand, cnt);
        base = __builtin_amdgcn_readfirstlane(base);
        if (base + cnt <= (uint32_t)kCandCap) {
            uint32_t run = base;
#pragma unroll
            for (int el = 0; el < 16; ++el) {
                if (msk[el] != 0) {
                    if (((pmask >> el) & 1u) && key[el] >= T0) {
                        uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
                        sh.cand[run + lanes_below(msk[el])] = ((uint64_t)key[el] << 12) | (uint64_t)(4095u - idx);
                    }
                    run += (uint32_t)__popcll(msk[el]);
                }
            }
        }
        __syncthreads();
        const uint32_t n = sh.ncand;
        if (n <= (uint32_t)kCandCap) {
            // ---- exact rank of every candidate among the candidates (composites are distinct) ----
            if ((uint32_t)tid < n) {
                const uint64_t mine = sh.cand[tid];
                uint32_t rank = 0;
                for (uint32_t i = 0; i < n; i += 2) {
                    uint64_t c0 = sh.cand[i], c1 = sh.cand[i + 1];
                    rank += (c0 > mine ? 1u : 0u) + (c1 > mine ? 1u : 0u);
                }
                if (rank == kappa_c - 1) sh.thr = mine;
                if (rank == 0) sh.wmax[0] = (uint32_t)(mine >> 12);
                if (rank < kappa_c) atomicAdd(&sh.bucket[(4095u - ((uint32_t)mine & 4095u)) >> 8], 1u);
            }
            selected_by_filter = true;
        }
    }
    if (group_ok) {
        if (tid == 0) group_ok[group] = selected_by_filter ? 1u : 0u;
        __syncthreads();
        selected_by_filter = (group_ok[0] & group_ok[1] & group_ok[2] & group_ok[3]) != 0;
    } else {
        __syncthreads();
    }
    if (!selected_by_filter) {
        if (lds_chunk) {
            // (the index is made opaque so that these reads are not merged with the caller's earlier ones, which
            // would keep all sixteen values in registers from there to here)
            int t = tid;
            asm volatile("" : "+v"(t));
            float y[16];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float4 v = *reinterpret_cast<const float4*>(lds_chunk + s * 1024 + t * 4);
                y[4 * s] = v.x; y[4 * s + 1] = v.y; y[4 * s + 2] = v.z; y[4 * s + 3] = v.w;
            }
            radix_select(sh, y, tid, pmask, kappa_c);
        } else {
            radix_select(sh, x, tid, pmask, kappa_c);
        }
        if (radix_counter && tid == 0) atomicAdd(radix_counter, 1u);      // diagnostic: chunks on the general path
    }
}

// Quantiser, packing and residual of the chunk held in x[16], given the threshold that find_threshold published
// in `sh`.  On return x holds the new error-feedback values; the chunk's pairs, its levels (or sent values) and
// its padding have been written.  It ends with every lane past its last read of `sh`, but callers that reuse
// `sh` must place a barrier first.
// With SUM, every sent value is also added to sum[index in the chunk] (LDS; an element is only ever touched by
// the lane that holds it, so replicas that follow each other in one workgroup need no synchronisation for it).
template <int QUANT, bool SUM>
__device__ __forceinline__ void quantise_pack_sum(const SelectShared& sh, float (&x)[16], float* sum, int tid,
                                                  int wave, uint32_t kappa_c, uint32_t kappa, uint32_t pmask,
                                                  uint16_t* __restrict__ pairs_c, float* __restrict__ values_c,
                                                  float* __restrict__ scales_c) {
    // ---- final pass: selection predicate, output positions, quantise, pack, residual ----
    const uint64_t thr = sh.thr;
    const uint32_t T = (uint32_t)(thr >> 12);
    const uint32_t idxT = 4095u - ((uint32_t)thr & 4095u);
    uint32_t amax_k = sh.wmax[0];
    amax_k = sh.wmax[1] > amax_k ? sh.wmax[1] : amax_k;
    amax_k = sh.wmax[2] > amax_k ? sh.wmax[2] : amax_k;
    amax_k = sh.wmax[3] > amax_k ? sh.wmax[3] : amax_k;
    // The smallest selected magnitude is the threshold key itself; the largest is the chunk maximum.
    const float amin = __uint_as_float(T), amax = __uint_as_float(amax_k);
    const float dd = __fsub_rn(amax, amin);
    const float lo = __fadd_rn(amin, __fmul_rn(0.25f, dd));
    const float tau = __fadd_rn(amin, __fmul_rn(0.5f, dd));
    const float hi = __fadd_rn(amin, __fmul_rn(0.75f, dd));
    const uint32_t tau_bits = __float_as_uint(tau);

    uint32_t base_of_slot[4];
    {
        uint32_t run = 0;
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            if ((b & 3) == wave) base_of_slot[b >> 2] = run;
            run += sh.bucket[b];
        }
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        bool sel[4];
        uint64_t m4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t idx = s * 1024 + tid * 4 + j;
            uint32_t key = __float_as_uint(x[4 * s + j]) & 0x7FFFFFFFu;
            sel[j] = (pmask & (1u << (4 * s + j))) && (key > T || (key == T && idx <= idxT));
            m4[j] = __ballot(sel[j]);
        }
        if ((m4[0] | m4[1] | m4[2] | m4[3]) != 0) {
            uint32_t pos = base_of_slot[s] + lanes_below(m4[0]) + lanes_below(m4[1]) + lanes_below(m4[2]) +
                           lanes_below(m4[3]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (sel[j]) {
                    uint32_t idx = s * 1024 + tid * 4 + j;
                    uint32_t bits = __float_as_uint(x[4 * s + j]);
                    if (QUANT == SPLC_QUANT_2BIT) {
                        uint32_t upper = (bits & 0x7FFFFFFFu) >= tau_bits ? 1u : 0u;
                        uint32_t sign = bits >> 31;
                        float q = __uint_as_float(__float_as_uint(upper ? hi : lo) | (bits & 0x80000000u));
                        pairs_c[pos] = (uint16_t)(idx | (((sign << 1) | upper) << 12));
                        if (SUM) sum[idx] = __fadd_rn(sum[idx], q);
                        x[4 * s + j] = __fsub_rn(x[4 * s + j], q);
                    } else {
                        pairs_c[pos] = (uint16_t)idx;
                        values_c[pos] = x[4 * s + j];
                        if (SUM) sum[idx] = __fadd_rn(sum[idx], x[4 * s + j]);
                        x[4 * s + j] = __fsub_rn(x[4 * s + j], x[4 * s + j]);
                    }
                    ++pos;
                }
            }
        }
    }
    for (uint32_t t = kappa_c + tid; t < kappa; t += kThreads) {
        pairs_c[t] = 0xFFFFu;
        if (QUANT == SPLC_QUANT_NONE) values_c[t] = 0.f;
    }
    if (QUANT == SPLC_QUANT_2BIT && tid == 0) {
        scales_c[0] = lo;
        scales_c[1] = hi;
    }
}

template <int QUANT>
__device__ __forceinline__ void quantise_pack(const SelectShared& sh, float (&x)[16], int tid, int wave,
                                              uint32_t kappa_c, uint32_t kappa, uint32_t pmask,
                                              uint16_t* __restrict__ pairs_c, float* __restrict__ values_c,
                                              float* __restrict__ scales_c) {
    quantise_pack_sum<QUANT, false>(sh, x, nullptr, tid, wave, kappa_c, kappa, pmask, pairs_c, values_c, scales_c);
}

// Both steps for a chunk that stays in registers throughout.
template <int QUANT>
__device__ __forceinline__ void select_quantise_pack(SelectShared& sh, float (&x)[16], int tid, int lane, int wave,
                                                     uint32_t n_c, uint32_t pmask, uint32_t kappa, int force_radix,
                                                     uint32_t* radix_counter, uint16_t* __restrict__ pairs_c,
                                                     float* __restrict__ values_c, float* __restrict__ scales_c) {
    const uint32_t kappa_c = kappa < n_c ? kappa : n_c;
    find_threshold(sh, x, tid, lane, wave, kappa_c, kappa, pmask, force_radix, radix_counter);
    quantise_pack<QUANT>(sh, x, tid, wave, kappa_c, kappa, pmask, pairs_c, values_c, scales_c);
}

// The error-feedback buffer is rewritten densely (line 4 of the update equations).
template <bool VEC>
__device__ __forceinline__ void store_ef(float* __restrict__ e, const ChunkDesc& d, int tid, uint32_t pmask,
                                         const float (&x)[16]) {
    float* pe = e + d.offset;
    if (VEC) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
            stream_store4(vec_at(pe, d, tid, s), make_float4(x[4 * s], x[4 * s + 1], x[4 * s + 2], x[4 * s + 3]));
    } else {
#pragma unroll
        for (int el = 0; el < 16; ++el) {
            const uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
            if (pmask & (1u << el)) pe[elem_of(d, idx)] = x[el];
        }
    }
}

// Lines 1-4 of the update equations, one replica, one chunk per workgroup.
// VEC = true: the chunk is complete and allows 4-element vector accesses (the streaming path);
// VEC = false: edge chunks and rows that start at odd bf16 elements, element by element.
template <int MODE, int QUANT, bool VEC>
__device__ __forceinline__ void compress_body(SelectShared& sh, const ChunkDesc* __restrict__ chunks,
                                              const void* const* __restrict__ src_a,
                                              const void* const* __restrict__ src_b,
                                              float* const* __restrict__ ef_tab, float beta, uint32_t kappa,
                                              int force_radix, uint32_t* radix_counter,
                                              uint16_t* __restrict__ pairs_out, float* __restrict__ aux_out) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const ChunkDesc d = chunks[blockIdx.x];
    const uint64_t c = d.id;
    const void* pa = src_a[d.tensor];
    const void* pb = MODE == MODE_PARAMS_F32 ? src_b[d.tensor] : nullptr;
    float* pe = ef_tab[d.tensor];

    const uint32_t pmask = VEC ? 0xFFFFu : present_mask(d, tid);
    const uint32_t n_c = VEC ? (uint32_t)kChunk : d.n_c;
    float x[16];
    if (VEC) load_fold_full<MODE>(pa, pb, pe, d, tid, beta, x);
    else load_fold_scalar<MODE>(pa, pb, pe, d, tid, beta, pmask, x);
    select_quantise_pack<QUANT>(sh, x, tid, lane, wave, n_c, pmask, kappa, force_radix, radix_counter,
                                pairs_out + c * kappa, aux_out + c * kappa, aux_out + 2 * c);
    store_ef<VEC>(pe, d, tid, pmask, x);
}

// The chunk table lists the n_gen element-wise chunks first: workgroups from n_gen on take the
// streaming path (one launch; the branch is uniform per workgroup).
template <int MODE, int QUANT>
__global__ __launch_bounds__(kThreads) void compress_kernel(const ChunkDesc* __restrict__ chunks, uint32_t n_gen,
                                                            const void* const* __restrict__ src_a,
                                                            const void* const* __restrict__ src_b,
                                                            float* const* __restrict__ ef_tab, float beta,
                                                            uint32_t kappa, int force_radix,
                                                            uint32_t* radix_counter,
                                                            uint16_t* __restrict__ pairs_out,
                                                            float* __restrict__ aux_out) {
    __shared__ __align__(16) SelectShared sh;
    if (blockIdx.x >= n_gen)
        compress_body<MODE, QUANT, true>(sh, chunks, src_a, src_b, ef_tab, beta, kappa, force_radix, radix_counter,
                                         pairs_out, aux_out);
    else
        compress_body<MODE, QUANT, false>(sh, chunks, src_a, src_b, ef_tab, beta, kappa, force_radix, radix_counter,
                                          pairs_out, aux_out);
}

// ---- 64 x 64 tiles, four at a time ("strip"): rows of a strip are 1024 contiguous bytes ----
//
// A workgroup that owns one 64 x 64 tile touches 256-byte row segments; when the matrix's row length is not a
// multiple of 32 floats every such segment straddles three 128-byte cache lines instead of two, and the lines on
// a tile's left and right edge are requested again by its neighbours.  So wherever four complete tiles lie side
// by side, ONE workgroup of 1024 lanes takes all four: global memory is accessed row by row (a wave covers one
// 1024-byte row of the strip per instruction: nine lines instead of twelve, none shared with another
// workgroup), the folded values pass through LDS, where each 256-lane group picks up "its" tile in the usual
// chunk layout and runs the selection exactly as the one-tile kernel does, and the new error-feedback values go
// back the same way.  Tiles left over at the end of a tile row, edge tiles and 1-D tensors stay with the
// one-tile kernels.
constexpr int kStripTiles = 4;
constexpr int kStripThreads = kStripTiles * kThreads;
// Two strip workgroups per compute unit (8 waves per SIMD, 64 registers per lane, 2 x 77 KB of LDS): one of
// them selects while the other one's rows are in flight.

struct StripShared {
    float tile[kStripTiles][kChunk];     // local index order: [row * 64 + column]
    SelectShared sel[kStripTiles];
    uint32_t group_ok[kStripTiles];
};

// Row-wise position of lane `lane` of wave `wave` (0..15) in round i (0..3): local row 16 i + wave of the strip,
// floats 4 lane .. 4 lane + 3 of that row, i.e. tile lane / 16, local columns 4 (lane % 16) ...
__device__ __forceinline__ uint32_t strip_row(int i, int wave) { return 16u * (uint32_t)i + (uint32_t)wave; }
// Addressing of the row-wise accesses: per array one base that is uniform over the wave (the array's origin of
// the strip plus `wave` rows), pinned into a scalar register pair, and per round i one 32-bit byte offset per
// lane (16 i rows plus the lane's position in the row) that all arrays share.  Written out like this the accesses
// are encoded as "scalar base + 32-bit lane offset"; left to itself the compiler keeps one 64-bit address per
// access in vector registers, two dozen registers that the 64-register budget of this kernel does not have.
template <class T>
__device__ __forceinline__ T* strip_base(T* origin, const ChunkDesc& d, int wave) {
    const uint64_t u = reinterpret_cast<uint64_t>(origin + (size_t)((uint32_t)wave * d.stride));
    uint32_t lo = (uint32_t)u, hi = (uint32_t)(u >> 32);
    asm volatile("" : "+s"(lo), "+s"(hi));
    return reinterpret_cast<T*>(((uint64_t)hi << 32) | lo);
}
// Byte offset (for 4-byte elements) of this lane's four elements in round i; 63 rows * stride * 4 < 2^32.
__device__ __forceinline__ uint32_t strip_offset(const ChunkDesc& d, int i, int lane) {
    return ((uint32_t)(16 * i) * d.stride + (uint32_t)lane * 4u) * 4u;
}
template <class T>
__device__ __forceinline__ T* strip_at(T* base, uint32_t offset_for_4_byte_elements) {
    using Byte = typename std::conditional<std::is_const<T>::value, const char, char>::type;
    return reinterpret_cast<T*>(reinterpret_cast<Byte*>(base) + offset_for_4_byte_elements / (4u / (uint32_t)sizeof(T)));
}

template <int MODE, int QUANT>
__global__ __launch_bounds__(kStripThreads, 8) void compress_strip_kernel(const ChunkDesc* __restrict__ strips,
                                                                       const void* const* __restrict__ src_a,
                                                                       const void* const* __restrict__ src_b,
                                                                       float* const* __restrict__ ef_tab, float beta,
                                                                       uint32_t kappa, int force_radix,
                                                                       uint32_t* radix_counter,
                                                                       uint16_t* __restrict__ pairs_out,
                                                                       float* __restrict__ aux_out) {
    __shared__ __align__(16) StripShared sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // 0..15
    const ChunkDesc d = strips[blockIdx.x];
    float* const pe = strip_base(ef_tab[d.tensor] + d.offset, d, wave);
    const uint32_t q = (uint32_t)lane >> 4, lc = ((uint32_t)lane & 15u) * 4u;
    uint32_t off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) off[i] = strip_offset(d, i, lane);

    // ---- rows in: fold in registers, e' to LDS ----
    {
        float4 ev[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) ev[i] = stream_load4(strip_at<const float>(pe, off[i]));
        float x[16];
        if (MODE == MODE_PARAMS_F32) {
            const float* po = strip_base(static_cast<const float*>(src_a[d.tensor]) + d.offset, d, wave);
            const float* pl = strip_base(static_cast<const float*>(src_b[d.tensor]) + d.offset, d, wave);
            float4 ov[4], lv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) ov[i] = stream_load4(strip_at(po, off[i]));
#pragma unroll
            for (int i = 0; i < 4; ++i) lv[i] = stream_load4(strip_at(pl, off[i]));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[4 * i + 0] = fold(beta, ev[i].x, __fsub_rn(ov[i].x, lv[i].x));
                x[4 * i + 1] = fold(beta, ev[i].y, __fsub_rn(ov[i].y, lv[i].y));
                x[4 * i + 2] = fold(beta, ev[i].z, __fsub_rn(ov[i].z, lv[i].z));
                x[4 * i + 3] = fold(beta, ev[i].w, __fsub_rn(ov[i].w, lv[i].w));
            }
        } else if (MODE == MODE_DIRECT_F32) {
            const float* pd = strip_base(static_cast<const float*>(src_a[d.tensor]) + d.offset, d, wave);
            float4 dv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dv[i] = stream_load4(strip_at(pd, off[i]));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[4 * i + 0] = fold(beta, ev[i].x, dv[i].x);
                x[4 * i + 1] = fold(beta, ev[i].y, dv[i].y);
                x[4 * i + 2] = fold(beta, ev[i].z, dv[i].z);
                x[4 * i + 3] = fold(beta, ev[i].w, dv[i].w);
            }
        } else {
            const uint16_t* pd = strip_base(static_cast<const uint16_t*>(src_a[d.tensor]) + d.offset, d, wave);
            uint2 dv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dv[i] = stream_load4(strip_at(pd, off[i]));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[4 * i + 0] = fold(beta, ev[i].x, __uint_as_float(dv[i].x << 16));
                x[4 * i + 1] = fold(beta, ev[i].y, __uint_as_float(dv[i].x & 0xFFFF0000u));
                x[4 * i + 2] = fold(beta, ev[i].z, __uint_as_float(dv[i].y << 16));
                x[4 * i + 3] = fold(beta, ev[i].w, __uint_as_float(dv[i].y & 0xFFFF0000u));
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<float4*>(&sm.tile[q][strip_row(i, wave) * 64u + lc]) =
                make_float4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
    }
    __syncthreads();

    // ---- each 256-lane group selects in its own tile ----
    {
        const int group = __builtin_amdgcn_readfirstlane(tid >> 8);
        const int gtid = tid & (kThreads - 1);
        const int gwave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);
        const uint64_t c = (uint64_t)d.id + (uint64_t)group;
        const uint32_t kappa_c = kappa < (uint32_t)kChunk ? kappa : (uint32_t)kChunk;
        float x[16];
        auto fetch_tile = [&]() {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float4 v = *reinterpret_cast<const float4*>(&sm.tile[group][s * 1024 + gtid * 4]);
                x[4 * s] = v.x; x[4 * s + 1] = v.y; x[4 * s + 2] = v.z; x[4 * s + 3] = v.w;
            }
        };
        // The threshold search reads the tile from LDS by itself (it needs only the magnitudes); the values are
        // fetched afterwards: 64 registers per lane (two of these workgroups per compute unit) do not hold values
        // and keys side by side.
        find_threshold(sm.sel[group], x, gtid, lane, gwave, kappa_c, kappa, 0xFFFFu, force_radix, radix_counter,
                       &sm.tile[group][0], sm.group_ok, group);
        fetch_tile();
        quantise_pack<QUANT>(sm.sel[group], x, gtid, gwave, kappa_c, kappa, 0xFFFFu, pairs_out + c * kappa,
                             aux_out + c * kappa, aux_out + 2 * c);
#pragma unroll
        for (int s = 0; s < 4; ++s)
            *reinterpret_cast<float4*>(&sm.tile[group][s * 1024 + gtid * 4]) =
                make_float4(x[4 * s], x[4 * s + 1], x[4 * s + 2], x[4 * s + 3]);
    }
    __syncthreads();

    // ---- rows out (offsets recomputed here, from an opaque copy of the lane number, so that they are not
    // carried in registers through the selection) ----
    int l = lane;
    asm volatile("" : "+v"(l));
#pragma unroll
    for (int i = 0; i < 4; ++i)
        stream_store4(strip_at(pe, strip_offset(d, i, l)),
                      *reinterpret_cast<const float4*>(&sm.tile[q][strip_row(i, wave) * 64u + lc]));
}

// Lines 1-4 for R replicas that share theta_outer (several replicas simulated on one GPU): the
// workgroup reads its theta_outer chunk once and walks the replicas, so theta_outer costs 4 bytes
// per parameter per launch instead of per replica.  Per replica the arithmetic, the selection and
// the outputs are those of compress_kernel.
// With STEP the workgroup finishes the outer step for its chunk (line 5): what each replica sends is
// added, replica after replica, to a sum in LDS (an element always sits in the same lane, so the mean needs
// neither the messages nor any synchronisation), and after the last replica the chunk's mean is applied to
// theta_outer, written to delta_bar if asked for, and the new parameters are copied to the replicas'
// theta_local if asked for.  The sums start at +0 and are divided once by M: the bits of
// sparseloco_aggregate_update.
// Table layout (device): theta_local[r][t] at tl_tab[r * n_tensors + t], likewise ef_tab; message
// buffers pairs_tab[r], aux_tab[r].
template <int QUANT, bool VEC, bool STEP>
__device__ __forceinline__ void compress_batch_body(SelectShared& sh, float* so, float* sum,
                                                    const ChunkDesc* __restrict__ chunks,
                                                    int n_replicas, uint32_t n_tensors,
                                                    float* const* __restrict__ to_tab, float* const* __restrict__ tl_tab,
                                                    float* const* __restrict__ ef_tab, float beta, uint32_t kappa,
                                                    int force_radix, uint32_t* radix_counter,
                                                    uint16_t* const* __restrict__ pairs_tab,
                                                    float* const* __restrict__ aux_tab, float eta,
                                                    float* const* __restrict__ dbar_tab, int reset) {
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const ChunkDesc d = chunks[blockIdx.x];
    const uint64_t c = d.id;
    const uint32_t n_c = VEC ? (uint32_t)kChunk : d.n_c;
    const uint32_t kappa_c = kappa < n_c ? kappa : n_c;
    const float* po = to_tab[d.tensor] + d.offset;
    const uint32_t pmask0 = VEC ? 0xFFFFu : present_mask(d, tid);

    // The theta_outer chunk waits in LDS (each lane re-reads only what it wrote, so no barrier is
    // needed); keeping it in registers across the replica loop would cost occupancy.
    float4* so4 = reinterpret_cast<float4*>(so);
    if (VEC) {
#pragma unroll
        for (int s = 0; s < 4; ++s) so4[s * kThreads + tid] = stream_load4(vec_at(po, d, tid, s));
    } else {
#pragma unroll
        for (int el = 0; el < 16; ++el) {
            const uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
            so[idx] = (pmask0 & (1u << el)) ? po[elem_of(d, idx)] : 0.f;
        }
    }
    float4* sum4 = reinterpret_cast<float4*>(sum);
    if (STEP) {
#pragma unroll
        for (int s = 0; s < 4; ++s) sum4[s * kThreads + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int r = 0; r < n_replicas; ++r) {
        // Per-lane index arithmetic is recomputed in every round: hoisting it out of the loop would
        // pin some 60 registers across the whole selection and halve the occupancy.
        int t = tid;
        uint32_t pmask = pmask0;
        asm volatile("" : "+v"(t), "+v"(pmask));
        const float* pl = tl_tab[(size_t)r * n_tensors + d.tensor] + d.offset;
        float* pe = ef_tab[(size_t)r * n_tensors + d.tensor];
        float x[16];
        if (VEC) {
            float4 lv[4], ev[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) lv[s] = stream_load4(vec_at(pl, d, t, s));
#pragma unroll
            for (int s = 0; s < 4; ++s) ev[s] = stream_load4(vec_at(pe + d.offset, d, t, s));
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float4 ov = so4[s * kThreads + t];
                x[4 * s + 0] = fold(beta, ev[s].x, __fsub_rn(ov.x, lv[s].x));
                x[4 * s + 1] = fold(beta, ev[s].y, __fsub_rn(ov.y, lv[s].y));
                x[4 * s + 2] = fold(beta, ev[s].z, __fsub_rn(ov.z, lv[s].z));
                x[4 * s + 3] = fold(beta, ev[s].w, __fsub_rn(ov.w, lv[s].w));
            }
        } else {
#pragma unroll
            for (int el = 0; el < 16; ++el) {
                const uint32_t idx = (el >> 2) * 1024 + t * 4 + (el & 3);
                const uint32_t at = elem_of(d, idx);
                x[el] = (pmask & (1u << el)) ? fold(beta, pe[d.offset + at], __fsub_rn(so[idx], pl[at])) : 0.f;
            }
        }
        float* aux_r = aux_tab[r];
        find_threshold(sh, x, t, t & 63, wave, kappa_c, kappa, pmask, force_radix, radix_counter);
        quantise_pack_sum<QUANT, STEP>(sh, x, sum, t, wave, kappa_c, kappa, pmask, pairs_tab[r] + c * kappa,
                                       aux_r + c * kappa, aux_r + 2 * c);
        store_ef<VEC>(pe, d, t, pmask, x);
        __syncthreads();          // every lane is done with `sh` before the next replica re-initialises it
    }
    if (!STEP) return;

    const float m = (float)n_replicas;
    float* th = to_tab[d.tensor] + d.offset;
    float* pd = dbar_tab ? dbar_tab[d.tensor] + d.offset : nullptr;
    const int n_reset = reset ? n_replicas : 0;
    if (VEC) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float4 v = sum4[s * kThreads + tid], tn = so4[s * kThreads + tid];
            v.x = __fdiv_rn(v.x, m); v.y = __fdiv_rn(v.y, m); v.z = __fdiv_rn(v.z, m); v.w = __fdiv_rn(v.w, m);
            if (pd) stream_store4(vec_at(pd, d, tid, s), v);
            tn.x = __fsub_rn(tn.x, __fmul_rn(eta, v.x));
            tn.y = __fsub_rn(tn.y, __fmul_rn(eta, v.y));
            tn.z = __fsub_rn(tn.z, __fmul_rn(eta, v.z));
            tn.w = __fsub_rn(tn.w, __fmul_rn(eta, v.w));
            stream_store4(vec_at(th, d, tid, s), tn);
            for (int r = 0; r < n_reset; ++r)
                stream_store4(vec_at(tl_tab[(size_t)r * n_tensors + d.tensor] + d.offset, d, tid, s), tn);
        }
    } else {
#pragma unroll
        for (int el = 0; el < 16; ++el) {
            if (!(pmask0 & (1u << el))) continue;
            const uint32_t idx = (el >> 2) * 1024 + tid * 4 + (el & 3);
            const uint32_t at = elem_of(d, idx);
            const float v = __fdiv_rn(sum[idx], m);
            if (pd) pd[at] = v;
            const float tn = __fsub_rn(so[idx], __fmul_rn(eta, v));
            th[at] = tn;
            for (int r = 0; r < n_reset; ++r) tl_tab[(size_t)r * n_tensors + d.tensor][d.offset + at] = tn;
        }
    }
}

// Four workgroups per compute unit: the register allocation is held to 128.
template <int QUANT, bool STEP>
__global__ __launch_bounds__(kThreads, 4) void compress_batch_kernel(const ChunkDesc* __restrict__ chunks, uint32_t n_gen,
                                                                  int n_replicas, uint32_t n_tensors,
                                                                  float* const* __restrict__ to_tab,
                                                                  float* const* __restrict__ tl_tab,
                                                                  float* const* __restrict__ ef_tab, float beta,
                                                                  uint32_t kappa, int force_radix,
                                                                  uint32_t* radix_counter,
                                                                  uint16_t* const* __restrict__ pairs_tab,
                                                                  float* const* __restrict__ aux_tab, float eta,
                                                                  float* const* __restrict__ dbar_tab, int reset) {
    __shared__ __align__(16) SelectShared sh;
    __shared__ __align__(16) float so[kChunk];
    __shared__ __align__(16) float sum[STEP ? kChunk : 4];
    if (blockIdx.x >= n_gen)
        compress_batch_body<QUANT, true, STEP>(sh, so, sum, chunks, n_replicas, n_tensors, to_tab, tl_tab, ef_tab, beta, kappa,
                                               force_radix, radix_counter, pairs_tab, aux_tab, eta, dbar_tab, reset);
    else
        compress_batch_body<QUANT, false, STEP>(sh, so, sum, chunks, n_replicas, n_tensors, to_tab, tl_tab, ef_tab, beta,
                                                kappa, force_radix, radix_counter, pairs_tab, aux_tab, eta, dbar_tab,
                                                reset);
}

// Line 5, first half: sum of the decoded messages of one chunk into a dense LDS accumulator.
// Replicas are applied in batches of eight; a batch is applied by ONE wave: LDS operations of a
// wave complete in program order, so the add of replica r+1 at some index sees the add of replica
// r at the same index without a barrier, and inside one replica the indices are distinct.  Batches
// follow each other in replica order with a workgroup barrier in between (the four waves take
// turns, so that the messages of four batches are in flight at once).  Every element therefore
// receives its addends in ascending replica order -- deterministic, no float atomics, no sort.
constexpr int kAggBatch = 8;

template <int QUANT, int KP>
struct MessageBatch {
    uint32_t p[kAggBatch][KP];
    float lo[kAggBatch], hi[kAggBatch], val[kAggBatch][KP];

    // Fetch replicas r0 .. r0+7 of chunk c (all loads issued together).
    __device__ __forceinline__ void load(uint64_t c, uint32_t kappa, uint32_t kappa_c, int r0, int n_replicas,
                                         const uint16_t* const* __restrict__ pairs_tab,
                                         const float* const* __restrict__ aux_tab, int lane) {
#pragma unroll
        for (int i = 0; i < kAggBatch; ++i) {
            lo[i] = hi[i] = 0.f;
#pragma unroll
            for (int k = 0; k < KP; ++k) { p[i][k] = 0xFFFFu; val[i][k] = 0.f; }
            if (r0 + i < n_replicas) {
                const uint16_t* pr = pairs_tab[r0 + i] + c * kappa;
                const float* ar = aux_tab[r0 + i];
                if (QUANT == SPLC_QUANT_2BIT) {
                    lo[i] = ar[2 * c];
                    hi[i] = ar[2 * c + 1];
                }
#pragma unroll
                for (int k = 0; k < KP; ++k) {
                    const uint32_t t = lane + 64 * k;
                    if (t < kappa_c) {
                        p[i][k] = pr[t];
                        if (QUANT == SPLC_QUANT_NONE) val[i][k] = ar[c * kappa + t];
                    }
                }
            }
        }
    }

    // Add them to the accumulator, replica after replica.
    __device__ __forceinline__ void apply(float* acc, uint32_t kappa_c, int r0, int n_replicas, int lane) const {
#pragma unroll
        for (int i = 0; i < kAggBatch; ++i) {
            if (r0 + i < n_replicas) {
#pragma unroll
                for (int k = 0; k < KP; ++k) {
                    const uint32_t t = lane + 64 * k;
                    const uint32_t idx = p[i][k] & 0xFFFu;
                    float q;
                    if (QUANT == SPLC_QUANT_2BIT) {
                        const float level = (p[i][k] & 0x1000u) ? hi[i] : lo[i];
                        q = (p[i][k] & 0x2000u) ? -level : level;
                    } else {
                        q = val[i][k];
                    }
                    if (t < kappa_c) acc[idx] = __fadd_rn(acc[idx], q);
                }
                // The adds of replica r0 + i + 1 must follow those of replica r0 + i in program order (two replicas
                // may hit the same index from different lanes): keep the compiler from moving LDS accesses across.
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
};

// All lanes of the workgroup call this after the accumulator has been cleared (no barrier needed
// before the call; one is taken inside before the first add).  Ends with a barrier.
template <int QUANT, int KP>
__device__ __forceinline__ void accumulate_chunk(float* acc, uint64_t c, uint32_t kappa, uint32_t kappa_c,
                                                 int n_replicas, const uint16_t* const* __restrict__ pairs_tab,
                                                 const float* const* __restrict__ aux_tab, int lane, int wave) {
    const int n_batches = (n_replicas + kAggBatch - 1) / kAggBatch;
    MessageBatch<QUANT, KP> mb;
    if (wave < n_batches) mb.load(c, kappa, kappa_c, wave * kAggBatch, n_replicas, pairs_tab, aux_tab, lane);
    __syncthreads();                                   // accumulator cleared by every lane
    for (int g = 0; g < n_batches; ++g) {
        if (wave == (g & 3)) {
            mb.apply(acc, kappa_c, g * kAggBatch, n_replicas, lane);
            if (g + 4 < n_batches)
                mb.load(c, kappa, kappa_c, (g + 4) * kAggBatch, n_replicas, pairs_tab, aux_tab, lane);
        }
        __syncthreads();
    }
}

// Any kappa: one replica after the other, no batching (used for kappa > 256).
template <int QUANT>
__device__ __forceinline__ void accumulate_chunk_any(float* acc, uint64_t c, uint32_t kappa,
                                                     uint32_t kappa_c, int n_replicas,
                                                     const uint16_t* const* __restrict__ pairs_tab,
                                                     const float* const* __restrict__ aux_tab, int lane) {
    for (int r = 0; r < n_replicas; ++r) {
        const uint16_t* pr = pairs_tab[r] + c * kappa;
        const float* ar = aux_tab[r];
        float lo = 0.f, hi = 0.f;
        if (QUANT == SPLC_QUANT_2BIT) { lo = ar[2 * c]; hi = ar[2 * c + 1]; }
        for (uint32_t t = lane; t < kappa_c; t += 64) {
            const uint32_t p = pr[t];
            const uint32_t idx = p & 0xFFFu;
            float q;
            if (QUANT == SPLC_QUANT_2BIT) {
                const float level = (p & 0x1000u) ? hi : lo;
                q = (p & 0x2000u) ? -level : level;
            } else {
                q = ar[c * kappa + t];
            }
            acc[idx] = __fadd_rn(acc[idx], q);
            __builtin_amdgcn_wave_barrier();         // keeps the LDS accesses of successive rounds in program order
        }
    }
}

// Line 5 of the update equations.  One workgroup per chunk; all lanes clear the 16 KB LDS
// accumulator, the waves apply the messages batch by batch, all lanes divide once by M and write.
//   UPDATE = 0: delta_bar = acc / M is written densely (sparseloco_aggregate).
//   UPDATE = 1: theta = fl(theta - fl(eta * delta_bar)) is applied in the same pass, and the new theta
//               is also copied into n_reset further parameter sets (the replicas' theta_local, which
//               restart from the synchronised parameters: section 2.1, inner step); delta_bar is
//               written only if a table for it is given (sparseloco_aggregate_update).
template <int QUANT, int UPDATE, bool VEC>
__device__ __forceinline__ void aggregate_body(float* acc, const ChunkDesc* __restrict__ chunks, int n_replicas,
                                                             uint32_t kappa,
                                                             const uint16_t* const* __restrict__ pairs_tab,
                                                             const float* const* __restrict__ aux_tab,
                                                             float* const* __restrict__ dbar_tab,
                                                             float* const* __restrict__ theta_tab, float eta, int n_reset,
                                               uint32_t n_tensors, float* const* __restrict__ reset_tab) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const ChunkDesc d = chunks[blockIdx.x];
    const uint64_t c = d.id;
    const uint32_t n_c = VEC ? (uint32_t)kChunk : d.n_c;
    const uint32_t kappa_c = kappa < n_c ? kappa : n_c;
    float4* acc4 = reinterpret_cast<float4*>(acc);
    float* th = UPDATE ? theta_tab[d.tensor] + d.offset : nullptr;
    float* po = dbar_tab ? dbar_tab[d.tensor] + d.offset : nullptr;
    float4 tv[4];
    if (UPDATE && VEC) {
#pragma unroll
        for (int s = 0; s < 4; ++s) tv[s] = stream_load4(vec_at(th, d, tid, s));
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) acc4[s * kThreads + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (kappa_c <= 64) {
        accumulate_chunk<QUANT, 1>(acc, c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane, wave);
    } else if (kappa_c <= 128) {
        accumulate_chunk<QUANT, 2>(acc, c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane, wave);
    } else if (kappa_c <= 256) {
        accumulate_chunk<QUANT, 4>(acc, c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane, wave);
    } else {
        __syncthreads();
        if (wave == 0) accumulate_chunk_any<QUANT>(acc, c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane);
        __syncthreads();
    }
    const float m = (float)n_replicas;
    if (VEC) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float4 v = acc4[s * kThreads + tid];
            v.x = __fdiv_rn(v.x, m); v.y = __fdiv_rn(v.y, m); v.z = __fdiv_rn(v.z, m); v.w = __fdiv_rn(v.w, m);
            if (po) stream_store4(vec_at(po, d, tid, s), v);
            if (UPDATE) {
                float4 t = tv[s];
                t.x = __fsub_rn(t.x, __fmul_rn(eta, v.x));
                t.y = __fsub_rn(t.y, __fmul_rn(eta, v.y));
                t.z = __fsub_rn(t.z, __fmul_rn(eta, v.z));
                t.w = __fsub_rn(t.w, __fmul_rn(eta, v.w));
                stream_store4(vec_at(th, d, tid, s), t);
                for (int r = 0; r < n_reset; ++r)
                    stream_store4(vec_at(reset_tab[(size_t)r * n_tensors + d.tensor] + d.offset, d, tid, s), t);
            }
        }
    } else {
        for (uint32_t idx = tid; idx < (uint32_t)kChunk; idx += kThreads) {
            if (!present(d, idx)) continue;
            const uint32_t at = elem_of(d, idx);
            const float v = __fdiv_rn(acc[idx], m);
            if (po) po[at] = v;
            if (UPDATE) {
                const float t = __fsub_rn(th[at], __fmul_rn(eta, v));
                th[at] = t;
                for (int r = 0; r < n_reset; ++r) reset_tab[(size_t)r * n_tensors + d.tensor][d.offset + at] = t;
            }
        }
    }
}

template <int QUANT, int UPDATE>
__global__ __launch_bounds__(kThreads) void aggregate_kernel(const ChunkDesc* __restrict__ chunks, uint32_t n_gen,
                                                             int n_replicas, uint32_t kappa,
                                                             const uint16_t* const* __restrict__ pairs_tab,
                                                             const float* const* __restrict__ aux_tab,
                                                             float* const* __restrict__ dbar_tab,
                                                             float* const* __restrict__ theta_tab, float eta,
                                                             int n_reset, uint32_t n_tensors,
                                                             float* const* __restrict__ reset_tab) {
    __shared__ __align__(16) float acc[kChunk];
    if (blockIdx.x >= n_gen)
        aggregate_body<QUANT, UPDATE, true>(acc, chunks, n_replicas, kappa, pairs_tab, aux_tab, dbar_tab, theta_tab, eta,
                                            n_reset, n_tensors, reset_tab);
    else
        aggregate_body<QUANT, UPDATE, false>(acc, chunks, n_replicas, kappa, pairs_tab, aux_tab, dbar_tab, theta_tab,
                                             eta, n_reset, n_tensors, reset_tab);
}

// Line 5 for a strip of four complete 64 x 64 tiles (see compress_strip_kernel): the four 256-lane groups
// accumulate the messages of their tiles side by side; the mean (and the parameters) leave and enter row by row.
template <int QUANT, int UPDATE>
__global__ __launch_bounds__(kStripThreads, 8) void aggregate_strip_kernel(const ChunkDesc* __restrict__ strips,
                                                                        int n_replicas, uint32_t kappa,
                                                                        const uint16_t* const* __restrict__ pairs_tab,
                                                                        const float* const* __restrict__ aux_tab,
                                                                        float* const* __restrict__ dbar_tab,
                                                                        float* const* __restrict__ theta_tab, float eta,
                                                                        int n_reset, uint32_t n_tensors,
                                                                        float* const* __restrict__ reset_tab) {
    __shared__ __align__(16) float acc[kStripTiles][kChunk];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = __builtin_amdgcn_readfirstlane(tid >> 8);
    const int gtid = tid & (kThreads - 1);
    const int gwave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);
    const ChunkDesc d = strips[blockIdx.x];
    const uint32_t q = (uint32_t)lane >> 4, lc = ((uint32_t)lane & 15u) * 4u;
    float* th = UPDATE ? strip_base(theta_tab[d.tensor] + d.offset, d, wave) : nullptr;
    float* po = dbar_tab ? strip_base(dbar_tab[d.tensor] + d.offset, d, wave) : nullptr;
    float4* acc4 = reinterpret_cast<float4*>(&acc[group][0]);
#pragma unroll
    for (int s = 0; s < 4; ++s) acc4[s * kThreads + gtid] = make_float4(0.f, 0.f, 0.f, 0.f);
    const uint32_t kappa_c = kappa < (uint32_t)kChunk ? kappa : (uint32_t)kChunk;
    const uint64_t c = (uint64_t)d.id + (uint64_t)group;
    if (kappa_c <= 64) {
        accumulate_chunk<QUANT, 1>(acc[group], c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane, gwave);
    } else if (kappa_c <= 128) {
        accumulate_chunk<QUANT, 2>(acc[group], c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane, gwave);
    } else if (kappa_c <= 256) {
        accumulate_chunk<QUANT, 4>(acc[group], c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane, gwave);
    } else {
        __syncthreads();
        if (gwave == 0) accumulate_chunk_any<QUANT>(acc[group], c, kappa, kappa_c, n_replicas, pairs_tab, aux_tab, lane);
        __syncthreads();
    }
    const float m = (float)n_replicas;
    // The parameters are fetched only now: held across the accumulation they would cost the registers that let
    // two of these workgroups share a compute unit, and the second workgroup hides this latency.
    float4 tv[4];
    if (UPDATE) {
#pragma unroll
        for (int i = 0; i < 4; ++i) tv[i] = stream_load4(strip_at<const float>(th, strip_offset(d, i, lane)));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float4 v = *reinterpret_cast<const float4*>(&acc[q][strip_row(i, wave) * 64u + lc]);
        v.x = __fdiv_rn(v.x, m); v.y = __fdiv_rn(v.y, m); v.z = __fdiv_rn(v.z, m); v.w = __fdiv_rn(v.w, m);
        if (po) stream_store4(strip_at(po, strip_offset(d, i, lane)), v);
        if (UPDATE) {
            float4 t = tv[i];
            t.x = __fsub_rn(t.x, __fmul_rn(eta, v.x));
            t.y = __fsub_rn(t.y, __fmul_rn(eta, v.y));
            t.z = __fsub_rn(t.z, __fmul_rn(eta, v.z));
            t.w = __fsub_rn(t.w, __fmul_rn(eta, v.w));
            stream_store4(strip_at(th, strip_offset(d, i, lane)), t);
            for (int r = 0; r < n_reset; ++r)
                stream_store4(strip_at(strip_base(reset_tab[(size_t)r * n_tensors + d.tensor] + d.offset, d, wave),
                                       strip_offset(d, i, lane)), t);
        }
    }
}

// Line 5, second half: theta = fl(theta - fl(eta * delta_bar)).
template <bool VEC>
__device__ __forceinline__ void outer_update_body(const ChunkDesc* __restrict__ chunks,
                                                  float* const* __restrict__ theta_tab,
                                                  const float* const* __restrict__ dbar_tab, float eta) {
    const int tid = threadIdx.x;
    const ChunkDesc d = chunks[blockIdx.x];
    float* th = theta_tab[d.tensor] + d.offset;
    const float* db = dbar_tab[d.tensor] + d.offset;
    if (VEC) {
        float4 t[4], g[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) t[s] = stream_load4(vec_at(th, d, tid, s));
#pragma unroll
        for (int s = 0; s < 4; ++s) g[s] = stream_load4(vec_at(db, d, tid, s));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            t[s].x = __fsub_rn(t[s].x, __fmul_rn(eta, g[s].x));
            t[s].y = __fsub_rn(t[s].y, __fmul_rn(eta, g[s].y));
            t[s].z = __fsub_rn(t[s].z, __fmul_rn(eta, g[s].z));
            t[s].w = __fsub_rn(t[s].w, __fmul_rn(eta, g[s].w));
            stream_store4(vec_at(th, d, tid, s), t[s]);
        }
    } else {
        for (uint32_t idx = tid; idx < (uint32_t)kChunk; idx += kThreads) {
            if (!present(d, idx)) continue;
            const uint32_t at = elem_of(d, idx);
            th[at] = __fsub_rn(th[at], __fmul_rn(eta, db[at]));
        }
    }
}

__global__ __launch_bounds__(kThreads) void outer_update_kernel(const ChunkDesc* __restrict__ chunks, uint32_t n_gen,
                                                                float* const* __restrict__ theta_tab,
                                                                const float* const* __restrict__ dbar_tab,
                                                                float eta) {
    if (blockIdx.x >= n_gen) outer_update_body<true>(chunks, theta_tab, dbar_tab, eta);
    else outer_update_body<false>(chunks, theta_tab, dbar_tab, eta);
}

}  // namespace

// ------------------------------------------------------------------ host side

struct sparseloco_plan {
    int device = 0;
    int n_tensors = 0;
    int kappa = 0;
    int quant = SPLC_QUANT_2BIT;
    int select = SPLC_SELECT_AUTO;
    uint32_t* radix_counter = nullptr;   // diagnostic (sparseloco_plan_set_radix_counter), normally null
    int64_t n_chunks = 0;
    int64_t n_params = 0;
    std::vector<int64_t> numel;
    int layout = SPLC_LAYOUT_FLAT;
    // Chunk table, ordered [edge chunks | complete, vector-able for fp32 only | complete, vector-able for
    // fp32 and bf16]; every entry carries its chunk number.  The slow element-wise chunks come first so
    // that they overlap with the streaming ones instead of forming the tail of the launch.
    // A tiled plan takes complete tiles four at a time where four lie side by side ("strips", one entry each:
    // origin, stride and chunk number of the first tile); only the other chunks are in the table above.  Its
    // outer update, which is element-wise, walks the tensors as flat chunks (a table of its own).
    // One device allocation holds [chunks | strips | flat chunks of the update | every chunk one by one].
    ChunkDesc* d_chunks = nullptr;
    ChunkDesc* h_chunks = nullptr;       // pinned source of the asynchronous upload, kept until destroy
    int64_t n_entries = 0;               // entries of the chunk table (= n_chunks unless there are strips)
    int64_t n_gen_f32 = 0;               // entries of the first class
    int64_t n_gen_bf16 = 0;              // entries of the first two classes
    int64_t n_strips = 0;
    ChunkDesc* d_strips = nullptr;       // inside d_chunks' allocation
    ChunkDesc* d_update = nullptr;       // = d_chunks for a flat plan
    int64_t n_update = 0, n_update_gen = 0;
    ChunkDesc* d_all = nullptr;          // every chunk one by one, for the batched compress (= d_chunks without strips)
    int64_t n_all_gen = 0;
};

// n_sets lists of n_tensors device pointers, set-major, resident on the device.
struct sparseloco_tensors {
    int device = 0;
    int n_tensors = 0;
    int n_sets = 0;
    int dtype = SPLC_F32;
    void** d_table = nullptr;
    void** h_table = nullptr;            // pinned source of the upload
};

// Message buffers of n_replicas replicas: device table [pairs: n_replicas][aux: n_replicas].
struct sparseloco_messages {
    int device = 0;
    int n_replicas = 0;
    int quant = SPLC_QUANT_2BIT;
    int kappa = 0;
    int64_t n_chunks = 0;
    void** d_table = nullptr;
    void** h_table = nullptr;
};

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
bool finite(float v) { return v == v && v - v == 0.f; }

int current_device_is(int device) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SPLC_EHIP;
    return dev == device ? SPLC_OK : SPLC_EPLAN;
}

// A binding fits the plan: same device, same tensor count, the wanted element type, enough sets.
int check_tensors(const sparseloco_plan* plan, const sparseloco_tensors* t, int dtype, int min_sets) {
    if (!t) return SPLC_EINVAL;
    if (t->device != plan->device || t->n_tensors != plan->n_tensors || t->dtype != dtype) return SPLC_EPLAN;
    return t->n_sets >= min_sets ? SPLC_OK : SPLC_EINVAL;
}
int check_messages(const sparseloco_plan* plan, const sparseloco_messages* m, int min_replicas) {
    if (!m) return SPLC_EINVAL;
    if (m->device != plan->device || m->quant != plan->quant || m->kappa != plan->kappa || m->n_chunks != plan->n_chunks)
        return SPLC_EPLAN;
    return m->n_replicas >= min_replicas ? SPLC_OK : SPLC_EINVAL;
}
// Device table of set `set` of a binding (a single-set binding serves every set index).
template <class T>
T const* set_table(const sparseloco_tensors* t, int set) {
    return reinterpret_cast<T const*>(t->d_table + (size_t)(t->n_sets == 1 ? 0 : set) * (size_t)t->n_tensors);
}

// A small table of device pointers: pinned host copy + device copy, uploaded asynchronously on `stream`.
int upload_table(size_t n_ptrs, void*** h_out, void*** d_out) {
    const size_t bytes = (n_ptrs ? n_ptrs : 1) * sizeof(void*);
    if (hipHostMalloc(reinterpret_cast<void**>(h_out), bytes, hipHostMallocDefault) != hipSuccess) return SPLC_ENOMEM;
    if (hipMalloc(reinterpret_cast<void**>(d_out), bytes) != hipSuccess) return SPLC_ENOMEM;
    return SPLC_OK;
}

// Entries of the chunk table that take the element-wise path (they come first in the table).
unsigned gen_entries(const sparseloco_plan* plan, bool bf16_source) {
    return (unsigned)(bf16_source ? plan->n_gen_bf16 : plan->n_gen_f32);
}

template <int MODE, int QUANT>
void launch_compress(const sparseloco_plan* plan, const void* const* a, const void* const* b, float* const* ef,
                     float beta, uint16_t* pairs_out, float* aux_out, hipStream_t stream) {
    const int force_radix = plan->select == SPLC_SELECT_RADIX ? 1 : 0;
    if (plan->n_strips > 0)
        hipLaunchKernelGGL((compress_strip_kernel<MODE, QUANT>), dim3((unsigned)plan->n_strips), dim3(kStripThreads), 0,
                           stream, plan->d_strips, a, b, ef, beta, (uint32_t)plan->kappa, force_radix,
                           plan->radix_counter, pairs_out, aux_out);
    if (plan->n_entries > 0)
        hipLaunchKernelGGL((compress_kernel<MODE, QUANT>), dim3((unsigned)plan->n_entries), dim3(kThreads), 0, stream,
                           plan->d_chunks, gen_entries(plan, MODE == MODE_DIRECT_BF16), a, b, ef, beta,
                           (uint32_t)plan->kappa, force_radix, plan->radix_counter, pairs_out, aux_out);
}

template <int QUANT, bool STEP>
void launch_compress_batch(const sparseloco_plan* plan, int n_replicas, float* const* to, float* const* tl,
                           float* const* ef, float beta, uint16_t* const* pairs, float* const* aux, float eta,
                           float* const* dbar, int reset, hipStream_t stream) {
    // Strips are taken tile by tile here: a strip entry is followed, in the device table, by nothing this kernel
    // could use, so the batched path walks the per-chunk view kept behind the update table.
    hipLaunchKernelGGL((compress_batch_kernel<QUANT, STEP>), dim3((unsigned)plan->n_chunks), dim3(kThreads), 0, stream,
                       plan->d_all, (unsigned)plan->n_all_gen, n_replicas, (uint32_t)plan->n_tensors, to, tl, ef,
                       beta, (uint32_t)plan->kappa, plan->select == SPLC_SELECT_RADIX ? 1 : 0, plan->radix_counter, pairs,
                       aux, eta, dbar, reset);
}

// Shared by sparseloco_compress_batch and sparseloco_outer_step_batch.
int compress_batch_impl(const sparseloco_plan* plan, int n_replicas, const sparseloco_tensors* theta_outer,
                        const sparseloco_tensors* theta_local, const sparseloco_tensors* ef, float beta,
                        const sparseloco_messages* messages_out, bool step, float outer_lr,
                        const sparseloco_tensors* delta_bar_out, int reset, void* stream) {
    if (!plan || n_replicas < 1 || n_replicas > SPLC_MAX_REPLICAS) return SPLC_EINVAL;
    int rc;
    if ((rc = check_tensors(plan, theta_outer, SPLC_F32, 1)) != SPLC_OK) return rc;
    if (theta_outer->n_sets != 1) return SPLC_EINVAL;
    if ((rc = check_tensors(plan, theta_local, SPLC_F32, n_replicas)) != SPLC_OK) return rc;
    if ((rc = check_tensors(plan, ef, SPLC_F32, n_replicas)) != SPLC_OK) return rc;
    if ((rc = check_messages(plan, messages_out, n_replicas)) != SPLC_OK) return rc;
    if (delta_bar_out) {
        if ((rc = check_tensors(plan, delta_bar_out, SPLC_F32, 1)) != SPLC_OK) return rc;
        if (delta_bar_out->n_sets != 1) return SPLC_EINVAL;
    }
    if (!finite(beta) || !finite(outer_lr)) return SPLC_EINVAL;
    if ((rc = current_device_is(plan->device)) != SPLC_OK) return rc;
    if (plan->n_chunks == 0) return SPLC_OK;

    hipStream_t st = static_cast<hipStream_t>(stream);
    float* const* d_to = set_table<float*>(theta_outer, 0);
    float* const* d_tl = reinterpret_cast<float* const*>(theta_local->d_table);
    float* const* d_ef = reinterpret_cast<float* const*>(ef->d_table);
    uint16_t* const* d_pairs = reinterpret_cast<uint16_t* const*>(messages_out->d_table);
    float* const* d_aux = reinterpret_cast<float* const*>(messages_out->d_table + messages_out->n_replicas);
    float* const* d_dbar = delta_bar_out ? set_table<float*>(delta_bar_out, 0) : nullptr;
    const bool q2 = plan->quant == SPLC_QUANT_2BIT;
    if (q2 && !step)
        launch_compress_batch<SPLC_QUANT_2BIT, false>(plan, n_replicas, d_to, d_tl, d_ef, beta, d_pairs, d_aux, 0.f, nullptr, 0, st);
    else if (q2)
        launch_compress_batch<SPLC_QUANT_2BIT, true>(plan, n_replicas, d_to, d_tl, d_ef, beta, d_pairs, d_aux, outer_lr, d_dbar, reset, st);
    else if (!step)
        launch_compress_batch<SPLC_QUANT_NONE, false>(plan, n_replicas, d_to, d_tl, d_ef, beta, d_pairs, d_aux, 0.f, nullptr, 0, st);
    else
        launch_compress_batch<SPLC_QUANT_NONE, true>(plan, n_replicas, d_to, d_tl, d_ef, beta, d_pairs, d_aux, outer_lr, d_dbar, reset, st);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

template <int QUANT, int UPDATE>
void launch_aggregate(const sparseloco_plan* plan, int n_replicas, const uint16_t* const* pairs,
                      const float* const* aux, float* const* dbar, float* const* theta, float eta, int n_reset,
                      float* const* reset, hipStream_t stream) {
    if (plan->n_strips > 0)
        hipLaunchKernelGGL((aggregate_strip_kernel<QUANT, UPDATE>), dim3((unsigned)plan->n_strips), dim3(kStripThreads),
                           0, stream, plan->d_strips, n_replicas, (uint32_t)plan->kappa, pairs, aux, dbar, theta, eta,
                           n_reset, (uint32_t)plan->n_tensors, reset);
    if (plan->n_entries > 0)
        hipLaunchKernelGGL((aggregate_kernel<QUANT, UPDATE>), dim3((unsigned)plan->n_entries), dim3(kThreads), 0, stream,
                           plan->d_chunks, gen_entries(plan, false), n_replicas, (uint32_t)plan->kappa, pairs, aux,
                           dbar, theta, eta, n_reset, (uint32_t)plan->n_tensors, reset);
}

// Shared by sparseloco_aggregate and sparseloco_aggregate_update.
int aggregate_impl(const sparseloco_plan* plan, const sparseloco_messages* messages,
                   const sparseloco_tensors* delta_bar_out, const sparseloco_tensors* theta_outer, float outer_lr,
                   bool update, const sparseloco_tensors* reset, void* stream) {
    if (!plan) return SPLC_EINVAL;
    int rc = check_messages(plan, messages, 1);
    if (rc != SPLC_OK) return rc;
    if (update ? !theta_outer : !delta_bar_out) return SPLC_EINVAL;
    if (delta_bar_out && (rc = check_tensors(plan, delta_bar_out, SPLC_F32, 1)) != SPLC_OK) return rc;
    if (update && (rc = check_tensors(plan, theta_outer, SPLC_F32, 1)) != SPLC_OK) return rc;
    if (reset && (rc = check_tensors(plan, reset, SPLC_F32, 1)) != SPLC_OK) return rc;
    if ((delta_bar_out && delta_bar_out->n_sets != 1) || (update && theta_outer->n_sets != 1)) return SPLC_EINVAL;
    if (!finite(outer_lr)) return SPLC_EINVAL;
    if ((rc = current_device_is(plan->device)) != SPLC_OK) return rc;
    if (plan->n_chunks == 0) return SPLC_OK;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nr = messages->n_replicas;
    const uint16_t* const* dp = reinterpret_cast<const uint16_t* const*>(messages->d_table);
    const float* const* dx = reinterpret_cast<const float* const*>(messages->d_table + nr);
    float* const* dout = delta_bar_out ? set_table<float*>(delta_bar_out, 0) : nullptr;
    float* const* dth = update ? set_table<float*>(theta_outer, 0) : nullptr;
    float* const* dreset = reset ? set_table<float*>(reset, 0) : nullptr;
    const int n_reset = reset ? reset->n_sets : 0;
    const bool q2 = plan->quant == SPLC_QUANT_2BIT;
    if (q2 && !update)
        launch_aggregate<SPLC_QUANT_2BIT, 0>(plan, nr, dp, dx, dout, dth, outer_lr, 0, dreset, st);
    else if (q2)
        launch_aggregate<SPLC_QUANT_2BIT, 1>(plan, nr, dp, dx, dout, dth, outer_lr, n_reset, dreset, st);
    else if (!update)
        launch_aggregate<SPLC_QUANT_NONE, 0>(plan, nr, dp, dx, dout, dth, outer_lr, 0, dreset, st);
    else
        launch_aggregate<SPLC_QUANT_NONE, 1>(plan, nr, dp, dx, dout, dth, outer_lr, n_reset, dreset, st);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

// Chunk table of one tensor.  rows == 1 (or flat layout): runs of 4096 elements; otherwise 64 x 64 tiles
// numbered row-major.
void append_chunks(std::vector<ChunkDesc>& table, uint32_t tensor, int64_t rows, int64_t cols, bool tiled) {
    if (rows * cols == 0) return;
    if (!tiled || rows == 1) {
        const int64_t numel = rows * cols;
        for (int64_t off = 0; off < numel; off += kChunk) {
            const int64_t n = (numel - off) < kChunk ? (numel - off) : kChunk;
            ChunkDesc cd = {};
            cd.tensor = tensor;
            cd.n_c = (uint32_t)n;
            cd.offset = (uint64_t)off;
            cd.stride = 64;
            cd.h = (uint8_t)((n + 63) / 64);
            cd.w = 64;
            cd.last_w = (uint8_t)(n - 64 * (cd.h - 1));
            cd.vec = n == kChunk ? 3 : 0;
            table.push_back(cd);
        }
        return;
    }
    for (int64_t r0 = 0; r0 < rows; r0 += 64) {
        for (int64_t c0 = 0; c0 < cols; c0 += 64) {
            const int64_t h = (rows - r0) < 64 ? (rows - r0) : 64, w = (cols - c0) < 64 ? (cols - c0) : 64;
            ChunkDesc cd = {};
            cd.tensor = tensor;
            cd.n_c = (uint32_t)(h * w);
            cd.offset = (uint64_t)(r0 * cols + c0);
            cd.stride = (uint32_t)cols;
            cd.h = (uint8_t)h;
            cd.w = (uint8_t)w;
            cd.last_w = (uint8_t)w;
            const bool full = h == 64 && w == 64;
            cd.vec = (uint8_t)((full ? 1 : 0) | ((full && cols % 2 == 0) ? 2 : 0));
            table.push_back(cd);
        }
    }
}

int chunk_class(const ChunkDesc& d) { return d.vec == 0 ? 0 : (d.vec == 1 ? 1 : 2); }

// Order in which workgroups take the entries: element-wise chunks first (they are the slow ones and should
// overlap with the rest instead of forming the tail), then the chunks that allow vector accesses for fp32 only,
// then those that allow them for bf16 too.  For a tiled plan, inside each class every XCD gets a run of
// consecutive tiles: workgroups go to the eight XCDs round-robin by number, neighbouring tiles of a tile row
// continue each other's row segments (and share the cache lines on their common edge when the row length is no
// multiple of 32 floats), so neighbours should meet in one L2.  Only the order of processing changes: a chunk's
// number, and with it the place of its pairs in the message, is its `id`.
void order_for_launch(std::vector<ChunkDesc>& table, bool deal_to_xcds) {
    std::stable_sort(table.begin(), table.end(),
                     [](const ChunkDesc& a, const ChunkDesc& b) { return chunk_class(a) < chunk_class(b); });
    if (!deal_to_xcds) return;
    size_t start = 0;
    while (start < table.size()) {
        size_t end = start;
        while (end < table.size() && chunk_class(table[end]) == chunk_class(table[start])) ++end;
        const std::vector<ChunkDesc> seg(table.begin() + (ptrdiff_t)start, table.begin() + (ptrdiff_t)end);
        size_t next = 0;
        for (size_t r = 0; r < 8; ++r)
            for (size_t pos = start + (r + 8 - start % 8) % 8; pos < end; pos += 8) table[pos] = seg[next++];
        start = end;
    }
}

struct ChunkTables {
    int64_t n_chunks = 0, n_params = 0;
    std::vector<ChunkDesc> all;          // every chunk, launch order
    std::vector<ChunkDesc> rest;         // tiled plans: the chunks outside strips, launch order
    std::vector<ChunkDesc> strips;       // tiled plans: one entry per strip (its first tile), launch order
    std::vector<ChunkDesc> update;       // tiled plans: flat chunks for the element-wise update
};

// Validates the tensor list and counts its chunks; fills the tables if asked to.
int build_chunk_tables(int n_tensors, const int64_t* rows, const int64_t* cols, bool tiled, ChunkTables& t, bool fill) {
    if (n_tensors < 1 || !cols || (tiled && !rows)) return SPLC_EINVAL;
    int64_t n_chunks = 0, n_params = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const int64_t r = tiled ? rows[i] : 1, c = cols[i];
        if (r < 0 || c < 0) return SPLC_EINVAL;
        if (r > 0 && c > (int64_t)0x7FFFFFFFFFFFFFFF / r) return SPLC_EINVAL;
        if (tiled && r > 1) {
            if (c >= (int64_t)1 << 24) return SPLC_EINVAL;        // byte offsets inside a tile must fit 32 bits
            n_chunks += ((r + 63) / 64) * ((c + 63) / 64);
        } else {
            n_chunks += (r * c + kChunk - 1) / kChunk;
        }
        n_params += r * c;
    }
    if (n_chunks > 0x7FFFFFFF) return SPLC_EINVAL;      // one workgroup per chunk in a 1-D grid
    t.n_chunks = n_chunks;
    t.n_params = n_params;
    if (!fill) return SPLC_OK;
    t.all.clear();
    t.all.reserve((size_t)n_chunks);
    for (int i = 0; i < n_tensors; ++i) append_chunks(t.all, (uint32_t)i, tiled ? rows[i] : 1, cols[i], tiled);
    for (size_t k = 0; k < t.all.size(); ++k) t.all[k].id = (uint32_t)k;
    t.rest.clear();
    t.strips.clear();
    t.update.clear();
    if (tiled) {
        // Strips: four complete tiles side by side, in matrices whose row length is no multiple of 32 floats (with
        // such a multiple a tile's 256-byte row segments are two whole cache lines already, and the one-tile
        // kernel, which needs no trip through LDS, is the faster one: measured 6.0 against 5.8 TB/s) but even (so
        // that rows of a bf16 source start on dword boundaries too).  Tiles of one tile row have consecutive numbers.
        size_t k = 0;
        for (int i = 0; i < n_tensors; ++i) {
            const int64_t r = rows[i], c = cols[i];
            if (r * c == 0) continue;
            if (r == 1) { k += (size_t)((c + kChunk - 1) / kChunk); continue; }
            const int64_t nbi = (r + 63) / 64, nbj = (c + 63) / 64, full_cols = c / 64;
            for (int64_t bi = 0; bi < nbi; ++bi, k += (size_t)nbj) {
                if (c % 32 == 0 || c % 2 != 0 || (bi + 1) * 64 > r) continue;
                for (int64_t s4 = 0; s4 + kStripTiles <= full_cols; s4 += kStripTiles)
                    for (int j = 0; j < kStripTiles; ++j) t.all[k + (size_t)(s4 + j)].reserved = 1u + (uint32_t)j;
            }
        }
        for (const ChunkDesc& cd : t.all) {
            if (cd.reserved == 0) t.rest.push_back(cd);
            else if (cd.reserved == 1) t.strips.push_back(cd);
        }
        order_for_launch(t.rest, true);
        // Strips of one tile row continue each other's rows: every XCD gets a run of consecutive strips.
        {
            const std::vector<ChunkDesc> seg(t.strips);
            size_t next = 0;
            for (size_t x = 0; x < 8; ++x)
                for (size_t pos = x; pos < seg.size(); pos += 8) t.strips[pos] = seg[next++];
        }
        for (int i = 0; i < n_tensors; ++i) append_chunks(t.update, (uint32_t)i, 1, rows[i] * cols[i], false);
        order_for_launch(t.update, false);
    }
    order_for_launch(t.all, tiled);
    return SPLC_OK;
}

int64_t count_class0(const std::vector<ChunkDesc>& v) {
    int64_t n = 0;
    for (const ChunkDesc& cd : v) n += cd.vec == 0;
    return n;
}

int plan_build(sparseloco_plan** out, int n_tensors, const int64_t* rows, const int64_t* cols, bool tiled, int chunk,
               int kappa, int quant_mode, void* stream) {
    if (!out) return SPLC_EINVAL;
    *out = nullptr;
    if (chunk != kChunk || kappa < 1 || kappa > kChunk) return SPLC_EINVAL;
    if (quant_mode != SPLC_QUANT_NONE && quant_mode != SPLC_QUANT_2BIT) return SPLC_EINVAL;
    ChunkTables t;
    int rc = build_chunk_tables(n_tensors, tiled ? rows : nullptr, cols, tiled, t, true);
    if (rc != SPLC_OK) return rc;
    sparseloco_plan* plan = new (std::nothrow) sparseloco_plan();
    if (!plan) return SPLC_ENOMEM;
    if (hipGetDevice(&plan->device) != hipSuccess) { delete plan; return SPLC_EHIP; }
    plan->n_tensors = n_tensors;
    plan->kappa = kappa;
    plan->quant = quant_mode;
    plan->layout = tiled ? SPLC_LAYOUT_TILE64 : SPLC_LAYOUT_FLAT;
    plan->n_chunks = t.n_chunks;
    plan->n_params = t.n_params;
    plan->numel.resize((size_t)n_tensors);
    for (int i = 0; i < n_tensors; ++i) plan->numel[(size_t)i] = (tiled ? rows[i] : 1) * cols[i];
    const bool with_strips = !t.strips.empty();
    const std::vector<ChunkDesc>& main_table = with_strips ? t.rest : t.all;
    plan->n_entries = (int64_t)main_table.size();
    for (const ChunkDesc& cd : main_table) {
        plan->n_gen_f32 += cd.vec == 0;
        plan->n_gen_bf16 += cd.vec != 3;
    }
    plan->n_strips = (int64_t)t.strips.size();
    plan->n_update = tiled ? (int64_t)t.update.size() : plan->n_entries;
    plan->n_update_gen = tiled ? count_class0(t.update) : plan->n_gen_f32;
    plan->n_all_gen = count_class0(t.all);
    // device layout: [main table | strips | update table (tiled) | every chunk (with strips)]
    const size_t n_main = main_table.size(), n_str = t.strips.size(), n_upd = tiled ? t.update.size() : 0,
                 n_all = with_strips ? t.all.size() : 0, total = n_main + n_str + n_upd + n_all;
    if (total > 0) {
        const size_t bytes = total * sizeof(ChunkDesc);
        if (hipHostMalloc(reinterpret_cast<void**>(&plan->h_chunks), bytes, hipHostMallocDefault) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&plan->d_chunks), bytes) != hipSuccess) {
            rc = SPLC_ENOMEM;
        } else {
            std::copy(main_table.begin(), main_table.end(), plan->h_chunks);
            std::copy(t.strips.begin(), t.strips.end(), plan->h_chunks + n_main);
            if (tiled) std::copy(t.update.begin(), t.update.end(), plan->h_chunks + n_main + n_str);
            if (with_strips) std::copy(t.all.begin(), t.all.end(), plan->h_chunks + n_main + n_str + n_upd);
            plan->d_strips = plan->d_chunks + n_main;
            plan->d_update = tiled ? plan->d_chunks + n_main + n_str : plan->d_chunks;
            plan->d_all = with_strips ? plan->d_chunks + n_main + n_str + n_upd : plan->d_chunks;
            if (hipMemcpyAsync(plan->d_chunks, plan->h_chunks, bytes, hipMemcpyHostToDevice,
                               static_cast<hipStream_t>(stream)) != hipSuccess)
                rc = SPLC_EHIP;
        }
    }
    if (rc != SPLC_OK) {
        sparseloco_plan_destroy(plan);
        return rc;
    }
    *out = plan;
    return SPLC_OK;
}

}  // namespace

extern "C" {

int sparseloco_plan_create(sparseloco_plan** out, int n_tensors, const int64_t* numel, int chunk, int kappa,
                           int quant_mode, void* stream) {
    return plan_build(out, n_tensors, nullptr, numel, false, chunk, kappa, quant_mode, stream);
}

int sparseloco_plan_create_2d(sparseloco_plan** out, int n_tensors, const int64_t* rows, const int64_t* cols,
                              int chunk, int kappa, int quant_mode, void* stream) {
    return plan_build(out, n_tensors, rows, cols, true, chunk, kappa, quant_mode, stream);
}

void sparseloco_plan_destroy(sparseloco_plan* plan) {
    if (!plan) return;
    if (plan->d_chunks) (void)hipFree(plan->d_chunks);              // waits for the device; holds all tables
    if (plan->h_chunks) (void)hipHostFree(plan->h_chunks);
    delete plan;
}

int64_t sparseloco_plan_num_chunks(const sparseloco_plan* plan) { return plan ? plan->n_chunks : SPLC_EINVAL; }
int64_t sparseloco_plan_num_params(const sparseloco_plan* plan) { return plan ? plan->n_params : SPLC_EINVAL; }
int sparseloco_plan_num_tensors(const sparseloco_plan* plan) { return plan ? plan->n_tensors : SPLC_EINVAL; }
int sparseloco_plan_kappa(const sparseloco_plan* plan) { return plan ? plan->kappa : SPLC_EINVAL; }
int sparseloco_plan_quant_mode(const sparseloco_plan* plan) { return plan ? plan->quant : SPLC_EINVAL; }
int sparseloco_plan_layout(const sparseloco_plan* plan) { return plan ? plan->layout : SPLC_EINVAL; }

int sparseloco_plan_set_select(sparseloco_plan* plan, int select_mode) {
    if (!plan || (select_mode != SPLC_SELECT_AUTO && select_mode != SPLC_SELECT_RADIX)) return SPLC_EINVAL;
    plan->select = select_mode;
    return SPLC_OK;
}

int sparseloco_plan_set_radix_counter(sparseloco_plan* plan, uint32_t* device_counter) {
    if (!plan || !aligned(device_counter, 4)) return SPLC_EINVAL;
    plan->radix_counter = device_counter;
    return SPLC_OK;
}

int64_t sparseloco_chunk_table(int n_tensors, const int64_t* rows, const int64_t* cols, int layout, void* out,
                               int64_t capacity) {
    if (layout != SPLC_LAYOUT_FLAT && layout != SPLC_LAYOUT_TILE64) return SPLC_EINVAL;
    if (capacity < 0 || (capacity > 0 && !out)) return SPLC_EINVAL;
    const bool tiled = layout == SPLC_LAYOUT_TILE64;
    std::vector<int64_t> flat;
    if (!tiled && rows && cols && n_tensors >= 1) {               // flat layout: only the element counts matter
        flat.resize((size_t)n_tensors);
        for (int i = 0; i < n_tensors; ++i) {
            if (rows[i] < 0 || cols[i] < 0 || (rows[i] > 0 && cols[i] > (int64_t)0x7FFFFFFFFFFFFFFF / rows[i]))
                return SPLC_EINVAL;
            flat[(size_t)i] = rows[i] * cols[i];
        }
        cols = flat.data();
    }
    ChunkTables t;
    int rc = build_chunk_tables(n_tensors, tiled ? rows : nullptr, cols, tiled, t, out != nullptr);
    if (rc != SPLC_OK) return rc;
    if (out) {
        // the entries workgroups of the one-chunk kernels walk, then the members of the strips in strip order
        std::vector<ChunkDesc> view = t.strips.empty() ? t.all : t.rest;
        if (!t.strips.empty()) {
            std::vector<const ChunkDesc*> by_id(t.all.size());
            for (const ChunkDesc& cd : t.all) by_id[cd.id] = &cd;
            for (const ChunkDesc& first : t.strips)
                for (int j = 0; j < kStripTiles; ++j) view.push_back(*by_id[first.id + (uint32_t)j]);
        }
        const int64_t n = t.n_chunks < capacity ? t.n_chunks : capacity;
        std::copy(view.begin(), view.begin() + (ptrdiff_t)n, static_cast<ChunkDesc*>(out));
    }
    return t.n_chunks;
}

int sparseloco_tensors_bind(sparseloco_tensors** out, const sparseloco_plan* plan, int n_sets,
                            const void* const* ptrs, int dtype, void* stream) {
    if (!out) return SPLC_EINVAL;
    *out = nullptr;
    if (!plan || !ptrs || n_sets < 1 || n_sets > SPLC_MAX_REPLICAS) return SPLC_EINVAL;
    if (dtype != SPLC_F32 && dtype != SPLC_BF16) return SPLC_EINVAL;
    const size_t nt = (size_t)plan->n_tensors, n = nt * (size_t)n_sets;
    for (size_t i = 0; i < n; ++i) {
        if (plan->numel[i % nt] == 0) continue;
        if (!ptrs[i]) return SPLC_EINVAL;
        if (!aligned(ptrs[i], 4)) return SPLC_EALIGN;             // for bf16 it keeps vector rows dword aligned
    }
    int rc = current_device_is(plan->device);
    if (rc != SPLC_OK) return rc;
    sparseloco_tensors* t = new (std::nothrow) sparseloco_tensors();
    if (!t) return SPLC_ENOMEM;
    t->device = plan->device;
    t->n_tensors = plan->n_tensors;
    t->n_sets = n_sets;
    t->dtype = dtype;
    if ((rc = upload_table(n, &t->h_table, &t->d_table)) == SPLC_OK) {
        for (size_t i = 0; i < n; ++i) t->h_table[i] = plan->numel[i % nt] == 0 ? nullptr : const_cast<void*>(ptrs[i]);
        if (hipMemcpyAsync(t->d_table, t->h_table, n * sizeof(void*), hipMemcpyHostToDevice,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
            rc = SPLC_EHIP;
    }
    if (rc != SPLC_OK) {
        sparseloco_tensors_release(t);
        return rc;
    }
    *out = t;
    return SPLC_OK;
}

void sparseloco_tensors_release(sparseloco_tensors* t) {
    if (!t) return;
    if (t->d_table) (void)hipFree(t->d_table);                     // waits for the device
    if (t->h_table) (void)hipHostFree(t->h_table);
    delete t;
}

int sparseloco_messages_bind(sparseloco_messages** out, const sparseloco_plan* plan, int n_replicas,
                             uint16_t* const* pairs, float* const* aux, void* stream) {
    if (!out) return SPLC_EINVAL;
    *out = nullptr;
    if (!plan || !pairs || !aux || n_replicas < 1 || n_replicas > SPLC_MAX_REPLICAS) return SPLC_EINVAL;
    for (int r = 0; r < n_replicas; ++r) {
        if (plan->n_chunks == 0) continue;
        if (!pairs[r] || !aux[r]) return SPLC_EINVAL;
        if (!aligned(pairs[r], 2) || !aligned(aux[r], 4)) return SPLC_EALIGN;
    }
    int rc = current_device_is(plan->device);
    if (rc != SPLC_OK) return rc;
    sparseloco_messages* m = new (std::nothrow) sparseloco_messages();
    if (!m) return SPLC_ENOMEM;
    m->device = plan->device;
    m->n_replicas = n_replicas;
    m->quant = plan->quant;
    m->kappa = plan->kappa;
    m->n_chunks = plan->n_chunks;
    const size_t nr = (size_t)n_replicas;
    if ((rc = upload_table(2 * nr, &m->h_table, &m->d_table)) == SPLC_OK) {
        for (size_t r = 0; r < nr; ++r) {
            m->h_table[r] = pairs[r];
            m->h_table[nr + r] = aux[r];
        }
        if (hipMemcpyAsync(m->d_table, m->h_table, 2 * nr * sizeof(void*), hipMemcpyHostToDevice,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
            rc = SPLC_EHIP;
    }
    if (rc != SPLC_OK) {
        sparseloco_messages_release(m);
        return rc;
    }
    *out = m;
    return SPLC_OK;
}

void sparseloco_messages_release(sparseloco_messages* m) {
    if (!m) return;
    if (m->d_table) (void)hipFree(m->d_table);
    if (m->h_table) (void)hipHostFree(m->h_table);
    delete m;
}

int sparseloco_compress(const sparseloco_plan* plan, int delta_mode, const sparseloco_tensors* src_a,
                        const sparseloco_tensors* src_b, const sparseloco_tensors* ef, int replica, float beta,
                        uint16_t* pairs_out, float* aux_out, void* stream) {
    if (!plan || !src_a || !ef || !pairs_out || !aux_out || replica < 0) return SPLC_EINVAL;
    int mode, rc;
    if (delta_mode == SPLC_DELTA_FROM_PARAMS) {
        if (!src_b) return SPLC_EINVAL;
        if ((rc = check_tensors(plan, src_a, SPLC_F32, 1)) != SPLC_OK) return rc;
        if ((rc = check_tensors(plan, src_b, SPLC_F32, 1)) != SPLC_OK) return rc;
        mode = MODE_PARAMS_F32;
    } else if (delta_mode == SPLC_DELTA_DIRECT) {
        if (src_b) return SPLC_EINVAL;
        if ((rc = check_tensors(plan, src_a, src_a->dtype, 1)) != SPLC_OK) return rc;
        mode = src_a->dtype == SPLC_BF16 ? MODE_DIRECT_BF16 : MODE_DIRECT_F32;
    } else {
        return SPLC_EINVAL;
    }
    if ((rc = check_tensors(plan, ef, SPLC_F32, 1)) != SPLC_OK) return rc;
    for (const sparseloco_tensors* t : {src_a, src_b, ef})
        if (t && t->n_sets > 1 && replica >= t->n_sets) return SPLC_EINVAL;
    if (!finite(beta)) return SPLC_EINVAL;
    if (!aligned(pairs_out, 2) || !aligned(aux_out, 4)) return SPLC_EALIGN;
    if ((rc = current_device_is(plan->device)) != SPLC_OK) return rc;
    if (plan->n_chunks == 0) return SPLC_OK;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const void* const* da = set_table<const void*>(src_a, replica);
    const void* const* db = src_b ? set_table<const void*>(src_b, replica) : nullptr;
    float* const* de = set_table<float*>(ef, replica);
    const bool q2 = plan->quant == SPLC_QUANT_2BIT;
    switch (mode) {
        case MODE_PARAMS_F32:
            if (q2) launch_compress<MODE_PARAMS_F32, SPLC_QUANT_2BIT>(plan, da, db, de, beta, pairs_out, aux_out, st);
            else launch_compress<MODE_PARAMS_F32, SPLC_QUANT_NONE>(plan, da, db, de, beta, pairs_out, aux_out, st);
            break;
        case MODE_DIRECT_F32:
            if (q2) launch_compress<MODE_DIRECT_F32, SPLC_QUANT_2BIT>(plan, da, db, de, beta, pairs_out, aux_out, st);
            else launch_compress<MODE_DIRECT_F32, SPLC_QUANT_NONE>(plan, da, db, de, beta, pairs_out, aux_out, st);
            break;
        default:
            if (q2) launch_compress<MODE_DIRECT_BF16, SPLC_QUANT_2BIT>(plan, da, db, de, beta, pairs_out, aux_out, st);
            else launch_compress<MODE_DIRECT_BF16, SPLC_QUANT_NONE>(plan, da, db, de, beta, pairs_out, aux_out, st);
            break;
    }
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

int sparseloco_compress_batch(const sparseloco_plan* plan, int n_replicas, const sparseloco_tensors* theta_outer,
                              const sparseloco_tensors* theta_local, const sparseloco_tensors* ef, float beta,
                              const sparseloco_messages* messages_out, void* stream) {
    return compress_batch_impl(plan, n_replicas, theta_outer, theta_local, ef, beta, messages_out, false, 0.f, nullptr, 0,
                               stream);
}

int sparseloco_outer_step_batch(const sparseloco_plan* plan, int n_replicas, const sparseloco_tensors* theta_outer,
                                const sparseloco_tensors* theta_local, const sparseloco_tensors* ef, float beta,
                                float outer_lr, const sparseloco_messages* messages_out,
                                const sparseloco_tensors* delta_bar_out, int reset_theta_local, void* stream) {
    return compress_batch_impl(plan, n_replicas, theta_outer, theta_local, ef, beta, messages_out, true, outer_lr,
                               delta_bar_out, reset_theta_local ? 1 : 0, stream);
}

int sparseloco_aggregate(const sparseloco_plan* plan, const sparseloco_messages* messages,
                         const sparseloco_tensors* delta_bar_out, void* stream) {
    return aggregate_impl(plan, messages, delta_bar_out, nullptr, 0.f, false, nullptr, stream);
}

int sparseloco_aggregate_update(const sparseloco_plan* plan, const sparseloco_messages* messages,
                                const sparseloco_tensors* theta_outer, float outer_lr,
                                const sparseloco_tensors* delta_bar_out, const sparseloco_tensors* theta_local_reset,
                                void* stream) {
    return aggregate_impl(plan, messages, delta_bar_out, theta_outer, outer_lr, true, theta_local_reset, stream);
}

int sparseloco_outer_update(const sparseloco_plan* plan, const sparseloco_tensors* theta_outer,
                            const sparseloco_tensors* delta_bar, float outer_lr, void* stream) {
    if (!plan) return SPLC_EINVAL;
    int rc;
    if ((rc = check_tensors(plan, theta_outer, SPLC_F32, 1)) != SPLC_OK) return rc;
    if ((rc = check_tensors(plan, delta_bar, SPLC_F32, 1)) != SPLC_OK) return rc;
    if (theta_outer->n_sets != 1 || delta_bar->n_sets != 1 || !finite(outer_lr)) return SPLC_EINVAL;
    if ((rc = current_device_is(plan->device)) != SPLC_OK) return rc;
    if (plan->n_chunks == 0) return SPLC_OK;
    hipLaunchKernelGGL(outer_update_kernel, dim3((unsigned)plan->n_update), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), plan->d_update, (unsigned)plan->n_update_gen,
                       set_table<float*>(theta_outer, 0), set_table<const float*>(delta_bar, 0), outer_lr);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

const char* sparseloco_strerror(int status) {
    switch (status) {
        case SPLC_OK: return "ok";
        case SPLC_EINVAL: return "invalid argument";
        case SPLC_EALIGN: return "tensor pointer not sufficiently aligned";
        case SPLC_ENOMEM: return "allocation failed";
        case SPLC_EHIP: return "HIP runtime call failed";
        case SPLC_EPLAN: return "call does not match the plan or a binding";
        case SPLC_ETOOBIG: return "problem exceeds the fixed workspace of this call";
        default: return "unknown status";
    }
}

}  // extern "C"

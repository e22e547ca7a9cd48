// Post-synchronisation token-embedding re-projection for gfx950 (paper section 2.4):
//
//     T_perp <- T_perp + (T_S - Pi_S(T_S)),   T_S <- Pi_S(T_S),   Pi_S(X) = X U U^T
//
// Two dense contractions, so this part does use the matrix cores: fp32 MFMA
// (v_mfma_f32_32x32x2_f32, fp32 accumulation), LDS-tiled, 128 x 128 output tile per
// 256-lane workgroup, each wave a 64 x 64 quarter (2 x 2 MFMA tiles).
//   pass 1:  C = T_S U                       (vocab x k, caller's workspace)
//   pass 2:  R = C U^T, fused with the update of T_perp and T_S (R is never stored separately)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparseloco.h"

namespace {

constexpr int TM = 128, TN = 128, TK = 16;
constexpr int PITCH = TM + 4;            // LDS row pitch in floats (TM == TN)
constexpr int kThreads = 256;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float vfloat4 __attribute__((ext_vector_type(4), aligned(4)));
#define SPLC_GLOBAL __attribute__((address_space(1)))

// Eight consecutive floats of row `row` starting at column `col` of a row-major matrix
// (rows x cols, leading dimension ld); zeros outside the matrix.
__device__ __forceinline__ void load8(const float* __restrict__ base, int64_t ld, int row, int col, int rows,
                                      int cols, float (&out)[8]) {
    if (row < rows && col + 8 <= cols) {
        const float* p = base + (int64_t)row * ld + col;
        vfloat4 a = *(const SPLC_GLOBAL vfloat4*)p;
        vfloat4 b = *(const SPLC_GLOBAL vfloat4*)(p + 4);
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            out[i] = (row < rows && col + i < cols) ? base[(int64_t)row * ld + col + i] : 0.f;
    }
}

// Epilogue of pass 1: store the coefficients.
struct StoreCoeff {
    float* c;
    int64_t ld;
    __device__ __forceinline__ void operator()(int row, int col, float v) const { c[(int64_t)row * ld + col] = v; }
};

// Epilogue of pass 2: v = Pi_S(T_S)[row][col].
struct UpdateEmbedding {
    float* t_s;
    float* t_perp;
    int64_t ld;
    __device__ __forceinline__ void operator()(int row, int col, float v) const {
        const int64_t at = (int64_t)row * ld + col;
        const float x = t_s[at];
        t_perp[at] = __fadd_rn(t_perp[at], __fsub_rn(x, v));
        t_s[at] = v;
    }
};

// C = A * B for row-major A (M x K, lda).  B_NK = false: B is row-major K x N (ldb).
// B_NK = true: B is given as its transpose, row-major N x K (ldb), i.e. B[k][n] = Bt[n][k].
// Every output element goes through epi(row, col, value).
template <bool B_NK, class Epi>
__global__ __launch_bounds__(kThreads) void gemm_f32_kernel(const float* __restrict__ A, int64_t lda,
                                                            const float* __restrict__ B, int64_t ldb, int M, int N,
                                                            int K, Epi epi) {
    __shared__ float As[2][TK][PITCH];
    __shared__ float Bs[2][TK][PITCH];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Staging assignment.  "Row-of-k" tiles (A always, B when given as N x K): lane t takes matrix
    // row t / 2 and eight consecutive k.  "k-major" tiles (B as K x N): lane t takes k = t / 16 and
    // eight consecutive n.
    const int ar = tid >> 1, ak = (tid & 1) * 8;
    const int bk = tid >> 4, bn = (tid & 15) * 8;
    float ra[8], rb[8];
    auto fetch = [&](int k0) {
        load8(A, lda, m0 + ar, k0 + ak, M, K, ra);
        if (B_NK) load8(B, ldb, n0 + ar, k0 + ak, N, K, rb);
        else load8(B, ldb, k0 + bk, n0 + bn, K, N, rb);
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) As[buf][ak + i][ar] = ra[i];
        if (B_NK) {
#pragma unroll
            for (int i = 0; i < 8; ++i) Bs[buf][ak + i][ar] = rb[i];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) Bs[buf][bk][bn + i] = rb[i];
        }
    };

    const int n_tiles = (K + TK - 1) / TK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < n_tiles) fetch((t + 1) * TK);
        // operand layout of v_mfma_f32_32x32x2_f32: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32]
        const int kq = lane >> 5, rc = lane & 31;
#pragma unroll
        for (int kk = 0; kk < TK; kk += 2) {
            const float a0 = As[buf][kk + kq][wm * 64 + rc], a1 = As[buf][kk + kq][wm * 64 + 32 + rc];
            const float b0 = Bs[buf][kk + kq][wn * 64 + rc], b1 = Bs[buf][kk + kq][wn * 64 + 32 + rc];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (t + 1 < n_tiles) stash(buf ^ 1);
        __syncthreads();
    }

    // result layout: register v of lane l holds D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int col = n0 + wn * 64 + j * 32 + (lane & 31);
                if (row < M && col < N) epi(row, col, acc[i][j][v]);
            }
}

bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

}  // namespace

extern "C" int sparseloco_reproject_embedding(float* t_s, float* t_perp, const float* u, float* coeff_ws,
                                              int64_t vocab, int d, int k, void* stream) {
    if (!t_s || !t_perp || !u || !coeff_ws) return SPLC_EINVAL;
    if (vocab < 0 || vocab > 0x7FFFFFFF - TM || d < 1 || k < 1 || k > d) return SPLC_EINVAL;
    if (!aligned4(t_s) || !aligned4(t_perp) || !aligned4(u) || !aligned4(coeff_ws)) return SPLC_EALIGN;
    if (vocab == 0) return SPLC_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int M = (int)vocab;
    // pass 1: coeff = T_S U            (M x k) = (M x d)(d x k)
    {
        dim3 grid((unsigned)((k + TN - 1) / TN), (unsigned)((M + TM - 1) / TM));
        hipLaunchKernelGGL((gemm_f32_kernel<false, StoreCoeff>), grid, dim3(kThreads), 0, st, t_s, (int64_t)d, u,
                           (int64_t)k, M, k, d, StoreCoeff{coeff_ws, (int64_t)k});
    }
    // pass 2: Pi = coeff U^T           (M x d) = (M x k)(k x d), U given as d x k = the N x K form
    {
        dim3 grid((unsigned)((d + TN - 1) / TN), (unsigned)((M + TM - 1) / TM));
        hipLaunchKernelGGL((gemm_f32_kernel<true, UpdateEmbedding>), grid, dim3(kThreads), 0, st, coeff_ws,
                           (int64_t)k, u, (int64_t)k, M, d, k, UpdateEmbedding{t_s, t_perp, (int64_t)d});
    }
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

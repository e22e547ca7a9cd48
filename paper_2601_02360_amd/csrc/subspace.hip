// Post-synchronisation token-embedding re-projection for gfx950 (paper section 2.4):
//
//     T_perp <- T_perp + (T_S - Pi_S(T_S)),   T_S <- Pi_S(T_S),   Pi_S(X) = X U U^T
//
// Two dense contractions, so this part does use the matrix cores: fp32 MFMA
// (v_mfma_f32_32x32x2_f32, fp32 accumulation), LDS-tiled, 128 x 128 output tile per
// 256-lane workgroup, each wave a 64 x 64 quarter (2 x 2 MFMA tiles); 64-row and 64-column
// tiles for the skinny shapes.
//   pass 1:  C = T_S U                       (vocab x k, caller's workspace)
//   pass 2:  R = C U^T, fused with the update of T_perp and T_S (R is never stored separately)
//
// The same GEMM kernel, with a prologue on its A operand or another epilogue, gives the compressed
// inter-stage traffic of section 2.2:
//     project      X~ = (X - T_perp[x] - PosEmbed) U        (also  grad_X U  with nothing subtracted)
//     reconstruct  X^ = X~ U^T + T_perp[x] + PosEmbed
// For a narrow basis (most of the subspace sizes the paper sweeps) these products are bound by memory
// traffic, not by the matrix pipe.  The GEMM kernel's 64 x 64 tile handles that well; where it does not
// (few or no tables to gather, small k), project_narrow_kernel takes over (16 x 16 x 4 MFMAs, operands
// loaded from global memory directly in MFMA layout, no barrier in the loop).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "sparseloco.h"

namespace {

constexpr int TM = 128, TK = 16;         // largest M tile (bounds the row counts accepted), K tile
constexpr int kThreads = 256;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t vuint4 __attribute__((ext_vector_type(4)));
typedef uint32_t vuint2 __attribute__((ext_vector_type(2)));

// How the fp32 products are formed.
//   MATH_F32:    v_mfma_f32_32x32x2_f32 on the operands as they are.
//   MATH_BF16X3: every fp32 operand is split exactly into three bf16 pieces, x = x0 + x1 + x2 (8 mantissa
//                bits each), and a product is the sum of the six piece products x_i y_j with i + j <= 2 on
//                v_mfma_f32_32x32x16_bf16, accumulated in fp32.  A piece product is exact in fp32; the three
//                dropped terms are below 2^-23 |x y|, the size of an fp32 rounding step.  The bf16 matrix
//                pipe is 16 times as fast as the fp32 one, so six products still cost less than half of one
//                fp32 product.
enum { MATH_F32 = 0, MATH_BF16X3 = 1 };

// The three bf16 pieces of x as bit patterns in the upper halves of h[0..2] (truncating splits: every
// subtraction is exact, and x == h0 + h1 + h2 exactly for a normal fp32 x).
__device__ __forceinline__ void split3(float x, uint32_t (&h)[3]) {
    h[0] = __float_as_uint(x) & 0xFFFF0000u;
    const float r1 = __fsub_rn(x, __uint_as_float(h[0]));
    h[1] = __float_as_uint(r1) & 0xFFFF0000u;
    h[2] = __float_as_uint(__fsub_rn(r1, __uint_as_float(h[1])));
}
// Two bf16 values (upper halves of lo and hi) as one dword, lo in the lower half.
__device__ __forceinline__ uint32_t pack_bf16(uint32_t lo, uint32_t hi) {
    return __builtin_amdgcn_perm(hi, lo, 0x07060302u);
}
typedef float vfloat4 __attribute__((ext_vector_type(4), aligned(4)));
#define SPLC_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ vfloat4 ldg4(const float* p) { return *(const SPLC_GLOBAL vfloat4*)p; }
__device__ __forceinline__ void stg4(float* p, vfloat4 v) { *(SPLC_GLOBAL vfloat4*)p = v; }
// The same for data that this call touches exactly once (the tables the re-projection updates, reconstructed
// activations): non-temporal, so that they do not displace the basis and the coefficients from the caches.
__device__ __forceinline__ vfloat4 ldg4_once(const float* p) {
    return __builtin_nontemporal_load((const SPLC_GLOBAL vfloat4*)p);
}
__device__ __forceinline__ void stg4_once(float* p, vfloat4 v) { __builtin_nontemporal_store(v, (SPLC_GLOBAL vfloat4*)p); }

// F (4 or 8) consecutive floats row[col .. col + F - 1] of a matrix row with `cols` columns, into out[0 .. F-1].
// GUARD = false: the caller knows that they all exist -- plain 16-byte loads, no branch (the compiler can then
// count the loads in flight and wait for the oldest alone).  GUARD = true: element by element, zeros from
// column `cols` on, 16-byte loads where a lane's values all exist (the K tail, and the workgroups on the right
// edge of B).
template <int F, bool GUARD>
__device__ __forceinline__ void row_load(const float* __restrict__ row, int col, int cols, float (&out)[8]) {
    if (!GUARD) {
        const vfloat4 a = ldg4(row + col);
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        if (F == 8) {
            const vfloat4 b = ldg4(row + col + 4);
            out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
        }
    } else if (col + F <= cols) {
        row_load<F, false>(row, col, cols, out);
    } else {
#pragma unroll
        for (int i = 0; i < F; ++i) out[i] = col + i < cols ? row[col + i] : 0.f;
    }
}


// Epilogues receive four consecutive columns of one output row (col is a multiple of 4).  Two forms:
// operator() for a tile on the edge of the output (columns at or beyond n_cols do not exist), and, for a
// tile that lies wholly inside, load() + store(): the kernel issues the loads of all its pieces of a
// 32-row slab before the slab goes through LDS, so that their latency hides behind that round trip
// instead of being paid piece by piece.

// Pass 1: store the coefficients.
struct StoreCoeff {
    static constexpr bool kStaggeredStart = false;
    float* c;
    int64_t ld;
    __device__ __forceinline__ void load(int, int, vfloat4 (&)[2]) const {}
    __device__ __forceinline__ void store(int row, int col, vfloat4 v, const vfloat4 (&)[2]) const {
        stg4(c + (int64_t)row * ld + col, v);
    }
    __device__ __forceinline__ void operator()(int row, int col, vfloat4 v, int n_cols) const {
        float* p = c + (int64_t)row * ld + col;
        if (col + 4 <= n_cols) {
            stg4(p, v);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (col + i < n_cols) p[i] = v[i];
        }
    }
};

// Pass 2: v = Pi_S(T_S)[row][col .. col+3].
struct UpdateEmbedding {
    // This epilogue moves four arrays; a kernel that carries it is as much bound by memory as by the matrix
    // pipe, and gains when the workgroups that share a compute unit are not all in their epilogue at once.
    static constexpr bool kStaggeredStart = true;
    float* t_s;
    float* t_perp;
    int64_t ld;
    int compute_units;       // of the device, for the staggered start
    __device__ __forceinline__ void load(int row, int col, vfloat4 (&r)[2]) const {
        const int64_t at = (int64_t)row * ld + col;
        r[0] = ldg4_once(t_s + at);
        r[1] = ldg4_once(t_perp + at);
    }
    __device__ __forceinline__ void store(int row, int col, vfloat4 v, const vfloat4 (&r)[2]) const {
        const int64_t at = (int64_t)row * ld + col;
        vfloat4 q;
#pragma unroll
        for (int i = 0; i < 4; ++i) q[i] = __fadd_rn(r[1][i], __fsub_rn(r[0][i], v[i]));
        stg4_once(t_perp + at, q);
        stg4_once(t_s + at, v);
    }
    __device__ __forceinline__ void operator()(int row, int col, vfloat4 v, int n_cols) const {
        const int64_t at = (int64_t)row * ld + col;
        if (col + 4 <= n_cols) {
            const vfloat4 x = ldg4(t_s + at), p = ldg4(t_perp + at);
            vfloat4 q;
#pragma unroll
            for (int i = 0; i < 4; ++i) q[i] = __fadd_rn(p[i], __fsub_rn(x[i], v[i]));
            stg4(t_perp + at, q);
            stg4(t_s + at, v);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (col + i < n_cols) {
                    t_perp[at + i] = __fadd_rn(t_perp[at + i], __fsub_rn(t_s[at + i], v[i]));
                    t_s[at + i] = v[i];
                }
        }
    }
};

// The high-rank part of an activation row (section 2.2): T_perp[token of the row] + PosEmbed[position of
// the row]; either table may be absent.  Rows are tokens of a [batch, seq_len, d] tensor, so the position
// of row r is r % seq_len.  Token ids are clamped into the table.
struct HighRank {
    const float* t_perp;     // [vocab, d] or nullptr
    const int32_t* token;    // [rows] (required with t_perp)
    int vocab;
    const float* pos;        // [seq_len, d] or nullptr
    int seq_len;
    int64_t ld;              // d
    __device__ __forceinline__ const float* perp_row(int row) const {
        int t = token[row];
        t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
        return t_perp + (int64_t)t * ld;
    }
    __device__ __forceinline__ const float* pos_row(int row) const { return pos + (int64_t)(row % seq_len) * ld; }
};

// A-operand prologues.  fetch() issues the loads of whatever is combined with F values (row, col .. col+F-1)
// of A; apply() combines them when the values go to LDS, one K tile later -- kept apart so that a tile's
// loads stay in flight while the previous tile is multiplied.  prepare() is called once per lane with the
// (valid) matrix row that the lane stages.
struct NoPrologue {
    static constexpr int kTables = 0;
    __device__ __forceinline__ void prepare(int) {}
    template <int F, bool GUARD>
    __device__ __forceinline__ void fetch(int, int, float (&)[2][8]) const {}
    template <int F>
    __device__ __forceinline__ void apply(float (&)[8], const float (&)[2][8]) const {}
};
// v <- fl(fl(v - T_perp[x]) - PosEmbed); TP / PE: which of the two tables exist (compile time, so that the
// number of loads per tile is fixed).
template <bool TP, bool PE>
struct SubtractHighRank {
    static constexpr int kTables = (TP ? 1 : 0) + (PE ? 1 : 0);
    HighRank h;
    const float* tabs[2];        // this lane's T_perp row and positional row: the token lookup leaves the K loop
    __device__ __forceinline__ void prepare(int row) {
        tabs[0] = TP ? h.perp_row(row) : nullptr;
        tabs[1] = PE ? h.pos_row(row) : nullptr;
    }
    template <int F, bool GUARD>
    __device__ __forceinline__ void fetch(int col, int cols, float (&t)[2][8]) const {
        if (TP) row_load<F, GUARD>(tabs[0], col, cols, t[0]);
        if (PE) row_load<F, GUARD>(tabs[1], col, cols, t[1]);
    }
    template <int F>
    __device__ __forceinline__ void apply(float (&v)[8], const float (&t)[2][8]) const {
        if (TP) {
#pragma unroll
            for (int i = 0; i < F; ++i) v[i] = __fsub_rn(v[i], t[0][i]);
        }
        if (PE) {
#pragma unroll
            for (int i = 0; i < F; ++i) v[i] = __fsub_rn(v[i], t[1][i]);
        }
    }
};

// Epilogue of reconstruct: out <- fl(fl(v + T_perp[x]) + PosEmbed); TP / PE: which tables exist.
template <bool TP, bool PE>
struct AddHighRank {
    static constexpr bool kStaggeredStart = false;     // measured: no gain for the reconstruction
    HighRank h;
    float* out;
    __device__ __forceinline__ void load(int row, int col, vfloat4 (&r)[2]) const {
        if (TP) r[0] = ldg4(h.perp_row(row) + col);
        if (PE) r[1] = ldg4(h.pos_row(row) + col);
    }
    __device__ __forceinline__ void store(int row, int col, vfloat4 v, const vfloat4 (&r)[2]) const {
        if (TP) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = __fadd_rn(v[i], r[0][i]);
        }
        if (PE) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = __fadd_rn(v[i], r[1][i]);
        }
        stg4_once(out + (int64_t)row * h.ld + col, v);
    }
    __device__ __forceinline__ void operator()(int row, int col, vfloat4 v, int n_cols) const {
        if (col + 4 <= n_cols) {
            vfloat4 r[2];
            load(row, col, r);
            store(row, col, v, r);
        } else {
            float* p = out + (int64_t)row * h.ld + col;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (col + i < n_cols) {
                    float x = v[i];
                    if (TP) x = __fadd_rn(x, h.perp_row(row)[col + i]);
                    if (PE) x = __fadd_rn(x, h.pos_row(row)[col + i]);
                    p[i] = x;
                }
        }
    }
};

// C = A * B for row-major A (M x K, lda).  B_NK = false: B is row-major K x N (ldb).
// B_NK = true: B is given as its transpose, row-major N x K (ldb), i.e. B[k][n] = Bt[n][k].
// The A values pass through pro(row, col, M, K, values[8]) on their way in; the output goes
// through epi(row, col, four values, N).
// Waves per SIMD the register allocation must leave room for: the 128 x 128 tile holds 64 accumulator
// registers, and a prologue with tables keeps up to 32 more values in flight per lane.
template <int MATH, int TM_, int TN_, class Pro>
constexpr int gemm_min_waves() {
    return (TM_ * TN_ == 128 * 128 ? 3 : 4) - (Pro::kTables > 0 ? 1 : 0) - (MATH == MATH_BF16X3 ? 1 : 0);
}

// Staging buffers of one workgroup, two K tiles deep.
//   MATH_F32:    k-major fp32 tiles with a padded pitch (operands are read one float per lane).
//   MATH_BF16X3: per operand three planes (one per bf16 piece) of rows of 16 k = 32 bytes; a lane reads the 16
//                bytes of one half row, and the halves of rows 8..15 (mod 16) are swapped so that sixteen
//                consecutive rows cover all LDS banks.
template <int MATH, int TM_, int TN_>
struct GemmStaging;
template <int TM_, int TN_>
struct GemmStaging<MATH_F32, TM_, TN_> {
    // Pitch of a tile staged "row of k" (A always, B when given as N x K): rows + 2.  The lanes that share a
    // matrix row store k values TK / (lanes per row) apart, i.e. 8 (4) pitches apart for the 128 (64) row
    // tile; with a pitch = 2 mod 8 these land 16 (8) banks apart and a store instruction is free of bank
    // conflicts.  The operand reads (consecutive rows of one k per half wave) are conflict free at any pitch.
    static constexpr int kPitchA = TM_ + 2, kPitchBRows = TN_ + 2;
    float a[2][TK][kPitchA];
    float b[2][TK][TN_ + 4];       // K x N tiles and the epilogue slab use this pitch; N x K tiles use kPitchBRows
};
template <int TM_, int TN_>
struct GemmStaging<MATH_BF16X3, TM_, TN_> {
    uint32_t a[2][3][TM_][8];
    uint32_t b[2][3][TN_][8];
};

template <int MATH, int TM_, int TN_, bool B_NK, class Pro, class Epi>
__global__ __launch_bounds__(kThreads, (gemm_min_waves<MATH, TM_, TN_, Pro>())) void gemm_kernel(
    const float* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb, int M, int N, int K, Pro pro,
    Epi epi) {
    // TM_ x TN_ output tile; the four waves form a 2 x 2 grid, each with MI x NJ MFMA tiles of 32 x 32
    // (128 x 128: 2 x 2 per wave; the smaller tiles give small problems more workgroups and waste less of
    // the last column tile when N is a multiple of 64 only).
    static_assert((TM_ == 128 || TM_ == 64) && (TN_ == 128 || TN_ == 64), "supported tiles");
    constexpr bool SPLIT = MATH == MATH_BF16X3;
    constexpr int MI = TM_ / 64, NJ = TN_ / 64;
    constexpr int AF = TM_ / 16, BF = TN_ / 16;      // floats of the A / B tile per lane: 8 or 4
    constexpr int PB = TN_ + 4;                      // row pitch of the epilogue slab (and of the fp32 B tile)
    __shared__ __attribute__((aligned(16))) GemmStaging<MATH, TM_, TN_> sm;
    static_assert(sizeof(sm.b) >= sizeof(float) * 32 * PB, "the epilogue slab reuses the B staging buffers");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    // Workgroups are handed to the eight XCDs round-robin by their linear number, and each XCD has an L2 of
    // its own.  The column tiles of one row block all read the same rows of A, so they are given numbers that
    // land on one XCD: XCD x takes the row blocks x, x + 8, ..., each with all of its column tiles in turn.
    // (The grid is one-dimensional and padded to a multiple of eight row blocks; the surplus groups leave.)
    const int col_tiles = (N + TN_ - 1) / TN_;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int row_block = (slot / col_tiles) * 8 + xcd;
    const int m0 = row_block * TM_, n0 = (slot % col_tiles) * TN_;
    if (m0 >= M) return;
    if constexpr (Epi::kStaggeredStart) {
        // The workgroups that start together on a compute unit run the same K loop and would then all reach
        // the memory-heavy epilogue together, leaving the matrix pipe idle meanwhile, round after round.  The
        // first batch of workgroups is therefore started a fraction of a tile apart: the r-th workgroup to land
        // on a compute unit (workgroups are dealt out one per unit before any unit gets its second) sleeps
        // r / R of one workgroup's lifetime, R = resident workgroups per unit; later ones inherit the phase of
        // the slot they take over.  A lifetime is about R times the K loop's matrix-pipe time,
        // n_tiles * 512 MI NJ cycles; s_sleep(127) is 8128 cycles.  Measured on the second pass of the
        // re-projection at 32000 x 2048, k = 256: 356 -> 322 us.
        constexpr int R = gemm_min_waves<MATH, TM_, TN_, Pro>();
        const int first = epi.compute_units * R;
        if ((int)blockIdx.x < first) {
            const int r = (int)blockIdx.x / epi.compute_units;
            const int sleeps = r * ((K + TK - 1) / TK) * (MI * NJ) / 16;
            for (int i = 0; i < sleeps; ++i) __builtin_amdgcn_s_sleep(127);
        }
    }

    v16f acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Staging assignment.  "Row-of-k" tiles (A always, B when given as N x K): a lane takes one matrix
    // row and AF (A) or BF (B) consecutive k.  "k-major" tiles (B as K x N): lane t takes k = t / 16 and
    // BF consecutive n.  A lane whose row lies beyond the matrix stages the last row instead: it only
    // feeds output rows (columns) that are never stored.
    // With split operands every tile is staged row-of-k (the MFMA wants eight consecutive k per lane), so for B
    // as K x N a lane then takes one column n = t % TN_ and loads its BF values of k one by one, each load
    // coalesced across the lanes.
    constexpr bool B_ROWS = B_NK || SPLIT;
    const int ar = tid / (TK / AF), ak = (tid % (TK / AF)) * AF;
    const int br = (SPLIT && !B_NK) ? tid % TN_ : tid / (TK / BF);
    const int bkk = (SPLIT && !B_NK) ? (tid / TN_) * BF : (tid % (TK / BF)) * BF;
    const int bk = tid >> 4, bn = (tid & 15) * BF;
    const int arow = m0 + ar < M ? m0 + ar : M - 1;
    const int brow = n0 + br < N ? n0 + br : N - 1;
    const float* const pa = A + (int64_t)arow * lda;
    // B as K x N: columns at and beyond N only feed outputs that are never stored, so whatever is read for
    // them will do.  A lane whose BF columns lie wholly beyond N reads columns 0 .. BF-1 instead; a lane that
    // straddles N reads on into the next row of B, which exists for every K tile but the last few rows
    // (see n_fast below).
    const int bcol = n0 + bn;
    const float* const pb = B_NK ? B + (int64_t)brow * ldb : (SPLIT ? B + brow : B + (bcol < N ? bcol : 0));
    pro.prepare(arow);

    // One K tile on its way from global memory to LDS: raw A values, what the prologue combines with them, B.
    struct Stage { float a[8], b[8], t[2][8]; };
    Stage s0, s1;
    // GUARD = false needs the whole K tile inside the matrix (and, for B as K x N, spare rows behind it).
    auto fetch = [&](auto guard, int k0, Stage& q) {
        constexpr bool GUARD = decltype(guard)::value;
        row_load<AF, GUARD>(pa, k0 + ak, K, q.a);
        pro.template fetch<AF, GUARD>(k0 + ak, K, q.t);
        if (B_NK) {
            row_load<BF, GUARD>(pb, k0 + bkk, K, q.b);
        } else if (SPLIT) {
#pragma unroll
            for (int i = 0; i < BF; ++i) {
                const int kk = k0 + bkk + i;
                q.b[i] = (!GUARD || kk < K) ? pb[(int64_t)(GUARD ? (kk < K ? kk : 0) : kk) * ldb] : 0.f;
            }
        } else if (!GUARD) {
            row_load<BF, false>(pb + (int64_t)(k0 + bk) * ldb, 0, BF, q.b);
        } else {
            // zeros beyond row K and beyond column N
            const bool k_inside = k0 + bk < K;
            row_load<BF, true>(B + (int64_t)(k_inside ? k0 + bk : 0) * ldb + (bcol < N ? bcol : 0), 0,
                               k_inside ? N - bcol : 0, q.b);
        }
    };
    // F consecutive k (starting at k = kfirst, a multiple of F) of one tile row, split and stored plane by plane
    auto stash_split = [&](uint32_t (*plane0)[8], int plane_rows, int row, int kfirst, const float (&v)[8], auto fcount) {
        constexpr int F = decltype(fcount)::value;
        uint32_t h[8][3];
#pragma unroll
        for (int i = 0; i < F; ++i) split3(v[i], h[i]);
        const int half = (kfirst >> 3) ^ ((row >> 3) & 1);
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            uint32_t* dst = &plane0[p * plane_rows + row][4 * half + ((kfirst & 7) >> 1)];
            if (F == 8)
                *reinterpret_cast<vuint4*>(dst) = vuint4{pack_bf16(h[0][p], h[1][p]), pack_bf16(h[2][p], h[3][p]),
                                                         pack_bf16(h[4][p], h[5][p]), pack_bf16(h[6][p], h[7][p])};
            else
                *reinterpret_cast<vuint2*>(dst) = vuint2{pack_bf16(h[0][p], h[1][p]), pack_bf16(h[2][p], h[3][p])};
        }
    };
    // fp32 B tile given as N x K: same memory as sm.b, pitch kPitchBRows
    auto b_rows = [&](int buf, int k, int n) -> float& {
        if constexpr (SPLIT) {
            return *reinterpret_cast<float*>(&sm.b[0][0][0][0]);        // not used with split operands
        } else {
            return reinterpret_cast<float*>(&sm.b[buf][0][0])[k * GemmStaging<MATH, TM_, TN_>::kPitchBRows + n];
        }
    };
    auto stash = [&](int buf, Stage& q) {
        pro.template apply<AF>(q.a, q.t);
        if constexpr (SPLIT) {
            stash_split(&sm.a[buf][0][0], TM_, ar, ak, q.a, std::integral_constant<int, AF>{});
            stash_split(&sm.b[buf][0][0], TN_, br, bkk, q.b, std::integral_constant<int, BF>{});
        } else {
#pragma unroll
            for (int i = 0; i < AF; ++i) sm.a[buf][ak + i][ar] = q.a[i];
            if (B_NK) {
#pragma unroll
                for (int i = 0; i < BF; ++i) b_rows(buf, bkk + i, br) = q.b[i];
            } else {
#pragma unroll
                for (int i = 0; i < BF; ++i) sm.b[buf][bk][bn + i] = q.b[i];
            }
        }
    };
    // operand layout of v_mfma_f32_32x32x2_f32: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32].
    // The operands of the next k pair are read from LDS before the MFMAs of the current pair are
    // issued, so that the LDS latency hides behind the matrix pipe.
    // With split operands: v_mfma_f32_32x32x16_bf16 takes from lane l the eight k = 8 (l / 32) .. + 7 of row
    // (column) l % 32 -- one 16-byte half row of a plane -- and one K tile is one such MFMA per piece pair.
    auto multiply = [&](int buf) {
        const int kq = lane >> 5, rc = lane & 31;
        if constexpr (SPLIT) {
            bf16x8 pa_[3][MI], pb_[3][NJ];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int row = wm * (32 * MI) + 32 * i + rc;
                    pa_[p][i] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const vuint4*>(&sm.a[buf][p][row][4 * (kq ^ ((row >> 3) & 1))]));
                }
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int row = wn * (32 * NJ) + 32 * j + rc;
                    pb_[p][j] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const vuint4*>(&sm.b[buf][p][row][4 * (kq ^ ((row >> 3) & 1))]));
                }
            }
            // smallest terms first
            constexpr int pairs[6][2] = {{2, 0}, {1, 1}, {0, 2}, {1, 0}, {0, 1}, {0, 0}};
#pragma unroll
            for (int c = 0; c < 6; ++c)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa_[pairs[c][0]][i], pb_[pairs[c][1]][j],
                                                                            acc[i][j], 0, 0, 0);
        } else {
        float fa[2][MI], fb[2][NJ];
        auto operands = [&](int kk, int st) {
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[st][i] = sm.a[buf][kk + kq][wm * (32 * MI) + 32 * i + rc];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int col = wn * (32 * NJ) + 32 * j + rc;
                fb[st][j] = B_NK ? b_rows(buf, kk + kq, col) : sm.b[buf][kk + kq][col];
            }
        };
        operands(0, 0);
#pragma unroll
        for (int p = 0; p < TK / 2; ++p) {
            const int st = p & 1;
            if (p + 1 < TK / 2) operands(2 * (p + 1), st ^ 1);
            __builtin_amdgcn_sched_barrier(0);      // keep the reads above ahead of the MFMAs below
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[st][i], fb[st][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        }
    };

    // Global loads run two K tiles ahead of the MFMAs (one tile of matrix work is shorter than the memory
    // latency): tile t+2 is fetched into one register set while tile t is multiplied and tile t+1, fetched one
    // iteration earlier, goes from the other set to LDS.  The leading n_fast tiles need no guard; their loop
    // is branch-free between the barriers, which lets the wait before the LDS stores name the older tile
    // alone.  What is left (a K tail, the last two tiles) goes through the guarded loop.
    const std::integral_constant<bool, false> plain;
    const std::integral_constant<bool, true> guarded;
    const int n_tiles = (K + TK - 1) / TK;
    // Rows of B that must follow a tile for the reads past column N to stay inside the array (none if no lane
    // straddles N: then every 16-byte read lies inside its row).
    const int64_t spare_rows = (B_ROWS || n0 + TN_ <= N || N % BF == 0) ? 0 : (BF - 1 + ldb - 1) / ldb;
    const int n_fast = K >= spare_rows ? (int)((K - spare_rows) / TK) : 0;
    auto fetch_any = [&](int t, Stage& q) {
        if (t < n_fast) fetch(plain, t * TK, q);
        else fetch(guarded, t * TK, q);
    };
    fetch_any(0, s0);
    stash(0, s0);
    if (n_tiles > 1) fetch_any(1, s0);
    __syncthreads();
    int t = 0;
    for (; t + 3 < n_fast; t += 2) {          // t is even here: tile t sits in LDS buffer 0
        fetch(plain, (t + 2) * TK, s1);
        multiply(0);
        stash(1, s0);
        __syncthreads();
        fetch(plain, (t + 3) * TK, s0);
        multiply(1);
        stash(0, s1);
        __syncthreads();
    }
    for (; t < n_tiles; ++t) {
        const int buf = t & 1;
        if (t + 2 < n_tiles) fetch_any(t + 2, s1);
        multiply(buf);
        if (t + 1 < n_tiles) stash(buf ^ 1, s0);
        s0 = s1;
        __syncthreads();
    }

    // Epilogue through LDS, 32 output rows at a time, so that global memory sees whole rows
    // (16 bytes per lane, 4 TN_ bytes per row) instead of the MFMA result layout, in which register v
    // of lane l holds D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32].  The slab reuses the B staging
    // buffers (same size); the K loop ended with a barrier, so they are free.
    float* slab = reinterpret_cast<float*>(&sm.b);
    const bool inside = m0 + TM_ <= M && n0 + TN_ <= N;      // the whole output tile exists
#pragma unroll
    for (int s = 0; s < TM_ / 32; ++s) {
        if (wm == s / MI) {
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    slab[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * PB + wn * (32 * NJ) + j * 32 + (lane & 31)] =
                        acc[s % MI][j][v];
        }
        constexpr int VPR = TN_ / 4;                // 16-byte pieces per slab row
        constexpr int NQ = 32 * VPR / kThreads;     // pieces per lane
        vfloat4 held[NQ][2];
        if (inside) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int f = tid + kThreads * q;
                epi.load(m0 + 32 * s + f / VPR, n0 + (f % VPR) * 4, held[q]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int f = tid + kThreads * q;
            const int r = f / VPR, c4 = (f % VPR) * 4;
            const int row = m0 + 32 * s + r, col = n0 + c4;
            const float* src = slab + r * PB + c4;
            const vfloat4 v = {src[0], src[1], src[2], src[3]};
            if (inside) epi.store(row, col, v, held[q]);
            else if (row < M && col < N) epi(row, col, v, N);
        }
        __syncthreads();
    }
}

// Projection onto a narrow basis: out[rows, k] = (x - T_perp[token] - PosEmbed) U with k <= 16 * NB
// (section 2.2; the subspace dimensions the paper sweeps go down to d/768).  Instantiated for NB = 1, 2.
// With so few output columns the product is bound by reading x (and the gathered table rows) once, not
// by the matrix pipe, and the wide GEMM tile above would spend most of its MFMAs on columns that do not
// exist.  So: v_mfma_f32_16x16x4_f32, one workgroup per 16 rows, and the four waves split the reduction
// dimension between them (wave w takes the 32-wide d tiles w, w + 4, ...), which gives four times the
// waves to keep HBM busy.  Inside the loop a wave synchronises with nobody:
//   * its x / table values go from global memory straight into the A operand layout.  Lane (g, c)
//     (g = lane / 16, c = lane % 16) loads four consecutive floats d0 + 4g .. 4g + 3 of row c; MFMA step
//     s then multiplies the set {d0 + 4g + s}, a permutation of a group of sixteen d that the B operand
//     follows -- a sum does not care which four d share a step;
//   * its own U tile (32 x k floats, L2 resident) goes through a private, double-buffered LDS slab whose
//     row pitch 16 NB + 4 makes the operand reads (rows 4g + s, columns c) conflict free.
// PD tiles of A loads are in flight per wave.  At the end the four partial sums meet in LDS and are
// added in wave order, so the result does not depend on timing.
// d must be a multiple of 32 (whole tiles: no load needs a guard); other d go to the general kernel.
// TP / PE: a T_perp table / a positional table is subtracted.  They are template parameters, not run-time
// tests, so that the number of loads in flight is known at every point of the loop and a wait can name
// the oldest load instead of draining the queue.
template <int NB, int PD, bool TP, bool PE>
__global__ __launch_bounds__(kThreads, NB == 1 ? 4 : (NB == 2 ? 3 : 2)) void project_narrow_kernel(
    const float* __restrict__ x, HighRank h, const float* __restrict__ u, float* __restrict__ out, int rows, int d,
    int k) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    constexpr int KT = 32;                       // d values per tile: one 128-byte line of every row
    constexpr int KP = 16 * NB + 4;              // LDS pitch of a U tile row
    constexpr int NLD = KT * 16 * NB / 256;      // 16-byte load instructions per U tile
    static_assert(PD == 2 || PD == 4, "the LDS buffer parity follows the stage index");
    __shared__ __attribute__((aligned(16))) float slab[4][2][KT * KP];
    static_assert(sizeof(float) * 4 * 2 * KT * KP >= sizeof(float) * 4 * NB * 256, "partial sums reuse the slab");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // tile indices stay in scalar registers
    const int g = lane >> 4, c = lane & 15;
    const int r0 = blockIdx.x * 16;
    const int row = r0 + c < rows ? r0 + c : rows - 1;         // rows past the end repeat the last one; never stored
    const float* const px = x + (int64_t)row * d + 4 * g;
    const float* const pt = TP ? h.perp_row(row) + 4 * g : nullptr;
    const float* const pp = PE ? h.pos_row(row) + 4 * g : nullptr;
    const int n_tiles = d / KT;

    struct Stage { vfloat4 x[2], t[2], p[2]; };
    Stage st[PD];
    vfloat4 ur[NLD];
    v4f acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = v4f{0.f, 0.f, 0.f, 0.f};

    auto fetch_a = [&](int t, Stage& q) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int at = t * KT + 16 * hh;
            q.x[hh] = ldg4(px + at);
            if (TP) q.t[hh] = ldg4(pt + at);
            if (PE) q.p[hh] = ldg4(pp + at);
        }
    };
    // A U tile -- 32 rows of k floats -- is one contiguous run of 32 k floats in memory (16-byte aligned when U
    // is) whatever k is, so it is loaded flat, four floats per lane and instruction, and each float finds its
    // (row, column) slot of the padded slab by a division by k (multiply-high with a reciprocal that is exact
    // for the 2048 positions of a tile).  A lane whose position lies beyond the tile (k < 16 NB) loads the
    // tile's first floats instead and stores nothing.
    const uint32_t kinv = ((1u << 20) + (uint32_t)k - 1) / (uint32_t)k;
    const uint32_t tile_floats = (uint32_t)(KT * k);
    auto fetch_u = [&](int t) {
        const float* base = u + (int64_t)t * tile_floats;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const uint32_t f = 4 * (lane + 64 * i);
            // a basis of this column-block count has more than 16 (NB - 1) columns, which puts the first
            // 2 (NB - 1) loads of every lane inside the tile
            ur[i] = ldg4(base + ((i < 2 * (NB - 1) || f < tile_floats) ? f : 0u));
        }
    };
    const bool k_by_4 = (k & 3) == 0;             // then the four floats of a load share a row of U
    auto stash_u = [&](int buf) {
        float* const tile_base = &slab[wave][buf][0];
        // Lanes beyond the tile store too -- into the four padding floats at the end of a slab row, which
        // nobody reads: a store under a condition would drag its load into the conditional block, and the
        // wait for that load with it.
        float* const spare = tile_base + (lane & 31) * KP + 16 * NB;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            uint32_t f = 4 * (lane + 64 * i);
            asm volatile("" : "+v"(f));           // recompute the slot every time instead of keeping NLD addresses live
            const bool inside = i < 2 * (NB - 1) || f < tile_floats;
            const uint32_t r = (f * kinv) >> 20;
            uint32_t col = f - r * (uint32_t)k;
            float* dst = tile_base + r * KP + col;
            if (k_by_4) {
                *reinterpret_cast<v4f*>(inside ? dst : spare) = v4f{ur[i][0], ur[i][1], ur[i][2], ur[i][3]};
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    *(inside ? dst : spare + j) = ur[i][j];
                    ++col;
                    dst += col == (uint32_t)k ? KP - k + 1 : 1;
                    col = col == (uint32_t)k ? 0 : col;
                }
            }
        }
    };
    auto multiply = [&](const Stage& q, int buf) {
        // all B operands of the tile are requested from LDS before the first MFMA, so that the matrix pipe
        // does not wait for them one pair at a time
        const float* b0 = &slab[wave][buf][4 * g * KP + c];
        float b[2][4][NB];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) b[hh][s][nb] = b0[(16 * hh + s) * KP + 16 * nb];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            vfloat4 a = q.x[hh];
            if (TP) {
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = __fsub_rn(a[i], q.t[hh][i]);
            }
            if (PE) {
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = __fsub_rn(a[i], q.p[hh][i]);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[hh][s][nb], acc[nb], 0, 0, 0);
        }
    };

    // Wave w owns the n_mine tiles w, w + 4, ...; its i-th tile uses A stage i % PD and LDS buffer i % 2.
    // Inside the loop every load is issued unconditionally -- near the end it simply repeats the last tile,
    // whose data nobody uses -- for the same reason as above: a known number of loads in flight.
    const int n_mine = wave < n_tiles ? (n_tiles - wave + 3) >> 2 : 0;
    const int t_last = wave + 4 * (n_mine - 1);
    auto tile = [&](int i) { const int t = wave + 4 * i; return t < t_last ? t : t_last; };
    auto step = [&](int i, int j) {
        // After this tile's products are issued, the next tile's U -- requested one iteration ago -- moves to
        // the other LDS buffer (whose reads were issued an iteration ago; a wave's LDS operations keep their
        // order), and the tile after that starts its way from L2.
        multiply(st[j], j & 1);
        stash_u((j & 1) ^ 1);
        fetch_u(tile(i + 2));
        fetch_a(tile(i + PD), st[j]);
    };
    if (n_mine > 0) {
        fetch_u(wave);
#pragma unroll
        for (int j = 0; j < PD; ++j) fetch_a(tile(j), st[j]);
        stash_u(0);
        fetch_u(tile(1));
        int i = 0;
        for (; i + PD <= n_mine; i += PD) {
#pragma unroll
            for (int j = 0; j < PD; ++j) step(i + j, j);
        }
#pragma unroll
        for (int j = 0; j < PD - 1; ++j)
            if (i + j < n_mine) step(i + j, j);
    }

    // D layout of the 16 x 16 MFMA: register v of lane l holds row 4 (l / 16) + v, column l % 16.
    __syncthreads();
    float* part = &slab[0][0][0];                 // [wave][nb][row][col]
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[((wave * NB + nb) * 16 + 4 * g + v) * 16 + c] = acc[nb][v];
    __syncthreads();
    const int orow = tid >> 4, oc = tid & 15;
    if (r0 + orow < rows) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int col = 16 * nb + oc;
            if (col < k) {
                float sum = part[((0 * NB + nb) * 16 + orow) * 16 + oc];
#pragma unroll
                for (int w = 1; w < 4; ++w) sum = __fadd_rn(sum, part[((w * NB + nb) * 16 + orow) * 16 + oc]);
                out[(int64_t)(r0 + orow) * k + col] = sum;
            }
        }
    }
}

template <bool TP, bool PE>
void launch_project_narrow_tables(const float* x, const HighRank& h, const float* u, float* out, int rows, int d,
                                  int k, hipStream_t st) {
    const dim3 grid((unsigned)((rows + 15) / 16)), block(kThreads);
    if (k <= 16)
        hipLaunchKernelGGL((project_narrow_kernel<1, 2, TP, PE>), grid, block, 0, st, x, h, u, out, rows, d, k);
    else
        hipLaunchKernelGGL((project_narrow_kernel<2, 2, TP, PE>), grid, block, 0, st, x, h, u, out, rows, d, k);
}
void launch_project_narrow(const float* x, const HighRank& h, const float* u, float* out, int rows, int d, int k,
                           hipStream_t st) {
    if (h.t_perp && h.pos) launch_project_narrow_tables<true, true>(x, h, u, out, rows, d, k, st);
    else if (h.t_perp) launch_project_narrow_tables<true, false>(x, h, u, out, rows, d, k, st);
    else if (h.pos) launch_project_narrow_tables<false, true>(x, h, u, out, rows, d, k, st);
    else launch_project_narrow_tables<false, false>(x, h, u, out, rows, d, k, st);
}
// Where the narrow projection beats the GEMM kernel's 64 x 64 tile (measured at d 1536 / 2048, 16384 and 32000
// rows): whole 32-wide d tiles, and at most 32 columns with at most one table to gather, or at most 16 with
// both.  The more there is to gather per row, the less the narrow kernel's higher occupancy buys.
bool narrow_applies(int d, int k, const HighRank& h) {
    const int tables = (h.t_perp ? 1 : 0) + (h.pos ? 1 : 0);
    return d % 32 == 0 && k <= (tables == 2 ? 16 : 32);
}

template <int TM_, int TN_, bool B_NK, class Pro, class Epi>
void launch_gemm_tile(const float* A, int64_t lda, const float* B, int64_t ldb, int M, int N, int K, Pro pro, Epi epi,
                      int matmul, hipStream_t st) {
    const int64_t row_blocks = ((int64_t)(M + TM_ - 1) / TM_ + 7) / 8 * 8;
    dim3 grid((unsigned)(row_blocks * ((N + TN_ - 1) / TN_)));
    if (matmul == SPLC_MATMUL_BF16X3)
        hipLaunchKernelGGL((gemm_kernel<MATH_BF16X3, TM_, TN_, B_NK, Pro, Epi>), grid, dim3(kThreads), 0, st, A, lda, B,
                           ldb, M, N, K, pro, epi);
    else
        hipLaunchKernelGGL((gemm_kernel<MATH_F32, TM_, TN_, B_NK, Pro, Epi>), grid, dim3(kThreads), 0, st, A, lda, B,
                           ldb, M, N, K, pro, epi);
}
// Tile choice (measured on the shapes of sections 2.2 and 2.4 at d 1536 / 2048, k = d/8 ... d/16):
//   columns: 64 wide when N spans an odd number of 64-column blocks (the last 128-wide tile would be at
//            most half used), else 128 wide;
//   rows:    128 when that still leaves (nearly) two workgroups per compute unit -- 480 of them: the first pass of
//            the re-projection at 32000 x 2048, k = 256 has 500 and takes 272 us so, 288 us with 64 rows --, else 64;
//   a product with the basis as the N x K operand has K = k: up to K = 192 the K loop is so short that
//            64 x 64 tiles win (more, smaller workgroups per compute unit overlap one group's epilogue
//            with another's products); beyond that the reconstruction (light_epilogue: one store per
//            output) still prefers 64 rows;
//   with split-bf16 products (measured separately): see below.
struct GemmTile { bool tall, wide; };
GemmTile choose_gemm_tile(bool b_nk, int M, int N, int K, bool light_epilogue, int matmul) {
    auto groups = [&](int tm, int tn) { return (int64_t)((M + tm - 1) / tm) * ((N + tn - 1) / tn); };
    bool wide = ((N + 63) / 64) % 2 == 0;
    bool tall;
    if (matmul == SPLC_MATMUL_BF16X3) {
        // split operands: a tile's matrix work is a third as long and splitting costs per staged value, so the
        // large tile, which stages fewest values per product, wins wherever it leaves 1.5 groups per compute unit
        tall = b_nk || groups(128, wide ? 128 : 64) >= 3 * 128;
    } else if (b_nk && K <= 192) {
        wide = tall = false;
    } else if (light_epilogue) {
        tall = false;
    } else {
        tall = groups(128, wide ? 128 : 64) >= 480;
    }
    return GemmTile{tall, wide};
}
template <bool B_NK, class Pro, class Epi>
void launch_gemm(const float* A, int64_t lda, const float* B, int64_t ldb, int M, int N, int K, Pro pro, Epi epi,
                 int matmul, hipStream_t st, bool light_epilogue = false) {
    const GemmTile t = choose_gemm_tile(B_NK, M, N, K, light_epilogue, matmul);
    if (t.tall && t.wide) launch_gemm_tile<128, 128, B_NK>(A, lda, B, ldb, M, N, K, pro, epi, matmul, st);
    else if (t.tall) launch_gemm_tile<128, 64, B_NK>(A, lda, B, ldb, M, N, K, pro, epi, matmul, st);
    else if (t.wide) launch_gemm_tile<64, 128, B_NK>(A, lda, B, ldb, M, N, K, pro, epi, matmul, st);
    else launch_gemm_tile<64, 64, B_NK>(A, lda, B, ldb, M, N, K, pro, epi, matmul, st);
}

bool valid_matmul(int matmul) { return matmul == SPLC_MATMUL_FP32 || matmul == SPLC_MATMUL_BF16X3; }

bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

}  // namespace

namespace {

// Compute units of the current device (256 on an MI355X).
int compute_units() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        return 256;
    return n;
}

// Both passes of the re-projection with the coefficients in `coeff_ws` (vocab * k floats of device memory).
int reproject_impl(float* t_s, float* t_perp, const float* u, float* coeff_ws, int64_t vocab, int d, int k,
                   int matmul, hipStream_t st) {
    const int M = (int)vocab;
    // pass 1: coeff = T_S U            (M x k) = (M x d)(d x k)
    if (narrow_applies(d, k, HighRank{nullptr, nullptr, 0, nullptr, 1, (int64_t)d}))
        launch_project_narrow(t_s, HighRank{nullptr, nullptr, 0, nullptr, 1, (int64_t)d}, u, coeff_ws, M, d, k, st);
    else
        launch_gemm<false>(t_s, (int64_t)d, u, (int64_t)k, M, k, d, NoPrologue{}, StoreCoeff{coeff_ws, (int64_t)k}, matmul,
                           st);
    // pass 2: Pi = coeff U^T           (M x d) = (M x k)(k x d), U given as d x k = the N x K form
    launch_gemm<true>(coeff_ws, (int64_t)k, u, (int64_t)k, M, d, k, NoPrologue{},
                      UpdateEmbedding{t_s, t_perp, (int64_t)d, compute_units()},
                      matmul, st);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

int check_reproject_args(const float* t_s, const float* t_perp, const float* u, int64_t vocab, int d, int k,
                         int matmul) {
    if (!t_s || !t_perp || !u || !valid_matmul(matmul)) return SPLC_EINVAL;
    if (vocab < 0 || vocab > 0x7FFFFFFF - TM || d < 1 || k < 1 || k > d) return SPLC_EINVAL;
    if (!aligned4(t_s) || !aligned4(t_perp) || !aligned4(u)) return SPLC_EALIGN;
    return SPLC_OK;
}

// Coefficient workspace of sparseloco_reproject_embedding_noalloc: one array per GPU, part of the code object, so
// it exists from the moment the library is loaded on a device until the process ends.  Host code never uses the
// name below as an address; it asks the runtime for the array's device address once per device (scratch_of) and
// passes that pointer to the kernels.
static __device__ __align__(256) float scratch[SPLC_NOALLOC_MAX_COEFF];

constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};          // per device: address of that device's copy of `scratch`
std::mutex g_scratch_mutex;

int scratch_of(float** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SPLC_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return SPLC_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SPLC_EHIP;
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *out = g_scratch_ptr[dev];
    return SPLC_OK;
}

}  // namespace

extern "C" int sparseloco_reproject_embedding(float* t_s, float* t_perp, const float* u, float* coeff_ws,
                                              int64_t vocab, int d, int k, int matmul, void* stream) {
    if (!coeff_ws) return SPLC_EINVAL;
    int rc = check_reproject_args(t_s, t_perp, u, vocab, d, k, matmul);
    if (rc != SPLC_OK) return rc;
    if (!aligned4(coeff_ws)) return SPLC_EALIGN;
    if (vocab == 0) return SPLC_OK;
    return reproject_impl(t_s, t_perp, u, coeff_ws, vocab, d, k, matmul, static_cast<hipStream_t>(stream));
}

extern "C" int sparseloco_reproject_embedding_noalloc(float* t_s, float* t_perp, const float* u, int64_t vocab, int d,
                                                      int k, int matmul, void* stream) {
    int rc = check_reproject_args(t_s, t_perp, u, vocab, d, k, matmul);
    if (rc != SPLC_OK) return rc;
    if (vocab * (int64_t)k > (int64_t)SPLC_NOALLOC_MAX_COEFF) return SPLC_ETOOBIG;
    if (vocab == 0) return SPLC_OK;
    float* ws = nullptr;
    if ((rc = scratch_of(&ws)) != SPLC_OK) return rc;
    // Nothing has to start at zero: pass 1 writes every coefficient that pass 2 reads.
    return reproject_impl(t_s, t_perp, u, ws, vocab, d, k, matmul, static_cast<hipStream_t>(stream));
}

namespace {
int check_high_rank(const float* t_perp, const int32_t* token_ids, int vocab, const float* pos_embed, int seq_len) {
    if (t_perp && (!token_ids || vocab < 1)) return SPLC_EINVAL;
    if (pos_embed && seq_len < 1) return SPLC_EINVAL;
    if ((t_perp && !aligned4(t_perp)) || (token_ids && !aligned4(token_ids)) || (pos_embed && !aligned4(pos_embed)))
        return SPLC_EALIGN;
    return SPLC_OK;
}
}  // namespace

extern "C" int sparseloco_subspace_kernel_choice(int op, int64_t rows, int d, int k, int tables, int matmul) {
    if (rows < 1 || rows > 0x7FFFFFFF - TM || d < 1 || k < 1 || k > d || tables < 0 || tables > 2 || !valid_matmul(matmul))
        return SPLC_EINVAL;
    const int M = (int)rows;
    const float* const some = reinterpret_cast<const float*>(&op);      // only tested for being non-null
    GemmTile t;
    switch (op) {
        case SPLC_OP_PROJECT:
        case SPLC_OP_REPROJECT_PASS1: {
            const int n_tab = op == SPLC_OP_PROJECT ? tables : 0;
            const HighRank h{n_tab >= 1 ? some : nullptr, nullptr, 0, n_tab >= 2 ? some : nullptr, 1, (int64_t)d};
            if (narrow_applies(d, k, h)) return 16 * 256 + (k <= 16 ? 16 : 32);
            t = choose_gemm_tile(false, M, k, d, false, matmul);
            break;
        }
        case SPLC_OP_RECONSTRUCT: t = choose_gemm_tile(true, M, d, k, true, matmul); break;
        case SPLC_OP_REPROJECT_PASS2: t = choose_gemm_tile(true, M, d, k, false, matmul); break;
        default: return SPLC_EINVAL;
    }
    return (t.tall ? 128 : 64) * 256 + (t.wide ? 128 : 64);
}

extern "C" int sparseloco_subspace_project(const float* x, const float* t_perp, const int32_t* token_ids, int vocab,
                                           const float* pos_embed, int seq_len, const float* u, float* x_tilde,
                                           int64_t rows, int d, int k, int matmul, void* stream) {
    if (!x || !u || !x_tilde || !valid_matmul(matmul)) return SPLC_EINVAL;
    if (rows < 0 || rows > 0x7FFFFFFF - TM || d < 1 || k < 1 || k > d) return SPLC_EINVAL;
    int rc = check_high_rank(t_perp, token_ids, vocab, pos_embed, seq_len);
    if (rc != SPLC_OK) return rc;
    if (!aligned4(x) || !aligned4(u) || !aligned4(x_tilde)) return SPLC_EALIGN;
    if (rows == 0) return SPLC_OK;
    const int M = (int)rows;
    const HighRank h{t_perp, token_ids, vocab, pos_embed, seq_len > 0 ? seq_len : 1, (int64_t)d};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (narrow_applies(d, k, h)) {
        launch_project_narrow(x, h, u, x_tilde, M, d, k, st);
    } else if (t_perp && pos_embed)
        launch_gemm<false>(x, (int64_t)d, u, (int64_t)k, M, k, d, SubtractHighRank<true, true>{h, {nullptr, nullptr}},
                           StoreCoeff{x_tilde, (int64_t)k}, matmul, st);
    else if (t_perp)
        launch_gemm<false>(x, (int64_t)d, u, (int64_t)k, M, k, d, SubtractHighRank<true, false>{h, {nullptr, nullptr}},
                           StoreCoeff{x_tilde, (int64_t)k}, matmul, st);
    else if (pos_embed)
        launch_gemm<false>(x, (int64_t)d, u, (int64_t)k, M, k, d, SubtractHighRank<false, true>{h, {nullptr, nullptr}},
                           StoreCoeff{x_tilde, (int64_t)k}, matmul, st);
    else
        launch_gemm<false>(x, (int64_t)d, u, (int64_t)k, M, k, d, NoPrologue{}, StoreCoeff{x_tilde, (int64_t)k}, matmul, st);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

extern "C" int sparseloco_subspace_reconstruct(const float* x_tilde, const float* t_perp, const int32_t* token_ids,
                                               int vocab, const float* pos_embed, int seq_len, const float* u,
                                               float* x_hat, int64_t rows, int d, int k, int matmul, void* stream) {
    if (!x_tilde || !u || !x_hat || !valid_matmul(matmul)) return SPLC_EINVAL;
    if (rows < 0 || rows > 0x7FFFFFFF - TM || d < 1 || k < 1 || k > d) return SPLC_EINVAL;
    int rc = check_high_rank(t_perp, token_ids, vocab, pos_embed, seq_len);
    if (rc != SPLC_OK) return rc;
    if (!aligned4(x_tilde) || !aligned4(u) || !aligned4(x_hat)) return SPLC_EALIGN;
    if (rows == 0) return SPLC_OK;
    const int M = (int)rows;
    const HighRank h{t_perp, token_ids, vocab, pos_embed, seq_len > 0 ? seq_len : 1, (int64_t)d};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (t_perp && pos_embed)
        launch_gemm<true>(x_tilde, (int64_t)k, u, (int64_t)k, M, d, k, NoPrologue{}, AddHighRank<true, true>{h, x_hat},
                          matmul, st, true);
    else if (t_perp)
        launch_gemm<true>(x_tilde, (int64_t)k, u, (int64_t)k, M, d, k, NoPrologue{}, AddHighRank<true, false>{h, x_hat},
                          matmul, st, true);
    else if (pos_embed)
        launch_gemm<true>(x_tilde, (int64_t)k, u, (int64_t)k, M, d, k, NoPrologue{}, AddHighRank<false, true>{h, x_hat},
                          matmul, st, true);
    else
        launch_gemm<true>(x_tilde, (int64_t)k, u, (int64_t)k, M, d, k, NoPrologue{}, AddHighRank<false, false>{h, x_hat},
                          matmul, st, true);
    return hipGetLastError() == hipSuccess ? SPLC_OK : SPLC_EHIP;
}

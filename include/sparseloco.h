/*
 * libsparseloco -- the SparseLoCo outer step on one MI355X (gfx950).
 *
 * C ABI.  Three operations, one per group of lines of the update equations in
 * section 2.1 of the paper ("Background: SparseLoCo", equations labelled
 * sparse_update), run over every parameter tensor of a replica:
 *
 *   sparseloco_compress      delta = theta_outer - theta_local
 *                            e     = beta * e + delta
 *                            hat   = Q(Top-kappa per chunk of e)
 *                            e     = e - hat
 *   sparseloco_aggregate     delta_bar = (1/M) * sum_m hat_m
 *   sparseloco_outer_update  theta_outer = theta_outer - eta * delta_bar
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  Arguments of
 *     type `T* const*` are HOST arrays of device pointers (one per tensor, or
 *     one per replica); the library copies them during the call, so the host
 *     arrays may be reused as soon as the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; no call synchronises the device.  A call may
 *     block on the host only to recycle one of the plan's staging slots, i.e.
 *     to wait for work that this plan enqueued 32 calls earlier.
 *   - A plan may be used from one host thread at a time and belongs to the
 *     device that was current when it was created.
 *   - Calls that take a plan stage their pointer tables through pinned host
 *     memory (one small asynchronous copy per call) and may wait on an event;
 *     they are therefore not meant to be recorded into a HIP graph.  The
 *     matrix entry points (sparseloco_reproject_embedding, sparseloco_subspace_*)
 *     take no plan, only enqueue kernels, and can be captured.
 *   - Every function returns SPLC_OK or a negative status; nothing aborts or
 *     throws.  Arguments are validated on the host before anything is enqueued.
 *   - fp32 arithmetic is IEEE-754 round-to-nearest, one rounding per operation
 *     (no fused multiply-add), denormals kept.  Inputs must be finite.
 *   - A tensor is its row-major flattening; chunk = SPLC_CHUNK consecutive
 *     elements (sparseloco_plan_create) or a 64 x 64 tile
 *     (sparseloco_plan_create_2d); an edge chunk with n_c elements keeps
 *     min(kappa, n_c) entries.  Chunks are numbered tensor by tensor in the
 *     order given at plan creation.  Magnitude ties go to the lower index.
 *   - Tensor pointers need 4-byte alignment only.
 *
 * Message layout (per replica)
 *   pairs  uint16[n_chunks * kappa]   pairs[c*kappa + t] = index | code << 12,
 *                                     ascending index inside a chunk, index in
 *                                     bits 0-11, code in bits 12-13 (bit 13 =
 *                                     sign, bit 12 = upper level), bits 14-15
 *                                     zero; unused slots (t >= kappa_c) 0xFFFF.
 *   SPLC_QUANT_2BIT: scales float[n_chunks * 2], scales[2c] = lo, [2c+1] = hi;
 *                    a code decodes to (sign ? -1 : +1) * (upper ? hi : lo).
 *   SPLC_QUANT_NONE: values float[n_chunks * kappa], values[c*kappa + t] = the
 *                    selected fp32 value itself (code bits zero); unused slots +0.
 */
#ifndef SPARSELOCO_H
#define SPARSELOCO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPLC_CHUNK 4096          /* 64 x 64: chunk size of the paper's experiments (section 3, appendix table) */

enum {
    SPLC_OK = 0,
    SPLC_EINVAL = -1,            /* bad argument (NULL, size, range, mode) */
    SPLC_EALIGN = -2,            /* a tensor pointer is not 4-byte aligned */
    SPLC_ENOMEM = -3,            /* host or device allocation failed */
    SPLC_EHIP = -4,              /* a HIP runtime call failed */
    SPLC_EPLAN = -5,             /* call does not match the plan (quantiser mode, device) */
    SPLC_ETOOBIG = -6            /* problem larger than the fixed workspace of a call that allocates nothing */
};

enum { SPLC_F32 = 0, SPLC_BF16 = 1 };

enum {
    SPLC_DELTA_FROM_PARAMS = 0,  /* delta = theta_outer - theta_local, both given (fp32) */
    SPLC_DELTA_DIRECT = 1        /* delta given directly, fp32 or bf16 (widened exactly) */
};

enum {
    SPLC_QUANT_NONE = 0,         /* Q = identity: the setting of the paper's experiments */
    SPLC_QUANT_2BIT = 1          /* sign + one magnitude bit, two levels per chunk */
};

enum {
    SPLC_LAYOUT_FLAT = 0,        /* chunk = 4096 consecutive elements of the flattened tensor */
    SPLC_LAYOUT_TILE64 = 1       /* chunk = 64 x 64 tile of the tensor seen as a matrix */
};

enum {
    SPLC_SELECT_AUTO = 0,        /* candidate filter + exact ranking, radix select when it does not apply */
    SPLC_SELECT_RADIX = 1        /* always the radix select (same result; for tests and comparison) */
};

typedef struct sparseloco_plan sparseloco_plan;

/*
 * Build a plan for a list of tensors: the per-chunk table in device memory and
 * the staging slots for pointer tables.  numel[i] >= 0 (empty tensors have no
 * chunk).  kappa in 1..SPLC_CHUNK (Top-kappa per chunk, section 2.1; 32 in the
 * paper's runs).  quant_mode: SPLC_QUANT_*.  The plan owns only what it
 * allocates here; sparseloco_plan_destroy frees it after synchronising the
 * device work that still uses it.
 */
int sparseloco_plan_create(sparseloco_plan** out, int n_tensors, const int64_t* numel,
                           int kappa, int quant_mode);
/*
 * The same with the chunk read literally as a 64 x 64 tile (section 3: "a chunk
 * size of 64 x 64 (i.e., 4096 elements per chunk)").  Tensor i is a row-major
 * rows[i] x cols[i] matrix (fold leading dimensions into rows); tile (bi, bj)
 * covers rows 64*bi.. and columns 64*bj.., tiles are numbered row-major and edge
 * tiles are smaller (h x w elements, kappa_c = min(kappa, h*w)).  Inside a tile
 * the element at local row lr, local column lc has index lr*64 + lc, so pairs
 * keep their 12-bit index.  Tensors with rows[i] == 1 are chunked flat.
 * cols[i] < 2^24.
 */
int sparseloco_plan_create_2d(sparseloco_plan** out, int n_tensors, const int64_t* rows,
                              const int64_t* cols, int kappa, int quant_mode);
void sparseloco_plan_destroy(sparseloco_plan* plan);

int64_t sparseloco_plan_num_chunks(const sparseloco_plan* plan);   /* sum over tensors of ceil(numel / SPLC_CHUNK) */
int64_t sparseloco_plan_num_params(const sparseloco_plan* plan);   /* sum of numel */
int sparseloco_plan_kappa(const sparseloco_plan* plan);
int sparseloco_plan_quant_mode(const sparseloco_plan* plan);
int sparseloco_plan_layout(const sparseloco_plan* plan);            /* SPLC_LAYOUT_* */
/* SPLC_SELECT_*: which selection algorithm the compress kernel uses. */
int sparseloco_plan_set_select(sparseloco_plan* plan, int select_mode);

/*
 * Lines 1-4 of the update equations for ONE replica, all tensors, one launch.
 *   delta_mode = SPLC_DELTA_FROM_PARAMS: src_a = theta_outer[n_tensors],
 *       src_b = theta_local[n_tensors], src_dtype must be SPLC_F32.
 *   delta_mode = SPLC_DELTA_DIRECT: src_a = delta[n_tensors] of src_dtype,
 *       src_b = NULL.
 *   ef[n_tensors]: fp32 error-feedback buffers, read and rewritten in place.
 *   beta: error-feedback momentum (0.95 in the paper).
 *   pairs_out: uint16[n_chunks * kappa]; aux_out: float[n_chunks * 2] (2-bit
 *   mode: scales) or float[n_chunks * kappa] (identity mode: values).  Both are
 *   fully overwritten.  Sources are never written.  No buffer may overlap
 *   another.
 */
int sparseloco_compress(sparseloco_plan* plan, int delta_mode, int src_dtype,
                        const void* const* src_a, const void* const* src_b,
                        float* const* ef, float beta,
                        uint16_t* pairs_out, float* aux_out, void* stream);

/*
 * Lines 1-4 for several replicas that share theta_outer and live on this GPU
 * (the single-node simulation of M replicas): one launch, theta_outer read once
 * per chunk instead of once per replica.  Per replica the result is bit-identical
 * to sparseloco_compress in SPLC_DELTA_FROM_PARAMS mode.
 *   theta_outer[n_tensors]; theta_local[r][n_tensors], ef[r][n_tensors] (host
 *   arrays of host arrays of device pointers); pairs_out[r], aux_out[r]: replica
 *   r's message buffers, sized as for sparseloco_compress.  1 <= n_replicas <= 64.
 */
int sparseloco_compress_batch(sparseloco_plan* plan, int n_replicas,
                              const float* const* theta_outer,
                              const float* const* const* theta_local,
                              float* const* const* ef, float beta,
                              uint16_t* const* pairs_out, float* const* aux_out, void* stream);

/*
 * Line 5, first half: the mean over n_replicas (the paper's M) of the decoded
 * messages.  pairs[r], aux[r]: replica r's message as written by
 * sparseloco_compress with the same plan.  Per element the contributions are
 * added in ascending replica order starting from +0, then divided once by
 * (float)n_replicas; the result does not depend on scheduling (no float
 * atomics).  delta_bar_out[n_tensors]: dense fp32, fully overwritten (zero
 * where no replica sent anything).  1 <= n_replicas <= 1024.
 */
int sparseloco_aggregate(sparseloco_plan* plan, int n_replicas,
                         const uint16_t* const* pairs, const float* const* aux,
                         float* const* delta_bar_out, void* stream);

/*
 * Line 5, second half: theta_outer[i] -= outer_lr * delta_bar[i], in place
 * (outer SGD without momentum; outer_lr = 1.0 in the paper's runs).
 */
int sparseloco_outer_update(sparseloco_plan* plan, float* const* theta_outer,
                            const float* const* delta_bar, float outer_lr, void* stream);

/*
 * Line 5 in one pass: the mean as in sparseloco_aggregate and the update as in
 * sparseloco_outer_update, bit-identical to calling the two in sequence, without
 * the round trip of delta_bar through memory.  theta_outer[n_tensors] is updated
 * in place.  delta_bar_out may be NULL; if given, the dense mean is written too.
 * The next inner phase starts every replica from the synchronised parameters
 * (section 2.1, inner step): if n_reset > 0, the new theta_outer is also written
 * into theta_local_reset[r][n_tensors] for r < n_reset (0 <= n_reset <= 64;
 * host array of host arrays of device pointers; NULL if n_reset == 0).
 */
int sparseloco_aggregate_update(sparseloco_plan* plan, int n_replicas,
                                const uint16_t* const* pairs, const float* const* aux,
                                float* const* theta_outer, float outer_lr,
                                float* const* delta_bar_out,
                                int n_reset, float* const* const* theta_local_reset, void* stream);

/*
 * How the dense products of the three entry points below (sections 2.2 and 2.4;
 * the paper fixes no precision for them) are formed on the matrix cores.
 * Process-wide; takes effect for calls made after it returns.
 *   SPLC_MATMUL_FP32    (default) fp32 MFMA on the fp32 operands.
 *   SPLC_MATMUL_BF16X3  every fp32 operand is split exactly into three bf16
 *                       pieces and a product is the sum of the six piece
 *                       products of leading order on the bf16 MFMA (16 times
 *                       the fp32 rate), accumulated in fp32.  Each piece
 *                       product is exact in fp32; what is dropped is below
 *                       2^-23 |x y| per product, the size of an fp32 rounding
 *                       step.  Operands must be finite and normal-or-zero.
 * A projection onto at most 32 columns (16 with both tables of section 2.2) is
 * bound by memory traffic and always uses fp32 products.
 * Measured: 1.15-1.45 times the fp32 rate (the chip lowers its clock under the
 * bf16 matrix load, which caps the gain).
 * sparseloco_set_matmul_mode returns SPLC_EINVAL for another value.
 */
enum { SPLC_MATMUL_FP32 = 0, SPLC_MATMUL_BF16X3 = 1 };
int sparseloco_set_matmul_mode(int mode);
int sparseloco_get_matmul_mode(void);

/*
 * Section 2.4 ("Token Embeddings and Heterogeneous Setting"): after every outer
 * synchronisation the embedding component T_S is projected back onto the
 * compression subspace S = Col(U) and the part the projection removes is
 * accumulated into T_perp, so that T_S + T_perp is unchanged:
 *     T_perp <- T_perp + (T_S - Pi_S(T_S)),  T_S <- Pi_S(T_S),  Pi_S(X) = X U U^T.
 * With T_perp = 0 on entry this is also the initialisation before training.
 *   t_s, t_perp: [vocab, d] row-major fp32 device arrays, updated in place.
 *   u: [d, k] row-major fp32, orthonormal columns (not checked), 1 <= k <= d.
 *   coeff_ws: device workspace of vocab * k floats owned by the caller; on return
 *   (after the stream reaches this point) it holds T_S U.
 * fp32 inputs, matrix-core products as set by sparseloco_set_matmul_mode (fp32
 * by default), fp32 accumulation; the result
 * differs from exact arithmetic by the usual dot-product rounding of length d
 * and k.  Pointers 4-byte aligned; vocab < 2^31 - 128.
 */
int sparseloco_reproject_embedding(float* t_s, float* t_perp, const float* u, float* coeff_ws,
                                   int64_t vocab, int d, int k, void* stream);

/*
 * sparseloco_reproject_embedding for callers that cannot allocate device memory or hold a workspace of their
 * own: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same kernels, same
 * results, bit for bit; the coefficients T_S U go to a fixed array of SPLC_NOALLOC_MAX_COEFF floats (32 MiB)
 * that is part of the library's code object: every GPU the library runs on holds one copy from load time until
 * the process ends.  The call makes no hipMalloc / hipFree and no other allocating call; its first call on a
 * device looks the array's address up once (do that first call outside a graph capture).
 *   vocab * k <= SPLC_NOALLOC_MAX_COEFF, else SPLC_ETOOBIG (nothing is enqueued).
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams
 * without an ordering between them) race on it.  Nothing in it has to be cleared between calls -- pass 1 writes
 * every coefficient pass 2 reads -- and its contents after the call are unspecified.
 */
#define SPLC_NOALLOC_MAX_COEFF (8 * 1024 * 1024)
int sparseloco_reproject_embedding_noalloc(float* t_s, float* t_perp, const float* u,
                                           int64_t vocab, int d, int k, void* stream);

/*
 * Section 2.2 ("Communication-Efficient Pipeline Parallelism"): what a pipeline
 * stage sends instead of its activations, and how the next stage rebuilds them.
 *     project      x_tilde = (x - T_perp[token] - PosEmbed[position]) U      [rows, k]
 *     reconstruct  x_hat   = x_tilde U^T + T_perp[token] + PosEmbed[position]   [rows, d]
 * rows = batch * seq_len tokens of a [batch, seq_len, d] row-major tensor; the
 * position of row r is r % seq_len.  t_perp [vocab, d] with token_ids [rows]
 * (int32, clamped into [0, vocab)) and pos_embed [seq_len, d] are each optional
 * (NULL): with both NULL, project is the plain product used for the backward
 * pass, (grad x) U.  u: [d, k] row-major, 1 <= k <= d.  All arrays fp32 device
 * memory, 4-byte aligned; matrix-core products as set by sparseloco_set_matmul_mode
 * (fp32 by default), fp32 accumulation.
 * The outputs are fully overwritten and must not overlap the inputs.
 */
int sparseloco_subspace_project(const float* x, const float* t_perp, const int32_t* token_ids, int vocab,
                                const float* pos_embed, int seq_len, const float* u, float* x_tilde,
                                int64_t rows, int d, int k, void* stream);
int sparseloco_subspace_reconstruct(const float* x_tilde, const float* t_perp, const int32_t* token_ids,
                                    int vocab, const float* pos_embed, int seq_len, const float* u,
                                    float* x_hat, int64_t rows, int d, int k, void* stream);

const char* sparseloco_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif

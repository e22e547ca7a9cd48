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
 *   - Every data pointer is a DEVICE pointer owned by the caller.  A list of
 *     tensors (one device pointer per tensor of the plan) or of messages (one
 *     pair of device pointers per replica) is BOUND once: sparseloco_tensors_bind
 *     / sparseloco_messages_bind copy a host array of device pointers into a
 *     small device-resident table and return a handle.  The operations take
 *     handles.  The host arrays may be reused as soon as the bind call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     The operations (compress, compress_batch, outer_step_batch, aggregate,
 *     aggregate_update, outer_update and the matrix entry points) ONLY ENQUEUE
 *     KERNELS on it: no allocation, no copy, no event, no host wait.  They can
 *     be recorded into a HIP graph.  plan_create and the bind calls allocate and enqueue one small
 *     host-to-device copy on their stream; work on ANOTHER stream that uses the
 *     plan or the handle must be ordered after that copy by the caller.
 *   - The plan and the handles are immutable once created (the exceptions,
 *     sparseloco_plan_set_select and sparseloco_plan_set_radix_counter, are test
 *     and diagnostic switches) and belong to the device that was current when
 *     they were created; every operation takes them as
 *     pointers to const and may be called from several host threads at once.
 *     Release a handle or destroy a plan only after the work that uses it has
 *     completed (the release calls free device memory, which waits for the
 *     device).
 *   - Every function returns SPLC_OK or a negative status; nothing aborts or
 *     throws.  Arguments are validated on the host before anything is enqueued
 *     (pointers: at bind time).
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
#define SPLC_MAX_REPLICAS 1024   /* most messages one binding holds, most sets one tensor binding holds */

enum {
    SPLC_OK = 0,
    SPLC_EINVAL = -1,            /* bad argument (NULL, size, range, mode) */
    SPLC_EALIGN = -2,            /* a tensor pointer is not 4-byte aligned */
    SPLC_ENOMEM = -3,            /* host or device allocation failed */
    SPLC_EHIP = -4,              /* a HIP runtime call failed */
    SPLC_EPLAN = -5,             /* call does not match the plan or a handle (tensor count, dtype, quantiser, device) */
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
typedef struct sparseloco_tensors sparseloco_tensors;      /* bound list(s) of the plan's tensors */
typedef struct sparseloco_messages sparseloco_messages;    /* bound message buffers of some replicas */

/*
 * Build a plan for a list of tensors: the per-chunk table in device memory
 * (uploaded by one asynchronous copy on `stream`).  numel[i] >= 0 (empty tensors
 * have no chunk).  chunk must be SPLC_CHUNK.  kappa in 1..SPLC_CHUNK (Top-kappa
 * per chunk, section 2.1; 32 in the paper's runs).  quant_mode: SPLC_QUANT_*.
 * The plan owns only what it allocates here.
 */
int sparseloco_plan_create(sparseloco_plan** out, int n_tensors, const int64_t* numel,
                           int chunk, int kappa, int quant_mode, void* stream);
/*
 * The same with the chunk read literally as a 64 x 64 tile (chunk size as given
 * in section 3 and the appendix hyper-parameter table).  Tensor i is a row-major
 * rows[i] x cols[i] matrix (fold leading dimensions into rows); tile (bi, bj)
 * covers rows 64*bi.. and columns 64*bj.., tiles are numbered row-major and edge
 * tiles are smaller (h x w elements, kappa_c = min(kappa, h*w)).  Inside a tile
 * the element at local row lr, local column lc has index lr*64 + lc, so pairs
 * keep their 12-bit index.  Tensors with rows[i] == 1 are chunked flat.
 * cols[i] < 2^24.  chunk must be SPLC_CHUNK.
 */
int sparseloco_plan_create_2d(sparseloco_plan** out, int n_tensors, const int64_t* rows,
                              const int64_t* cols, int chunk, int kappa, int quant_mode, void* stream);
void sparseloco_plan_destroy(sparseloco_plan* plan);

/* Chunks of the plan: per tensor ceil(numel / SPLC_CHUNK) (flat layout, and 1-D tensors of a tiled plan) or
 * ceil(rows / 64) * ceil(cols / 64) (tiles), summed over the tensors. */
int64_t sparseloco_plan_num_chunks(const sparseloco_plan* plan);
int64_t sparseloco_plan_num_params(const sparseloco_plan* plan);   /* sum of numel */
int sparseloco_plan_num_tensors(const sparseloco_plan* plan);
int sparseloco_plan_kappa(const sparseloco_plan* plan);
int sparseloco_plan_quant_mode(const sparseloco_plan* plan);
int sparseloco_plan_layout(const sparseloco_plan* plan);            /* SPLC_LAYOUT_* */
/* SPLC_SELECT_*: which selection algorithm the compress kernel uses.  A test switch: not to be called while
 * another thread uses the plan. */
int sparseloco_plan_set_select(sparseloco_plan* plan, int select_mode);
/* Diagnostic: while device_counter (one uint32 in device memory, owned by the caller) is set, every compress
 * launch adds to it the number of (chunk, replica) selections that took the general radix path instead of the
 * candidate filter.  NULL switches it off (the default).  Same caveat as sparseloco_plan_set_select. */
int sparseloco_plan_set_radix_counter(sparseloco_plan* plan, uint32_t* device_counter);

/*
 * The chunk table a plan with these tensors holds, computed on the host (no GPU needed): for checking tools.
 * layout: SPLC_LAYOUT_*; rows may be NULL for the flat layout (then cols[i] = numel).  Writes up to `capacity`
 * entries of 32 bytes each to `out` (may be NULL):
 *   uint32 tensor; uint32 n_c; uint64 offset; uint32 stride; uint8 h, w, last_w, vec; uint32 id; uint32 strip
 * -- local index idx of chunk `id` (present iff idx/64 < h-1 and idx%64 < w, or idx/64 == h-1 and idx%64 < last_w)
 * is element offset + (idx / 64) * stride + idx % 64 of tensor `tensor`.  vec: bit 0 = the chunk is complete and
 * is read with 4-element vector accesses as fp32, bit 1 = also as bf16.  strip: 0, or 1 + j for the j-th of four
 * complete tiles side by side that a tiled plan hands to one workgroup (which then reads whole 256-element rows
 * from the first tile's origin).  Order: first the chunks that workgroups take one by one, in launch order, then
 * the strips' members.  Returns the number of chunks, or a negative status.
 */
int64_t sparseloco_chunk_table(int n_tensors, const int64_t* rows, const int64_t* cols, int layout,
                               void* out, int64_t capacity);

/*
 * Bind n_sets lists of tensors of the plan.  ptrs: host array of n_sets * n_tensors device pointers, set-major
 * (ptrs[s * n_tensors + t] = tensor t of set s); a tensor with numel 0 may be NULL.  dtype: SPLC_F32 or
 * SPLC_BF16 (what the pointers point at).  1 <= n_sets <= SPLC_MAX_REPLICAS.  Sets are what the replicas of a
 * single-node simulation index: theta_local and the error-feedback buffers of replica r are set r of their
 * bindings; parameters shared by all replicas are bound as one set.
 * Checks on the host: pointers present and 4-byte aligned.  What they point at is not touched.
 */
int sparseloco_tensors_bind(sparseloco_tensors** out, const sparseloco_plan* plan, int n_sets,
                            const void* const* ptrs, int dtype, void* stream);
void sparseloco_tensors_release(sparseloco_tensors* tensors);

/*
 * Bind the message buffers of n_replicas replicas (1..SPLC_MAX_REPLICAS): pairs[r] uint16[n_chunks * kappa],
 * aux[r] float[n_chunks * 2] (2-bit mode: scales) or float[n_chunks * kappa] (identity mode: values).
 */
int sparseloco_messages_bind(sparseloco_messages** out, const sparseloco_plan* plan, int n_replicas,
                             uint16_t* const* pairs, float* const* aux, void* stream);
void sparseloco_messages_release(sparseloco_messages* messages);

/*
 * Lines 1-4 of the update equations for ONE replica, all tensors, one launch.
 *   delta_mode = SPLC_DELTA_FROM_PARAMS: src_a = theta_outer, src_b = theta_local, both fp32.
 *   delta_mode = SPLC_DELTA_DIRECT: src_a = delta (fp32 or bf16 binding), src_b = NULL.
 *   ef: fp32 error-feedback buffers, read and rewritten in place.
 *   replica: which set of each binding to use; a binding with a single set serves every replica.
 *   beta: error-feedback momentum (0.95 in the paper).
 *   pairs_out: uint16[n_chunks * kappa]; aux_out: float[n_chunks * 2] (2-bit mode: scales) or
 *   float[n_chunks * kappa] (identity mode: values).  Both are fully overwritten.  Sources are never
 *   written.  No buffer may overlap another.
 */
int sparseloco_compress(const sparseloco_plan* plan, int delta_mode,
                        const sparseloco_tensors* src_a, const sparseloco_tensors* src_b,
                        const sparseloco_tensors* ef, int replica, float beta,
                        uint16_t* pairs_out, float* aux_out, void* stream);

/*
 * Lines 1-4 for several replicas that share theta_outer and live on this GPU
 * (the single-node simulation of M replicas): one launch, theta_outer read once
 * per chunk instead of once per replica.  Per replica the result is bit-identical
 * to sparseloco_compress in SPLC_DELTA_FROM_PARAMS mode.
 *   theta_outer: one set; theta_local, ef: at least n_replicas sets (replica r = set r); messages_out: at
 *   least n_replicas messages (replica r writes message r).  1 <= n_replicas <= SPLC_MAX_REPLICAS.
 */
int sparseloco_compress_batch(const sparseloco_plan* plan, int n_replicas,
                              const sparseloco_tensors* theta_outer, const sparseloco_tensors* theta_local,
                              const sparseloco_tensors* ef, float beta,
                              const sparseloco_messages* messages_out, void* stream);

/*
 * Line 5, first half: the mean over the bound messages (their number is the
 * paper's M), as written by sparseloco_compress with the same plan.  Per element
 * the contributions are added in ascending replica order starting from +0, then
 * divided once by (float)M; the result does not depend on scheduling (no float
 * atomics).  delta_bar_out (one set): dense fp32, fully overwritten (zero where
 * no replica sent anything).
 */
int sparseloco_aggregate(const sparseloco_plan* plan, const sparseloco_messages* messages,
                         const sparseloco_tensors* delta_bar_out, void* stream);

/*
 * Line 5, second half: theta_outer[i] -= outer_lr * delta_bar[i], in place
 * (outer SGD without momentum; outer_lr = 1.0 in the paper's runs).
 */
int sparseloco_outer_update(const sparseloco_plan* plan, const sparseloco_tensors* theta_outer,
                            const sparseloco_tensors* delta_bar, float outer_lr, void* stream);

/*
 * Line 5 in one pass: the mean as in sparseloco_aggregate and the update as in
 * sparseloco_outer_update, bit-identical to calling the two in sequence, without
 * the round trip of delta_bar through memory.  theta_outer (one set) is updated
 * in place.  delta_bar_out may be NULL; if given, the dense mean is written too.
 * The next inner phase starts every replica from the synchronised parameters
 * (section 2.1, inner step): if theta_local_reset is given, the new theta_outer
 * is also written into every set of that binding.
 */
int sparseloco_aggregate_update(const sparseloco_plan* plan, const sparseloco_messages* messages,
                                const sparseloco_tensors* theta_outer, float outer_lr,
                                const sparseloco_tensors* delta_bar_out,
                                const sparseloco_tensors* theta_local_reset, void* stream);

/*
 * The whole outer step of a single-node simulation in one launch: lines 1-4 for the first
 * n_replicas sets of theta_local / ef as in sparseloco_compress_batch, then line 5 as in
 * sparseloco_aggregate_update over exactly those replicas' messages.  Results are bit-identical to
 * the two calls in sequence (the messages are still written: they are outputs).  Every chunk is
 * handled by one workgroup from its first read to the update of theta_outer, so the sent values
 * are averaged where they are produced and theta_outer is read once and written once.
 *   theta_outer: one set, updated in place.  delta_bar_out: may be NULL; if given (one set), the
 *   dense mean is written.  reset_theta_local != 0: the new theta_outer is also written into
 *   theta_local sets 0 .. n_replicas-1 (section 2.1, inner step: replicas restart from the
 *   synchronised parameters).  1 <= n_replicas <= SPLC_MAX_REPLICAS.
 */
int sparseloco_outer_step_batch(const sparseloco_plan* plan, int n_replicas,
                                const sparseloco_tensors* theta_outer, const sparseloco_tensors* theta_local,
                                const sparseloco_tensors* ef, float beta, float outer_lr,
                                const sparseloco_messages* messages_out,
                                const sparseloco_tensors* delta_bar_out, int reset_theta_local, void* stream);

/*
 * How the dense products of the matrix entry points below (sections 2.2 and 2.4;
 * the paper fixes no precision for them) are formed on the matrix cores: the
 * `matmul` argument of those calls.
 *   SPLC_MATMUL_FP32    fp32 MFMA on the fp32 operands.
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
 * bf16 matrix load, which caps the gain).  Another value: SPLC_EINVAL.
 */
enum { SPLC_MATMUL_FP32 = 0, SPLC_MATMUL_BF16X3 = 1 };

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
 * fp32 inputs, matrix-core products as `matmul` says (SPLC_MATMUL_*), fp32
 * accumulation; the result
 * differs from exact arithmetic by the usual dot-product rounding of length d
 * and k.  Pointers 4-byte aligned; vocab < 2^31 - 128.
 */
int sparseloco_reproject_embedding(float* t_s, float* t_perp, const float* u, float* coeff_ws,
                                   int64_t vocab, int d, int k, int matmul, void* stream);

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
                                           int64_t vocab, int d, int k, int matmul, void* stream);

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
 * memory, 4-byte aligned; matrix-core products as `matmul` says (SPLC_MATMUL_*),
 * fp32 accumulation.
 * The outputs are fully overwritten and must not overlap the inputs.
 */
int sparseloco_subspace_project(const float* x, const float* t_perp, const int32_t* token_ids, int vocab,
                                const float* pos_embed, int seq_len, const float* u, float* x_tilde,
                                int64_t rows, int d, int k, int matmul, void* stream);
int sparseloco_subspace_reconstruct(const float* x_tilde, const float* t_perp, const int32_t* token_ids,
                                    int vocab, const float* pos_embed, int seq_len, const float* u,
                                    float* x_hat, int64_t rows, int d, int k, int matmul, void* stream);

/*
 * Which kernel variant a matrix call takes for a shape: host logic only (nothing is launched), for tests and
 * tuning.  op: SPLC_OP_*; rows = rows of x (project / reconstruct) or the vocabulary (re-projection);
 * tables: how many of the two tables of section 2.2 are present (0..2; ignored for the re-projection).
 * Returns tile_rows * 256 + tile_cols of a workgroup's output tile -- 128 or 64 by 128 or 64 for the GEMM
 * kernel, 16 by 16 or 16 by 32 for the narrow projection kernel -- or a negative status.
 */
enum { SPLC_OP_PROJECT = 0, SPLC_OP_RECONSTRUCT = 1, SPLC_OP_REPROJECT_PASS1 = 2, SPLC_OP_REPROJECT_PASS2 = 3 };
int sparseloco_subspace_kernel_choice(int op, int64_t rows, int d, int k, int tables, int matmul);

/*
 * Measurement aid: what the chip streams for the access patterns of the kernels above, with their launch shape
 * (one 256-lane workgroup per 4096 floats, 16-byte non-temporal accesses).  The practical ceiling next to which
 * the achieved bandwidths are read; not part of the method.
 *   SPLC_STREAM_READ     a is read                                     4 bytes per element
 *   SPLC_STREAM_WRITE    c is written                                  4
 *   SPLC_STREAM_COPY     c = a                                         8
 *   SPLC_STREAM_R2W1     c = c - a        (pattern of outer_update)    12
 *   SPLC_STREAM_R3W1     c = (a - b) + c  (pattern of compress)        16
 * a, b, c: n floats each of device memory (n a multiple of 4096; unused ones may be NULL); sink: one float of
 * device memory that keeps the read-only pattern from being optimised away.
 */
enum { SPLC_STREAM_READ = 0, SPLC_STREAM_WRITE = 1, SPLC_STREAM_COPY = 2, SPLC_STREAM_R2W1 = 3, SPLC_STREAM_R3W1 = 4 };
int sparseloco_stream_probe(int pattern, const float* a, const float* b, float* c, float* sink, int64_t n,
                            void* stream);
/*
 * The same patterns with the launch shape varied:
 *   slots                4 (the kernels' shape: a workgroup covers 16 KB of each array) or 1 (4 KB);
 *   run                  0 = workgroup i takes chunk i (eight neighbouring chunks run on the eight XCDs); > 0 =
 *                        every XCD walks runs of `run` consecutive chunks (the number of workgroups must then
 *                        be a multiple of 8 * run);
 *   max_groups_per_unit  0 = as many workgroups per compute unit as fit, else at most this many (1..8).
 * sparseloco_stream_probe is (slots 4, run 0, max_groups_per_unit 0).
 */
int sparseloco_stream_probe_shaped(int pattern, const float* a, const float* b, float* c, float* sink, int64_t n,
                                   int slots, int run, int max_groups_per_unit, void* stream);

const char* sparseloco_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif

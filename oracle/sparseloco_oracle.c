/*
 * CPU oracle for the SparseLoCo outer step (paper section 2.1, the update
 * equations labelled "sparse_update").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what the
 * outer step computes, written to be checked against the paper by eye.  Only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the GPU library shares no code, header, table or helper with this file.
 *
 * Every floating-point operation is IEEE-754 binary32, round to nearest even,
 * one rounding per written operation (compile with -ffp-contract=off, never
 * with fast-math), denormals kept.
 *
 * Readings where the paper is silent (all of them are restated in the design
 * notes of the repository):
 *   - chunk geometry.  The paper gives the chunk size as 64 x 64, that is 4096 elements
 *     (section 3, training configuration; appendix hyper-parameter table).
 *     Two readings are implemented:
 *       flat   a chunk is `chunk` consecutive elements of the row-major
 *              flattened tensor; the last chunk of a tensor may be shorter;
 *       tiled  the tensor is a rows x cols matrix cut into tile x tile blocks
 *              (tile = 64 in the paper); block (bi, bj) is one chunk, blocks
 *              are numbered row-major, edge blocks are smaller; inside a
 *              block the element at local row lr, local column lc has index
 *              lr * tile + lc.  A matrix with rows == 1 is chunked flat with
 *              chunk = tile * tile.
 *     A chunk with n_c elements keeps kappa_c = min(kappa, n_c) entries;
 *   - magnitude ties go to the lower index;
 *   - Q() is a 2-bit code: sign bit plus one magnitude bit choosing between
 *     two per-chunk levels lo/hi at the 1/4 and 3/4 points of the range
 *     [amin, amax] of the selected magnitudes.  The paper names Q() without
 *     defining it (its experiments ran without quantisation), so this part is
 *     "parity unpinned" with respect to the paper; it is pinned only to the
 *     closed forms that follow from the rule itself;
 *   - quant_mode 0 (Q = identity, the setting of the paper's experiments)
 *     sends the selected fp32 values unchanged;
 *   - a pair is uint16 = index | code << 12; unused slots hold 0xFFFF.
 *
 * Pins: tests/test_oracle_*.py (brute-force full sort, closed forms,
 * hand-computed exact cases, conservation, dense mean, tile geometry against
 * numpy slicing).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL -1
#define MAX_CHUNK 4096

static uint32_t bits_of(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float float_of(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ------------------------------------------------------------ chunk geometry */

typedef struct {
    int64_t rows, cols;      /* the tensor as a row-major matrix (flat: rows = 1, cols = numel) */
    int tiled;               /* 0: flat chunks of `chunk` elements; 1: tile x tile blocks */
    int chunk;               /* flat: elements per chunk; tiled: tile * tile */
    int tile;                /* tiled only: block side */
} geometry;

static int geometry_init(geometry* g, int64_t rows, int64_t cols, int chunk_or_tile, int tiled) {
    if (rows < 0 || cols < 0 || chunk_or_tile < 1) return ORACLE_EINVAL;
    if (tiled && rows > 1) {
        if ((int64_t)chunk_or_tile * chunk_or_tile > MAX_CHUNK) return ORACLE_EINVAL;
        g->rows = rows; g->cols = cols; g->tiled = 1; g->tile = chunk_or_tile;
        g->chunk = chunk_or_tile * chunk_or_tile;
    } else {
        int chunk = tiled ? chunk_or_tile * chunk_or_tile : chunk_or_tile;
        if (chunk > MAX_CHUNK) return ORACLE_EINVAL;
        g->rows = 1; g->cols = rows * cols; g->tiled = 0; g->tile = 0; g->chunk = chunk;
    }
    return ORACLE_OK;
}

static int64_t geometry_chunks(const geometry* g) {
    if (g->rows * g->cols == 0) return 0;
    if (!g->tiled) return (g->cols + g->chunk - 1) / g->chunk;
    return ((g->rows + g->tile - 1) / g->tile) * ((g->cols + g->tile - 1) / g->tile);
}

/* Position in the flattened tensor of local index idx of chunk c, or -1 if that index is outside the tensor. */
static int64_t geometry_pos(const geometry* g, int64_t c, uint32_t idx) {
    if (!g->tiled) {
        int64_t p = c * (int64_t)g->chunk + idx;
        return (idx < (uint32_t)g->chunk && p < g->cols) ? p : -1;
    }
    int64_t blocks_per_row = (g->cols + g->tile - 1) / g->tile;
    int64_t bi = c / blocks_per_row, bj = c % blocks_per_row;
    int64_t r = bi * g->tile + idx / (uint32_t)g->tile, col = bj * g->tile + idx % (uint32_t)g->tile;
    if (idx >= (uint32_t)g->chunk || r >= g->rows || col >= g->cols) return -1;
    return r * g->cols + col;
}

/* The chunk's elements in ascending local index: pos[i] in the tensor, lidx[i] inside the chunk. */
static int geometry_members(const geometry* g, int64_t c, int64_t* pos, uint32_t* lidx) {
    int n = 0;
    uint32_t idx;
    for (idx = 0; idx < (uint32_t)g->chunk; ++idx) {
        int64_t p = geometry_pos(g, c, idx);
        if (p >= 0) { pos[n] = p; lidx[n] = idx; ++n; }
    }
    return n;
}

/* ------------------------------------------------------------------ compress */

typedef struct { uint32_t key; uint32_t idx; } keyed;

/* total order: larger magnitude first, then lower index first */
static int by_key_desc_idx_asc(const void* pa, const void* pb) {
    const keyed* a = (const keyed*)pa;
    const keyed* b = (const keyed*)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
    return 0;
}

static int by_u32_asc(const void* pa, const void* pb) {
    uint32_t a = *(const uint32_t*)pa, b = *(const uint32_t*)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

/*
 * One replica, one tensor: section 2.1, lines 1-4 of the update equations.
 *
 *   delta_i = theta_outer_i - theta_local_i          (or given directly)
 *   e'_i    = beta * e_i + delta_i
 *   S_c     = Top-kappa of |e'| inside each chunk
 *   hat_i   = Q(e'_i) for i in S_c, 0 elsewhere
 *   e_i     = e'_i - hat_i
 *
 * Geometry: rows x cols row-major; tiled = 0 -> flat chunks of chunk_or_tile
 * elements; tiled = 1 -> chunk_or_tile x chunk_or_tile blocks.
 * Exactly one source of delta must be given:
 *   theta_outer and theta_local (fp32), or delta_f32, or delta_bf16 (raw
 *   bfloat16 bit patterns, widened exactly).
 * quant_mode 1: pairs_out[c*kappa + t] = idx | code << 12, scales_out[2c] = lo,
 *               scales_out[2c+1] = hi, values_out unused (may be NULL).
 * quant_mode 0: pairs_out[c*kappa + t] = idx (code bits zero),
 *               values_out[c*kappa + t] = e'_idx, scales_out unused.
 * Unused slots t >= kappa_c: pairs 0xFFFF, values +0.
 */
int oracle_compress(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, float beta,
                    int quant_mode,
                    const float* theta_outer, const float* theta_local,
                    const float* delta_f32, const uint16_t* delta_bf16,
                    float* ef, uint16_t* pairs_out, float* scales_out, float* values_out)
{
    geometry g;
    if (geometry_init(&g, rows, cols, chunk_or_tile, tiled) != ORACLE_OK) return ORACLE_EINVAL;
    if (kappa < 1 || !ef || !pairs_out) return ORACLE_EINVAL;
    int have_params = theta_outer && theta_local;
    int n_src = (have_params ? 1 : 0) + (delta_f32 ? 1 : 0) + (delta_bf16 ? 1 : 0);
    if (n_src != 1) return ORACLE_EINVAL;
    if (quant_mode == 1 && !scales_out) return ORACLE_EINVAL;
    if (quant_mode == 0 && !values_out) return ORACLE_EINVAL;
    if (quant_mode != 0 && quant_mode != 1) return ORACLE_EINVAL;

    int64_t n_chunks = geometry_chunks(&g);
    int64_t c;
#pragma omp parallel for schedule(static)
    for (c = 0; c < n_chunks; ++c) {
        int64_t* pos = (int64_t*)malloc(sizeof(int64_t) * MAX_CHUNK);
        uint32_t* lidx = (uint32_t*)malloc(sizeof(uint32_t) * MAX_CHUNK);
        int n_c = geometry_members(&g, c, pos, lidx);
        int kappa_c = kappa < n_c ? kappa : n_c;
        float* eprime = (float*)malloc(sizeof(float) * MAX_CHUNK);          /* indexed by member number */
        keyed* order = (keyed*)malloc(sizeof(keyed) * MAX_CHUNK);
        uint32_t* sel = (uint32_t*)malloc(sizeof(uint32_t) * MAX_CHUNK);    /* member numbers kept */
        int i, t;

        /* pseudo-gradient and error-feedback fold */
        for (i = 0; i < n_c; ++i) {
            float delta;
            if (have_params) delta = theta_outer[pos[i]] - theta_local[pos[i]];
            else if (delta_f32) delta = delta_f32[pos[i]];
            else delta = float_of((uint32_t)delta_bf16[pos[i]] << 16);
            float scaled = beta * ef[pos[i]];
            eprime[i] = scaled + delta;
        }

        /* Top-kappa by magnitude: full sort of the chunk.  Members are in ascending local index,
           so the member number orders ties exactly as the local index does. */
        for (i = 0; i < n_c; ++i) {
            order[i].key = bits_of(eprime[i]) & 0x7FFFFFFFu;
            order[i].idx = (uint32_t)i;
        }
        qsort(order, (size_t)n_c, sizeof(keyed), by_key_desc_idx_asc);
        for (t = 0; t < kappa_c; ++t) sel[t] = order[t].idx;
        qsort(sel, (size_t)kappa_c, sizeof(uint32_t), by_u32_asc);

        if (quant_mode == 1) {
            /* two-level magnitude codebook over the selected entries */
            float amin = 0.f, amax = 0.f;
            for (t = 0; t < kappa_c; ++t) {
                float a = float_of(bits_of(eprime[sel[t]]) & 0x7FFFFFFFu);
                if (t == 0 || a < amin) amin = a;
                if (t == 0 || a > amax) amax = a;
            }
            float d = amax - amin;
            float q1 = 0.25f * d, q2 = 0.5f * d, q3 = 0.75f * d;
            float lo = amin + q1, tau = amin + q2, hi = amin + q3;
            scales_out[2 * c] = lo;
            scales_out[2 * c + 1] = hi;
            for (t = 0; t < kappa_c; ++t) {
                uint32_t mem = sel[t];
                uint32_t b = bits_of(eprime[mem]);
                float a = float_of(b & 0x7FFFFFFFu);
                uint32_t s = b >> 31;
                uint32_t m = (a >= tau) ? 1u : 0u;
                uint32_t code = (s << 1) | m;
                float level = m ? hi : lo;
                float q = s ? -level : level;
                pairs_out[c * (int64_t)kappa + t] = (uint16_t)(lidx[mem] | (code << 12));
                eprime[mem] = eprime[mem] - q;     /* what was sent leaves the buffer */
            }
        } else {
            for (t = 0; t < kappa_c; ++t) {
                uint32_t mem = sel[t];
                float v = eprime[mem];
                pairs_out[c * (int64_t)kappa + t] = (uint16_t)lidx[mem];
                values_out[c * (int64_t)kappa + t] = v;
                eprime[mem] = eprime[mem] - v;
            }
        }
        for (t = kappa_c; t < kappa; ++t) {
            pairs_out[c * (int64_t)kappa + t] = 0xFFFFu;
            if (quant_mode == 0) values_out[c * (int64_t)kappa + t] = 0.f;
        }
        for (i = 0; i < n_c; ++i) ef[pos[i]] = eprime[i];
        free(pos); free(lidx); free(eprime); free(order); free(sel);
    }
    return ORACLE_OK;
}

/* Value a pair stands for. */
static float decode_pair(uint16_t p, int quant_mode, const float* scales_c, float value) {
    uint32_t code = (p >> 12) & 3u;
    if (quant_mode == 1) {
        float level = (code & 1u) ? scales_c[1] : scales_c[0];
        return (code & 2u) ? -level : level;
    }
    return value;
}

static int pairs_in_chunk(const geometry* g, int64_t c, int kappa) {
    int n = 0;
    uint32_t idx;
    for (idx = 0; idx < (uint32_t)g->chunk && n < kappa; ++idx)
        if (geometry_pos(g, c, idx) >= 0) ++n;
    return n;
}

/*
 * Decode one replica's message for one tensor into a dense fp32 array
 * (zeros where nothing was sent).  Used by tests.
 */
int oracle_decode(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, int quant_mode,
                  const uint16_t* pairs, const float* scales, const float* values,
                  float* dense_out)
{
    geometry g;
    if (geometry_init(&g, rows, cols, chunk_or_tile, tiled) != ORACLE_OK) return ORACLE_EINVAL;
    if (kappa < 1 || !pairs || !dense_out) return ORACLE_EINVAL;
    int64_t n_chunks = geometry_chunks(&g);
    int64_t c, i;
    for (i = 0; i < rows * cols; ++i) dense_out[i] = 0.f;
    for (c = 0; c < n_chunks; ++c) {
        int kappa_c = pairs_in_chunk(&g, c, kappa);
        int t;
        for (t = 0; t < kappa_c; ++t) {
            uint16_t p = pairs[c * (int64_t)kappa + t];
            int64_t where = geometry_pos(&g, c, p & 0x0FFFu);
            if (where < 0) return ORACLE_EINVAL;
            dense_out[where] = decode_pair(p, quant_mode, quant_mode == 1 ? scales + 2 * c : NULL,
                                           quant_mode == 0 ? values[c * (int64_t)kappa + t] : 0.f);
        }
    }
    return ORACLE_OK;
}

/*
 * Section 2.1, line 5 of the update equations, first half:
 *   delta_bar = (1/M) * sum_m hat_m, summed in ascending replica order
 *   starting from +0, then one division by (float)M.
 */
int oracle_aggregate(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, int quant_mode,
                     int n_replicas,
                     const uint16_t* const* pairs, const float* const* scales,
                     const float* const* values, float* delta_bar_out)
{
    geometry g;
    if (geometry_init(&g, rows, cols, chunk_or_tile, tiled) != ORACLE_OK) return ORACLE_EINVAL;
    if (n_replicas < 1 || kappa < 1) return ORACLE_EINVAL;
    int64_t n_chunks = geometry_chunks(&g);
    int64_t c, i;
    int r;
    for (i = 0; i < rows * cols; ++i) delta_bar_out[i] = 0.f;
    for (r = 0; r < n_replicas; ++r) {
        for (c = 0; c < n_chunks; ++c) {
            int kappa_c = pairs_in_chunk(&g, c, kappa);
            int t;
            for (t = 0; t < kappa_c; ++t) {
                uint16_t p = pairs[r][c * (int64_t)kappa + t];
                int64_t where = geometry_pos(&g, c, p & 0x0FFFu);
                if (where < 0) return ORACLE_EINVAL;
                float q = decode_pair(p, quant_mode, quant_mode == 1 ? scales[r] + 2 * c : NULL,
                                      quant_mode == 0 ? values[r][c * (int64_t)kappa + t] : 0.f);
                delta_bar_out[where] = delta_bar_out[where] + q;
            }
        }
    }
    float m = (float)n_replicas;
    for (i = 0; i < rows * cols; ++i) delta_bar_out[i] = delta_bar_out[i] / m;
    return ORACLE_OK;
}

/*
 * Section 2.1, line 5 of the update equations, second half (outer SGD without
 * momentum, appendix hyper-parameter table):  theta = theta - eta * delta_bar.
 */
int oracle_outer_update(int64_t numel, float* theta_outer, const float* delta_bar, float outer_lr)
{
    int64_t i;
    if (numel < 0 || !theta_outer || !delta_bar) return ORACLE_EINVAL;
    for (i = 0; i < numel; ++i) {
        float step = outer_lr * delta_bar[i];
        theta_outer[i] = theta_outer[i] - step;
    }
    return ORACLE_OK;
}

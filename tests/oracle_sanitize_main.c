/*
 * Driver that runs the CPU oracle (oracle/sparseloco_oracle.c, compiled into this program with
 * -fsanitize=address,undefined) over cases read from a file and writes every output to another file.
 * tests/test_oracle_sanitize.py builds it, feeds it the worked example, ragged, tiled and kappa >= n_c cases,
 * and compares the outputs byte for byte with the ordinary build of the oracle.  Any out-of-bounds access or
 * undefined behaviour inside the oracle aborts the program.
 *
 * Input:  int32 n_cases; per case  int64 rows, cols; int32 geom (chunk size, or tile side), tiled, kappa, quant,
 *         n_replicas, mode (0: theta_outer/theta_local, 1: fp32 delta, 2: bf16 delta); float beta, lr;
 *         float theta_outer[numel]; per replica  source[numel] (float, or uint16 for mode 2), float ef[numel].
 * Output: per case, per replica  uint16 pairs[n_chunks * kappa], float aux[n_chunks * (quant ? 2 : kappa)],
 *         float ef[numel]; then float delta_bar[numel], float theta_outer[numel].
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_compress(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, float beta, int quant_mode,
                    const float* theta_outer, const float* theta_local, const float* delta_f32,
                    const uint16_t* delta_bf16, float* ef, uint16_t* pairs_out, float* scales_out, float* values_out);
int oracle_aggregate(int64_t rows, int64_t cols, int chunk_or_tile, int tiled, int kappa, int quant_mode,
                     int n_replicas, const uint16_t* const* pairs, const float* const* scales,
                     const float* const* values, float* delta_bar_out);
int oracle_outer_update(int64_t numel, float* theta_outer, const float* delta_bar, float outer_lr);

static void must_read(void* p, size_t size, size_t n, FILE* f) {
    if (n && fread(p, size, n, f) != n) { fprintf(stderr, "short read\n"); exit(2); }
}
static void must_write(const void* p, size_t size, size_t n, FILE* f) {
    if (n && fwrite(p, size, n, f) != n) { fprintf(stderr, "short write\n"); exit(2); }
}

int main(int argc, char** argv) {
    if (argc != 3) { fprintf(stderr, "usage: %s cases.bin out.bin\n", argv[0]); return 2; }
    FILE* in = fopen(argv[1], "rb");
    FILE* out = fopen(argv[2], "wb");
    if (!in || !out) { fprintf(stderr, "cannot open files\n"); return 2; }
    int32_t n_cases;
    must_read(&n_cases, 4, 1, in);
    for (int c = 0; c < n_cases; ++c) {
        int64_t rows, cols;
        int32_t geom, tiled, kappa, quant, R, mode;
        float beta, lr;
        must_read(&rows, 8, 1, in); must_read(&cols, 8, 1, in);
        must_read(&geom, 4, 1, in); must_read(&tiled, 4, 1, in); must_read(&kappa, 4, 1, in);
        must_read(&quant, 4, 1, in); must_read(&R, 4, 1, in); must_read(&mode, 4, 1, in);
        must_read(&beta, 4, 1, in); must_read(&lr, 4, 1, in);
        const size_t n = (size_t)(rows * cols);
        size_t n_chunks;
        if (tiled && rows > 1) n_chunks = (size_t)(((rows + geom - 1) / geom) * ((cols + geom - 1) / geom));
        else { const size_t ch = tiled ? (size_t)geom * geom : (size_t)geom; n_chunks = (n + ch - 1) / ch; }
        const size_t n_aux = n_chunks * (size_t)(quant ? 2 : kappa);
        /* exact-size heap blocks: one element past any of them is caught */
        float* theta = malloc(n * 4 + 1);
        must_read(theta, 4, n, in);
        uint16_t** pairs = malloc(sizeof(*pairs) * (size_t)R);
        float** aux = malloc(sizeof(*aux) * (size_t)R);
        for (int r = 0; r < R; ++r) {
            void* src = malloc(n * (mode == 2 ? 2 : 4) + 1);
            float* ef = malloc(n * 4 + 1);
            must_read(src, mode == 2 ? 2 : 4, n, in);
            must_read(ef, 4, n, in);
            pairs[r] = malloc(n_chunks * (size_t)kappa * 2 + 1);
            aux[r] = malloc(n_aux * 4 + 1);
            int rc = oracle_compress(rows, cols, geom, tiled, kappa, beta, quant, mode == 0 ? theta : NULL,
                                     mode == 0 ? (const float*)src : NULL, mode == 1 ? (const float*)src : NULL,
                                     mode == 2 ? (const uint16_t*)src : NULL, ef, pairs[r], quant ? aux[r] : NULL,
                                     quant ? NULL : aux[r]);
            if (rc != 0) { fprintf(stderr, "case %d: oracle_compress returned %d\n", c, rc); return 3; }
            must_write(pairs[r], 2, n_chunks * (size_t)kappa, out);
            must_write(aux[r], 4, n_aux, out);
            must_write(ef, 4, n, out);
            free(src); free(ef);
        }
        float* dbar = malloc(n * 4 + 1);
        int rc = oracle_aggregate(rows, cols, geom, tiled, kappa, quant, R, (const uint16_t* const*)pairs,
                                  quant ? (const float* const*)aux : NULL, quant ? NULL : (const float* const*)aux, dbar);
        if (rc != 0) { fprintf(stderr, "case %d: oracle_aggregate returned %d\n", c, rc); return 3; }
        rc = oracle_outer_update((int64_t)n, theta, dbar, lr);
        if (rc != 0) { fprintf(stderr, "case %d: oracle_outer_update returned %d\n", c, rc); return 3; }
        must_write(dbar, 4, n, out);
        must_write(theta, 4, n, out);
        for (int r = 0; r < R; ++r) { free(pairs[r]); free(aux[r]); }
        free(pairs); free(aux); free(dbar); free(theta);
    }
    fclose(in);
    if (fclose(out) != 0) return 2;
    printf("%d cases\n", n_cases);
    return 0;
}

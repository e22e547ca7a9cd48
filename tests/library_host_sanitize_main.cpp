// Host logic of the library under sanitizers: the chunk tables of many shape lists, checked for bounds here too.
#include <cstdio>
#include <cstdint>
#include <cstdlib>
#include <vector>
#include "sparseloco.h"
struct Entry { uint32_t tensor, n_c; uint64_t offset; uint32_t stride; uint8_t h, w, last_w, vec; uint32_t id, strip; };
static uint64_t rng_state = 88172645463325252ull;
static uint64_t rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return rng_state; }
int main() {
    static_assert(sizeof(Entry) == 32, "entry size");
    long checked = 0;
    for (int iter = 0; iter < 400; ++iter) {
        const int n = 1 + (int)(rnd() % 12);
        std::vector<int64_t> rows(n), cols(n);
        for (int i = 0; i < n; ++i) {
            const int kind = (int)(rnd() % 6);
            rows[i] = kind == 0 ? 1 : (kind == 1 ? 0 : 1 + (int64_t)(rnd() % 300));
            cols[i] = kind == 2 ? 0 : 1 + (int64_t)(rnd() % (kind == 3 ? 6000 : 700));
        }
        for (int layout = 0; layout < 2; ++layout) {
            const int64_t nc = sparseloco_chunk_table(n, rows.data(), cols.data(), layout, nullptr, 0);
            if (nc < 0) { printf("negative count %ld\n", (long)nc); return 1; }
            std::vector<Entry> t((size_t)nc + 1);
            const int64_t nc2 = sparseloco_chunk_table(n, rows.data(), cols.data(), layout, t.data(), nc);
            if (nc2 != nc) { printf("count changed\n"); return 1; }
            std::vector<char> seen((size_t)nc, 0);
            for (int64_t c = 0; c < nc; ++c) {
                const Entry& e = t[(size_t)c];
                if (e.tensor >= (uint32_t)n || e.id >= (uint32_t)nc || seen[e.id]) { printf("bad entry\n"); return 1; }
                seen[e.id] = 1;
                const uint64_t numel = (uint64_t)rows[e.tensor] * (uint64_t)cols[e.tensor];
                uint64_t present = 0;
                for (uint32_t idx = 0; idx < 4096; ++idx) {
                    const uint32_t r = idx / 64, k = idx % 64;
                    const bool in = (r + 1 < e.h && k < e.w) || (r + 1 == e.h && k < e.last_w);
                    if (!in) continue;
                    ++present;
                    if (e.offset + (uint64_t)r * e.stride + k >= numel) { printf("out of bounds\n"); return 1; }
                }
                if (present != e.n_c) { printf("n_c mismatch %lu %u\n", (unsigned long)present, e.n_c); return 1; }
                ++checked;
            }
        }
    }
    // refusals
    int64_t bad[1] = {-1}, one[1] = {1};
    if (sparseloco_chunk_table(1, one, bad, 0, nullptr, 0) >= 0) return 2;
    if (sparseloco_chunk_table(0, one, one, 0, nullptr, 0) >= 0) return 2;
    if (sparseloco_chunk_table(1, one, one, 7, nullptr, 0) >= 0) return 2;
    printf("ok: %ld chunk entries checked\n", checked);
    return 0;
}

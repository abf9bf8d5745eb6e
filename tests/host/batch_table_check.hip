// Host-only check of the bucket lookup of the batched launches (csrc/batch.hpp): for random bucket lists, the table
// that batch_fill_lut writes and batch_find reads must name, for every unit of the launch, the bucket a linear scan
// over the buckets' first units names.  Built with `hipcc --cuda-host-only` by tests/test_batch_table_cpu.py.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "batch.hpp"
using namespace bagua;
int main()
{
    unsigned long long seed = 12345;
    auto rnd = [&]() { seed = seed * 6364136223846793005ull + 1442695040888963407ull; return (unsigned)(seed >> 33); };
    long checked = 0;
    for (int trial = 0; trial < 400; ++trial) {
        const size_t B = 1 + rnd() % (trial < 200 ? 40 : 1500);
        const size_t ew = 5;
        std::vector<uint64_t> table(batch_table_words(B, ew), 0);
        size_t total = 0;
        const int mode = trial % 4;
        for (size_t b = 0; b < B; ++b) {
            table[b] = total;
            size_t units = mode == 0 ? 1 : mode == 1 ? 1 + rnd() % 7 : mode == 2 ? 1 + rnd() % 5000 : (rnd() % 50 == 0 ? 1 + rnd() % 200000 : 1);
            total += units;
        }
        table[B] = total;
        batch_fill_lut(table.data(), B, ew);
        const BatchView bv = batch_view(table.data(), B, ew, total);
        size_t want = 0;
        const size_t stride = total > 3000000 ? 7 : 1;
        for (size_t g = 0; g < total; g += stride) {
            while (table[want + 1] <= g) ++want;
            const uint32_t got = batch_find(bv, g);
            if (got != want) { std::printf("MISMATCH trial %d B %zu g %zu got %u want %zu\n", trial, B, g, got, want); return 1; }
            ++checked;
        }
        if (batch_find(bv, total - 1) != B - 1) { std::printf("LAST trial %d\n", trial); return 1; }
    }
    std::printf("OK %ld\n", checked);
    return 0;
}

// Driver for the sanitizer run of tests/test_sanitizers.py: the host-only part of the library
// (codebook and search-table builder, csrc/q8opt_host.cpp, linked in as source) on buffers of
// exactly the documented sizes, every 16-bit key of the table looked up, good and bad codebooks.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "q8opt.h"

int main()
{
    long checks = 0;
    for (int is_signed = 0; is_signed < 2; ++is_signed) {
        float* q = static_cast<float*>(std::malloc(256 * sizeof(float)));
        if (q8_build_codebook(is_signed, q) != Q8_OK) return 2;
        void* tab = std::malloc(q8_qtable_bytes());
        if (q8_build_qtable(q, tab) != Q8_OK) return 3;
        for (uint32_t key = 0; key < 65536; ++key) {               // every bucket, also NaN and Inf patterns
            const uint32_t bits = key << 16;
            float x;
            std::memcpy(&x, &bits, 4);
            const int c = q8_host_nearest_code(tab, x);
            if (c < 0 || c > 255) return 4;
            ++checks;
        }
        // codebooks the builder must refuse without reading or writing out of bounds
        float bad[256];
        std::memcpy(bad, q, sizeof bad);
        bad[10] = bad[9];
        if (q8_build_qtable(bad, tab) != Q8_ECODEBOOK) return 5;
        std::memcpy(bad, q, sizeof bad);
        bad[255] = 1.5f;
        if (q8_build_qtable(bad, tab) != Q8_ECODEBOOK) return 6;
        for (int j = 0; j < 256; ++j) bad[j] = -1.0f + 2.0f * (float)j / 255.0f;      // linear map: accepted
        if (q8_build_qtable(bad, tab) != Q8_OK) return 7;
        for (int j = 0; j < 256; ++j) bad[j] = 0.5f + std::ldexp((float)j, -24);          // 256 neighbouring values: too fine for the table
        if (q8_build_qtable(bad, tab) == Q8_OK) return 8;
        std::free(tab);
        std::free(q);
    }
    if (q8_build_codebook(1, nullptr) != Q8_EINVAL || q8_build_qtable(nullptr, nullptr) != Q8_EINVAL) return 9;
    for (int s = 1; s >= -9; --s) (void)q8_status_str(s);
    std::printf("host sanitizer driver: %ld lookups ok\n", checks);
    return 0;
}

// Layout of the search table ("qtable") shared by the host builder and the kernels.
#pragma once
#include <stdint.h>

namespace q8 {

// The table is one flat byte blob (device copy 16-byte aligned):
//   [0, 64)          header (QTabHeader)
//   [64, 1088)       codebook Q^map, 256 binary32 values, ascending
//   [1088, 2112)     thresholds: thr[j] = first binary32 above (Q_j + Q_j+1)/2 for
//                    j < 255, thr[255] = NaN (no x, not even +Inf, compares >= it); code(x) = #{j : thr[j] <= x}
//   [2112, 67648)    bucket table, one byte per bucket, indexed by the upper 16
//                    bits of the binary32 pattern of x (sign, exponent, 7 mantissa
//                    bits).  The entry is the code of the smallest x in the bucket;
//                    every bucket with |x| <= 1 holds at most one threshold, so
//                    code(x) = c + (x >= thr[c]).  Buckets beyond |x| = 1 hold the
//                    code of +1 or -1, so that any bit pattern indexes safely.
struct QTabHeader {
    uint32_t magic;      // kMagic
    uint32_t key_bits;   // 16
    uint32_t zero_code;  // code(0.0)
    uint32_t pad[13];
};
static_assert(sizeof(QTabHeader) == 64, "header is 64 bytes");

constexpr uint32_t kMagic = 0x51384f51u;      // "Q8OQ"
constexpr int kOffQmap = 64;
constexpr int kOffThr = kOffQmap + 1024;
constexpr int kOffLut = kOffThr + 1024;
constexpr int kLutEntries = 65536;
constexpr int kQTabBytes = kOffLut + kLutEntries;          // 67648
constexpr uint32_t kKeyOne = 0x3f80;                        // upper half of 1.0f
static_assert(kQTabBytes % 64 == 0, "table size is a multiple of 64");

}  // namespace q8

// Layout of the search table ("qtable") shared by the host builder and the kernels.
#pragma once
#include <stdint.h>

namespace q8 {

// The table is one flat byte blob so that a kernel can stage it into LDS with
// 128-bit copies:
//   [0, 64)        header (QTabHeader)
//   [64, 1088)     codebook  Q^map, 256 binary32 values, ascending
//   [1088, 2112)   thresholds: thr[j] = first binary32 above (Q_j + Q_j+1)/2 for
//                  j < 255, thr[255] = +inf; code(x) = #{j : thr[j] <= x}
//   [2112, ...)    bucket table, one byte per bucket: 2*L entries, the first L
//                  for x >= 0 and the next L for x < 0.  The bucket of x is
//                  clamp((|x| bits >> shift) - kbase, 0, L-1): the binary
//                  exponent and the top M mantissa bits of |x|, counted from
//                  2^-24 (everything smaller shares bucket 0; |x| = 1 is the
//                  last bucket).  The entry is the code of the smallest x in
//                  the bucket; every bucket holds at most one threshold, so
//                  code(x) = c + (x >= thr[c]).
struct QTabHeader {
    uint32_t magic;      // kMagic
    uint32_t M;          // mantissa bits in the bucket key
    uint32_t shift;      // 23 - M
    uint32_t width;      // 8 + M  (exponent + mantissa bits kept)
    uint32_t kbase;      // (127 - 24) << M
    uint32_t L;          // 24 * 2^M + 1 buckets per sign
    uint32_t zero_code;  // code(0.0)
    uint32_t pad[9];
};
static_assert(sizeof(QTabHeader) == 64, "header is 64 bytes");

constexpr uint32_t kMagic = 0x51384f50u;      // "Q8OP"
constexpr int kMaxM = 7;
constexpr int kMinExp = 24;                    // buckets start at 2^-24
constexpr int kOffQmap = 64;
constexpr int kOffThr = kOffQmap + 1024;
constexpr int kOffLut = kOffThr + 1024;
constexpr int kLutMax = 2 * (kMinExp * (1 << kMaxM) + 1);   // 6146
constexpr int kQTabBytes = 8320;               // multiple of 64, >= kOffLut + kLutMax
static_assert(kOffLut + kLutMax <= kQTabBytes, "table fits");

}  // namespace q8

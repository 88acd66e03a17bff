// Host-side parts of the library: codebook, search-table builder, status strings.
// No GPU calls in this file.
#include <cmath>
#include <cstring>
#include <limits>

#include "q8opt.h"
#include "q8opt_internal.h"

using namespace q8;

extern "C" const char* q8_status_str(q8_status s)
{
    switch (s) {
    case Q8_OK: return "Q8_OK";
    case Q8_EINVAL: return "Q8_EINVAL: invalid argument";
    case Q8_EALIGN: return "Q8_EALIGN: misaligned pointer";
    case Q8_EBLOCK: return "Q8_EBLOCK: block size must be a power of two in [64, 4096]";
    case Q8_ELAUNCH: return "Q8_ELAUNCH: HIP launch or copy failed";
    case Q8_ENOMEM: return "Q8_ENOMEM: device allocation failed";
    case Q8_ECODEBOOK: return "Q8_ECODEBOOK: unusable codebook";
    case Q8_ELIMIT: return "Q8_ELIMIT: list exceeds the static workspace (1024 tensors, 131072 units)";
    default: return "unknown q8_status";
    }
}

// Dynamic-tree codebook (Sec. IV-B): decade E holds 2^F bin centres of the
// mantissa range [0.1, 1] scaled by 10^-E, with F = 6-E (signed) or 7-E
// (unsigned); plus 0 and +1.  Emitted directly in ascending order.
extern "C" q8_status q8_build_codebook(int is_signed, float* qmap_out)
{
    if (!qmap_out) return Q8_EINVAL;
    const int fbits0 = is_signed ? 6 : 7;
    float mags[254];
    int nm = 0;
    for (int E = 6; E >= 0; --E) {                 // smallest decade first
        const int F = fbits0 - E;
        double scale = 1.0;
        for (int e = 0; e < E; ++e) scale *= 10.0;
        for (int k = 0; k < (1 << F); ++k) {
            double frac = 0.1 + (0.9 * (double)(2 * k + 1)) / (double)(1 << (F + 1));
            mags[nm++] = (float)(frac / scale);
        }
    }
    int o = 0;
    if (is_signed) {
        for (int i = nm - 1; i >= 0; --i) qmap_out[o++] = -mags[i];
    }
    qmap_out[o++] = 0.0f;
    for (int i = 0; i < nm; ++i) qmap_out[o++] = mags[i];
    qmap_out[o++] = 1.0f;
    return (o == 256) ? Q8_OK : Q8_ECODEBOOK;
}

extern "C" size_t q8_qtable_bytes(void) { return (size_t)kQTabBytes; }

namespace {

inline float bits_to_float(uint32_t b) { float f; std::memcpy(&f, &b, 4); return f; }
inline uint32_t float_to_bits(float f) { uint32_t b; std::memcpy(&b, &f, 4); return b; }

// number of thresholds <= x
int count_le(const float* thr, float x)
{
    int lo = 0, hi = 255;                          // thr[255] is not a threshold: never looked at
    while (lo < hi) {
        int mid = (lo + hi) / 2;
        if (thr[mid] <= x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

}  // namespace

extern "C" q8_status q8_build_qtable(const float* qmap, void* qtable_out)
{
    if (!qmap || !qtable_out) return Q8_EINVAL;
    for (int j = 0; j < 256; ++j) {
        if (!(qmap[j] >= -1.0f && qmap[j] <= 1.0f)) return Q8_ECODEBOOK;
        if (j && !(qmap[j] > qmap[j - 1])) return Q8_ECODEBOOK;
        // every decision threshold stays far above the subnormal quotients, whose last bits the
        // kernels' short division does not guarantee
        if (qmap[j] != 0.0f && std::fabs(qmap[j]) < 0x1p-99f) return Q8_ECODEBOOK;
    }
    unsigned char* blob = static_cast<unsigned char*>(qtable_out);
    std::memset(blob, 0, kQTabBytes);
    float* q = reinterpret_cast<float*>(blob + kOffQmap);
    float* thr = reinterpret_cast<float*>(blob + kOffThr);
    unsigned char* lut = blob + kOffLut;
    std::memcpy(q, qmap, 1024);

    // Thresholds.  The midpoint of two binary32 values within [-1, 1] whose
    // magnitudes are either zero or at least 2^-100 is exact in binary64.
    for (int j = 0; j < 255; ++j) {
        double mid = ((double)q[j] + (double)q[j + 1]) * 0.5;
        float f = (float)mid;
        if (!((double)f > mid)) f = std::nextafterf(f, std::numeric_limits<float>::infinity());
        thr[j] = f;
        if (j && !(thr[j] > thr[j - 1])) return Q8_ECODEBOOK;
    }
    thr[255] = std::numeric_limits<float>::quiet_NaN();      // x >= thr[255] is false for every x: code 255 is the last

    // Bucket table over all 65536 upper halves of a binary32 pattern.
    const int code_p1 = count_le(thr, 1.0f), code_m1 = count_le(thr, -1.0f);
    for (uint32_t key = 0; key < (uint32_t)kLutEntries; ++key) {
        const bool neg = (key >> 15) != 0;
        const uint32_t a = key & 0x7fffu;
        int c;
        if (a > kKeyOne) {                                  // |x| > 1, Inf, NaN: clamp
            c = neg ? code_m1 : code_p1;
        } else {
            const float lo = bits_to_float(a << 16);
            const float hi = (a == kKeyOne) ? 1.0f : bits_to_float((a << 16) | 0xffffu);
            const int c0 = neg ? count_le(thr, -hi) : count_le(thr, lo);
            const int c1 = neg ? count_le(thr, -lo) : count_le(thr, hi);
            if (c1 - c0 > 1) return Q8_ECODEBOOK;          // two thresholds in one bucket
            c = c0;
        }
        lut[key] = (unsigned char)c;
    }
    QTabHeader h{};
    h.magic = kMagic;
    h.key_bits = 16;
    h.zero_code = (uint32_t)count_le(thr, 0.0f);
    std::memcpy(blob, &h, sizeof h);
    return Q8_OK;
}

extern "C" int q8_host_nearest_code(const void* qtable, float x)
{
    if (!qtable) return Q8_EINVAL;
    const unsigned char* blob = static_cast<const unsigned char*>(qtable);
    QTabHeader h;
    std::memcpy(&h, blob, sizeof h);
    if (h.magic != kMagic) return Q8_EINVAL;
    const float* thr = reinterpret_cast<const float*>(blob + kOffThr);
    const unsigned char* lut = blob + kOffLut;
    const uint32_t idx = float_to_bits(x) >> 16;
    int c = lut[idx];
    return c + (x >= thr[c] ? 1 : 0);
}

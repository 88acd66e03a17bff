// Device code of the fused 8-bit optimizer step for gfx950, shared by the translation units
// of the library (one per storage type of w and g, so that they compile in parallel).
//
// Work decomposition: one wave64 owns 1024 consecutive elements of one tensor, read
// as 4 rows of 256 elements; lane l of the wave holds elements [256 r + 4 l,
// 256 r + 4 l + 4) of row r, so every fp32 access is one coalesced 128-bit
// load/store per lane and every code access one coalesced 32-bit one.  New states
// stay in registers between the update and the re-quantization, so HBM is touched
// once per byte.  The block absmax is reduced with DPP steps inside the wave; for
// B <= 1024 a wave holds whole blocks, for B = 2048 (4096) the 2 (4) waves that
// share a block exchange their maxima through LDS with one barrier.
//
// Scheduling: workgroups of 8 waves are persistent.  They stage the search tables
// into 64 KB of LDS once and then draw "jobs" of 8 consecutive wave tiles from an
// atomic counter in device memory.  Handing work out in address order to whichever
// workgroup is free keeps the set of addresses in flight one dense, slowly
// advancing window over each stream, which is what the HBM controllers reward: on
// a bandwidth skeleton of this access pattern a static grid-stride assignment
// reached 5.1 TB/s, chunks 5.4 TB/s, dynamic jobs of 8 x 2048 elements 5.9 TB/s and
// dynamic jobs of 8 x 1024 elements (half the window) 6.4 TB/s.
//
// Every wave of a workgroup passes the same two barrier sites per job (one in the
// draw, one in the exchange of block maxima), whatever kind of tile it holds: a
// tile is processed in two phases (update, then re-quantization) around the
// exchange, and the branches on the kind of tile sit inside the phases.
//
// Nearest-code search (Eq. quant2): the upper 16 bits of the binary32 pattern of
// x = m / N index a byte table in LDS that holds the code at the lower end of that
// bucket; one threshold read and one compare finish the decision exactly.
//
// Exact arithmetic: the update formulas are written one operation per statement
// and the file is compiled with -ffp-contract=off.  The normalisation x = m / N
// (Eq. quant1) is a correctly rounded quotient: N is uniform over a block, so
// y = RN(1/N) is formed once and each element takes a product and one
// residual-correction fma pair (q8opt_exact.h states why that is exact); blocks
// whose N lies outside [2^-60, 2^60] use the plain divide.  The
// square root and the division of the Adam weight update take short, equally exact
// forms on rows whose new states all lie in [2^-80, 2^40], sqrtf and a / b otherwise.
//
// Storage type: weights and gradients are binary32, bfloat16 or binary16 (template
// parameter WT of the step kernels); the arithmetic and the 8-bit states are the same.
#ifndef Q8OPT_DEVICE_H
#define Q8OPT_DEVICE_H

#include <hip/hip_runtime.h>

#include <stdint.h>

#include <atomic>

#include "q8opt.h"
#include "q8opt_exact.h"
#include "q8opt_internal.h"

namespace q8 {

// ---------------------------------------------------------------------------
// Types and functions shared between the translation units of the library.
// ---------------------------------------------------------------------------
struct TensorDesc {                       // device-side mirror of q8_tensor
    void* w;                              // float or bfloat16 elements: fixed by the kernel's WT
    const void* g;
    uint8_t* m_q;
    uint8_t* r_q;
    float* N_m;
    float* N_r;
    float* m_f32;
    float* r_f32;
    int64_t n;
};

struct TileRef { int32_t tensor; int32_t tile; };

struct AdamScalars {
    float beta1, beta2, omb1, omb2, eps, wd, alpha_t, isbc2, alpha_wd;
    int wd_mode;                          // 0 none, 1 coupled (g += wd*w), 2 decoupled
    int bias;                             // bias-correction extension: scale the root by isbc2, step alpha_t
    int fast_ok;                          // eps and isbc2 allow the short square root / division
};
struct SgdScalars { float alpha, beta, wd; };

// Job counter of the dynamic scheduler (see "Dynamic scheduling" below).
struct Sched { unsigned long long next, done; };

struct StepArgs {
    const TensorDesc* descs;      // device list, or nullptr: use `single`
    const TileRef* tiles;         // device unit table for lists, else nullptr
    TensorDesc single;
    int64_t nunits;
    const void* qtab_s;
    const void* qtab_u;
    Sched* sched;
};

// Defined once, in q8opt_kernels.hip.  device_cus: CU count of the current device.
// acquire_sched: the job counter this launch on `stream` may use without sharing it with any
// launch that can run at the same time, or nullptr: then the kernel walks its jobs in a
// fixed grid-stride order and needs no counter.
q8_status device_cus(int& cus);
q8_status acquire_sched(hipStream_t stream, Sched** out);

// Everything below has internal linkage: each translation unit instantiates only the
// kernels it launches.
namespace {

constexpr int kWgThreads = 512;
constexpr int kWavesPerWg = kWgThreads / 64;
constexpr int kMinWavesPerEu = 4;         // launch bound: two workgroups per CU, up to 128 VGPRs
constexpr int kRow = 256;                 // elements per wave row: 64 lanes x 4

// Pointers into HBM carry the global address space so that loads and stores
// are global_* instructions (a generic pointer would make them flat_*).
#define Q8_GLOBAL __attribute__((address_space(1)))
typedef Q8_GLOBAL float gfloat;
typedef Q8_GLOBAL const float gcfloat;
typedef Q8_GLOBAL uint8_t gbyte;
typedef Q8_GLOBAL const uint8_t gcbyte;
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef Q8_GLOBAL v4f gfloat4;
typedef Q8_GLOBAL const v4f gcfloat4;
typedef Q8_GLOBAL uint32_t gu32;
typedef Q8_GLOBAL const uint32_t gcu32;
typedef Q8_GLOBAL const v4u gcuint4;
typedef Q8_GLOBAL uint16_t gu16;
typedef Q8_GLOBAL const uint16_t gcu16;
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef Q8_GLOBAL v2u gv2u;
typedef Q8_GLOBAL const v2u gcv2u;




// ---------------------------------------------------------------------------
// LDS map (52 KB per workgroup, so that three workgroups fit a CU's 160 KB).  The bucket
// table is indexed by the upper half of a binary32 pattern: keys of x in [0, 1] are
// 0 .. 0x3F80 and keys of x in [-1, -0] are 0x8000 .. 0xBF80, which leaves two holes.  The
// first hole hosts the non-negative half of the second table (used for the state r >= 0),
// the space above the negative keys the two codebooks and threshold arrays.  Finite inputs
// give |x| <= 1 and stay inside the staged ranges; any other bit pattern (NaN, Inf) is
// clamped to the last byte of the map, so that every access stays inside the 52 KB.
// ---------------------------------------------------------------------------
constexpr int kLdsBytes = 0xD000;
constexpr int kLutHalf = 0x3F90;          // bytes staged per half: keys 0 .. 0x3F8F
constexpr int kLdsNeg = 0x8000;           // keys of negative x
constexpr int kLdsU = 0x3F90;             // second table, keys of x >= 0
constexpr int kLdsQ1 = 0xC000;            // first table: codebook, then thresholds
constexpr int kLdsT1 = 0xC400;
constexpr int kLdsQ2 = 0xC800;            // second table
constexpr int kLdsT2 = 0xCC00;
constexpr uint32_t kLdsLastKey = kLdsBytes - 1;
static_assert(kLdsU + kLutHalf <= kLdsNeg && kLdsNeg + kLutHalf <= kLdsQ1 && kLdsT2 + 1024 <= kLdsBytes, "LDS map");
static_assert(kLdsU + 0x7fff < kLdsBytes, "every 15-bit key of the second table stays inside the map");

// Staging of the search tables.  A copy of BYTES bytes takes ceil(BYTES / 16 / kWgThreads)
// 16-byte pieces per thread; all loads of all copies are issued before the first LDS store
// waits for its data, so that the workgroup pays one round trip to L2 for its tables, not
// one per piece.
template <int BYTES>
struct Copy16 {
    static constexpr int N = BYTES / 16, K = (N + kWgThreads - 1) / kWgThreads;
    v4u v[K];
    __device__ __forceinline__ void load(const unsigned char* src, int tid)
    {
        gcuint4* s4 = (gcuint4*)src;
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (k * kWgThreads + tid < N) v[k] = s4[k * kWgThreads + tid];
    }
    __device__ __forceinline__ void store(unsigned char* dst, int tid) const
    {
        v4u* d4 = reinterpret_cast<v4u*>(dst);
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (k * kWgThreads + tid < N) d4[k * kWgThreads + tid] = v[k];
    }
};

// first table (both signs) and, if qtab_u != nullptr, the second one (non-negative half only)
__device__ __forceinline__ void stage_tables(unsigned char* lds, const void* qtab_s, const void* qtab_u, int tid)
{
    const unsigned char* s = static_cast<const unsigned char*>(qtab_s);
    const unsigned char* u = static_cast<const unsigned char*>(qtab_u);
    Copy16<kLutHalf> pos, neg, upos;
    Copy16<2048> q1, q2;
    pos.load(s + kOffLut, tid);
    neg.load(s + kOffLut + 0x8000, tid);
    q1.load(s + kOffQmap, tid);
    if (u) {
        upos.load(u + kOffLut, tid);
        q2.load(u + kOffQmap, tid);
    }
    pos.store(lds, tid);
    neg.store(lds + kLdsNeg, tid);
    q1.store(lds + kLdsQ1, tid);
    if (u) {
        upos.store(lds + kLdsU, tid);
        q2.store(lds + kLdsQ2, tid);
    }
}

// Nearest code of x (Eq. quant2) by bucket lookup + one exact threshold compare.
// SECOND selects the second table, whose inputs are non-negative.
template <bool SECOND>
__device__ __forceinline__ uint32_t nearest_code(const unsigned char* lds, float x)
{
    const uint32_t bits = __float_as_uint(x);
    uint32_t c;
    float t;
    if (SECOND) {
        c = lds[kLdsU + __builtin_amdgcn_ubfe(bits, 16, 15)];
        t = *reinterpret_cast<const float*>(lds + kLdsT2 + 4 * c);
    } else {
        const uint32_t key = bits >> 16;
        c = lds[key < kLdsLastKey ? key : kLdsLastKey];
        t = *reinterpret_cast<const float*>(lds + kLdsT1 + 4 * c);
    }
    return c + ((x >= t) ? 1u : 0u);
}

template <bool SECOND>
__device__ __forceinline__ float dequant(const unsigned char* lds, uint32_t code, float N)
{
    return *reinterpret_cast<const float*>(lds + (SECOND ? kLdsQ2 : kLdsQ1) + 4 * code) * N;
}

// ---------------------------------------------------------------------------
// Cross-lane max of non-negative binary32 values held as bit patterns (the
// unsigned-integer order of such patterns is their numeric order).
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max_step(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
    return max(v, o);
}

// max over each aligned group of GROUP lanes, returned in every lane of the group
template <int GROUP>
__device__ __forceinline__ uint32_t group_max(uint32_t v, int lane)
{
    v = dpp_max_step<0xB1>(v);            // quad_perm [1,0,3,2]
    v = dpp_max_step<0x4E>(v);            // quad_perm [2,3,0,1]
    v = dpp_max_step<0x141>(v);           // row_half_mirror
    v = dpp_max_step<0x140>(v);           // row_mirror: every lane has its 16-lane max
    if (GROUP >= 32) {
        uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 16) << 2, (int)v);
        v = max(v, o);
    }
    if (GROUP >= 64) {
        uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
        uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
        v = max(a, b);
    }
    return v;
}

using exact::div_fast;
using exact::norm_in_fast_range;
using exact::kFastLo;
using exact::kFastHi;

__device__ __forceinline__ float div_any(float a, float N)
{
    return (N == 0.0f) ? 0.0f : a / N;
}

struct BlockNorm { float N, y; bool fast; };

// Reciprocal data of one block maximum held per lane (used when lanes of a wave
// belong to different blocks, B < 256).
__device__ __forceinline__ BlockNorm make_norm(uint32_t nbits)
{
    BlockNorm b;
    b.N = __uint_as_float(nbits);
    b.fast = norm_in_fast_range(nbits);
    b.y = exact::reciprocal_rn(b.fast ? b.N : 1.0f);
    return b;
}

// Reciprocal data of K wave-uniform block maxima with ONE division sequence: the
// K values are spread over lanes 0..K-1, divided there, and read back.
template <int K>
__device__ __forceinline__ void make_norms(const uint32_t (&nbits)[K], BlockNorm (&out)[K], int lane)
{
    int v = (int)nbits[0];
#pragma unroll
    for (int k = 1; k < K; ++k) v = (lane == k) ? (int)nbits[k] : v;
    const float y = exact::reciprocal_rn(norm_in_fast_range((uint32_t)v) ? __int_as_float(v) : 1.0f);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        out[k].N = __uint_as_float(nbits[k]);
        out[k].fast = norm_in_fast_range(nbits[k]);
        out[k].y = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y), k));
    }
}

// Short forms of the square root and of the division in the Adam weight update (q8opt_exact.h),
// seeded with the hardware's approximate reciprocal and reciprocal square root; used on rows where every
// new state lies in [kFastLo, kFastHi], all other rows take sqrtf and the general a / b.
__device__ __forceinline__ float div_rn_inrange(float a, float b)
{
    return exact::div_rn_from_seed(a, b, __builtin_amdgcn_rcpf(b));
}

__device__ __forceinline__ float sqrt_rn_fast(float r)
{
    return exact::sqrt_rn_from_rsq(r, __builtin_amdgcn_rsqf(r));
}

// ---------------------------------------------------------------------------
// Per-lane row access.  cnt = number of valid elements (0..4) of this lane in
// the row; FULL tiles have cnt == 4 everywhere.  The bulk data is touched once
// per step, so full-width accesses carry the non-temporal hint.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int lane_count(int64_t n, int64_t e0)
{
    int64_t left = n - e0;
    return left >= 4 ? 4 : (left <= 0 ? 0 : (int)left);
}

// Running maximum of |x| over a lane's elements, kept as the bit pattern of a
// non-negative float (finite inputs: the order of such floats is the order of their
// bit patterns).  Written as a float maximum so that it compiles to v_max3_f32 with
// |.| source modifiers, two elements per instruction.
__device__ __forceinline__ uint32_t absmax4(uint32_t acc, const float (&v)[4])
{
    float a = __uint_as_float(acc);
    a = __builtin_fmaxf(__builtin_fmaxf(a, __builtin_fabsf(v[0])), __builtin_fabsf(v[1]));
    a = __builtin_fmaxf(__builtin_fmaxf(a, __builtin_fabsf(v[2])), __builtin_fabsf(v[3]));
    return __float_as_uint(a);
}

__device__ __forceinline__ void load4f(gcfloat* p, int cnt, float (&v)[4])
{
    if (cnt == 4) {
        const v4f t = __builtin_nontemporal_load((gcfloat4*)p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (j < cnt) ? p[j] : 0.0f;
    }
}

__device__ __forceinline__ void store4f(gfloat* p, int cnt, const float (&v)[4])
{
    if (cnt == 4) {
        const v4f t = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(t, (gfloat4*)p);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < cnt) p[j] = v[j];
    }
}

__device__ __forceinline__ uint32_t load4b(gcbyte* p, int cnt)
{
    if (cnt == 4) return __builtin_nontemporal_load((gcu32*)p);
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (j < cnt) v |= (uint32_t)p[j] << (8 * j);
    return v;
}

__device__ __forceinline__ void store4b(gbyte* p, int cnt, uint32_t v)
{
    if (cnt == 4) {
        __builtin_nontemporal_store(v, (gu32*)p);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < cnt) p[j] = (uint8_t)(v >> (8 * j));
    }
}

// Storage type WT of weights and gradients: float, Bf16 (bfloat16 = the upper half of
// a binary32) or F16 (IEEE binary16).  Widening is exact; narrowing is the hardware's
// round-to-nearest-even conversion (v_cvt_pk_bf16_f32 / v_cvt_pk_f16_f32, binary16
// subnormals kept), applied once to the new weight.
struct Bf16 { uint16_t bits; };
struct F16 { uint16_t bits; };

template <typename WT> struct Wide;
template <> struct Wide<float> { typedef gfloat* ptr; typedef gcfloat* cptr; };
template <> struct Wide<Bf16> { typedef gu16* ptr; typedef gcu16* cptr; };
template <> struct Wide<F16> { typedef gu16* ptr; typedef gcu16* cptr; };

// Launch shape of the step kernels by storage type of w and g.  With binary32 storage the step
// is bound by its memory access pattern: two workgroups per CU (16 waves, up to 128 VGPRs) and
// one job per draw measured best.  With 16-bit storage it moves 10 instead of 16 bytes per
// parameter and is bound by instruction issue: three workgroups per CU (24 waves, 80 VGPRs; the
// 52 KB LDS map fits three times) measured 6 % faster there (3 % slower with binary32), two jobs
// per draw another 2 % (7 % slower with binary32: a wider window of addresses in flight).
template <typename WT> struct Occupancy { static constexpr int kWgPerCu = 2, kSpan = 1; };
template <> struct Occupancy<Bf16> { static constexpr int kWgPerCu = 3, kSpan = 2; };
template <> struct Occupancy<F16> { static constexpr int kWgPerCu = 3, kSpan = 2; };

template <typename WT> __device__ __forceinline__ void widen2(uint32_t pair, float& lo, float& hi);
template <> __device__ __forceinline__ void widen2<Bf16>(uint32_t pair, float& lo, float& hi)
{
    lo = __uint_as_float(pair << 16);
    hi = __uint_as_float(pair & 0xffff0000u);
}
template <> __device__ __forceinline__ void widen2<F16>(uint32_t pair, float& lo, float& hi)
{
    const v2f f = __builtin_convertvector(__builtin_bit_cast(v2h, pair), v2f);
    lo = f.x;
    hi = f.y;
}

template <typename WT> __device__ __forceinline__ uint32_t narrow2(float lo, float hi);
template <> __device__ __forceinline__ uint32_t narrow2<Bf16>(float lo, float hi)
{
    const v2f x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, v2bf));
}
template <> __device__ __forceinline__ uint32_t narrow2<F16>(float lo, float hi)
{
    const v2f x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, v2h));
}

// Four loaded elements as they sit in registers until they are used: binary32 values as
// they are, 16-bit values still packed in pairs (widened only where the arithmetic starts,
// which keeps a tile's loads in half the registers).
template <typename WT> struct Raw4 { uint32_t a, b; };
template <> struct Raw4<float> { float v[4]; };

template <typename WT>
__device__ __forceinline__ void load4raw(gcfloat* p, int cnt, Raw4<float>& out) { load4f(p, cnt, out.v); }
template <typename WT>
__device__ __forceinline__ void store4w(gfloat* p, int cnt, const float (&v)[4]) { store4f(p, cnt, v); }

template <typename WT>
__device__ __forceinline__ void load4raw(gcu16* p, int cnt, Raw4<WT>& out)
{
    if (cnt == 4) {
        const v2u t = __builtin_nontemporal_load((gcv2u*)p);
        out.a = t.x;
        out.b = t.y;
    } else {
        uint32_t h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) h[j] = (j < cnt) ? (uint32_t)p[j] : 0u;
        out.a = h[0] | (h[1] << 16);
        out.b = h[2] | (h[3] << 16);
    }
}

__device__ __forceinline__ void zero4raw(Raw4<float>& x) { x.v[0] = x.v[1] = x.v[2] = x.v[3] = 0.0f; }
template <typename WT> __device__ __forceinline__ void zero4raw(Raw4<WT>& x) { x.a = 0; x.b = 0; }

__device__ __forceinline__ void widen4(const Raw4<float>& x, float (&v)[4])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = x.v[j];
}
template <typename WT>
__device__ __forceinline__ void widen4(const Raw4<WT>& x, float (&v)[4])
{
    widen2<WT>(x.a, v[0], v[1]);
    widen2<WT>(x.b, v[2], v[3]);
}

template <typename WT, typename P>
__device__ __forceinline__ void load4w(P p, int cnt, float (&v)[4])
{
    Raw4<WT> raw;
    load4raw<WT>(p, cnt, raw);
    widen4(raw, v);
}

template <typename WT>
__device__ __forceinline__ void store4w(gu16* p, int cnt, const float (&v)[4])
{
    const uint32_t a = narrow2<WT>(v[0], v[1]), b = narrow2<WT>(v[2], v[3]);
    if (cnt == 4) {
        const v2u t = {a, b};
        __builtin_nontemporal_store(t, (gv2u*)p);
    } else {
        if (cnt > 0) p[0] = (uint16_t)a;
        if (cnt > 1) p[1] = (uint16_t)(a >> 16);
        if (cnt > 2) p[2] = (uint16_t)b;
    }
}

// Geometry.  A wave owns 1024 consecutive elements (4 rows).  A "unit" is
// max(B, 1024) elements: the granule of the tile table and of scheduling.  For
// B <= 1024 a unit is one wave and holds 1024/B whole blocks; for B = 2048 (4096)
// the 2 (4) waves of a unit share one block and exchange their maxima through LDS.
constexpr int kWaveRows = 4;
constexpr int kWaveElems = kWaveRows * kRow;

template <int B>
struct Shape {
    static constexpr int UNIT = (B > kWaveElems) ? B : kWaveElems;
    static constexpr int WPB = UNIT / kWaveElems;                       // waves per unit: 1, 2, 4
    static constexpr int UPJ = kWavesPerWg / WPB;                       // units per job
    static constexpr int RPB = (B >= kWaveElems) ? kWaveRows : (B >= kRow ? B / kRow : 1);   // rows per block slot
    static constexpr int GROUP = (B >= kRow) ? 64 : B / 4;              // lanes per block in a row
    static constexpr int NBLK = kWaveRows / RPB;                        // block slots per lane
};

// Block maxima of NSTATE states x NBLK slots -> reciprocal data.
template <int B, int NSTATE>
__device__ __forceinline__ void norms_of(const uint32_t (&nbits)[NSTATE][Shape<B>::NBLK],
                                         BlockNorm (&out)[NSTATE][Shape<B>::NBLK], int lane)
{
    using S = Shape<B>;
    if (S::GROUP == 64) {
        uint32_t flat[NSTATE * S::NBLK];
        BlockNorm bn[NSTATE * S::NBLK];
#pragma unroll
        for (int st = 0; st < NSTATE; ++st)
#pragma unroll
            for (int k = 0; k < S::NBLK; ++k) flat[st * S::NBLK + k] = nbits[st][k];
        make_norms<NSTATE * S::NBLK>(flat, bn, lane);
#pragma unroll
        for (int st = 0; st < NSTATE; ++st)
#pragma unroll
            for (int k = 0; k < S::NBLK; ++k) out[st][k] = bn[st * S::NBLK + k];
    } else {
#pragma unroll
        for (int st = 0; st < NSTATE; ++st)
#pragma unroll
            for (int k = 0; k < S::NBLK; ++k) out[st][k] = make_norm(nbits[st][k]);
    }
}

// LDS words for the exchange of wave maxima: [parity][state][wave].
struct Exchange { uint32_t part[2][2][kWavesPerWg]; };

// Wave-wide maxima of K = 1, 2, 4 or 8 values per lane at once ("transpose and reduce"): a
// step over lane bit 32, 16 or 8 exchanges one value of each pair with the partner lane and
// keeps the maximum of the other, halving the number of values a lane carries; the last
// value goes through the remaining butterfly steps.  Returns, in every lane, ONE result:
// lane l holds the wave-wide maximum of value number l / (64 / K).
__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

template <int K>
__device__ __forceinline__ uint32_t wave_max_many(const uint32_t (&v)[K], int lane)
{
    static_assert(K == 1 || K == 2 || K == 4 || K == 8, "K");
    constexpr int K1 = (K >= 2) ? K / 2 : 1;      // values per lane after the step over lane bit 32
    constexpr int K2 = (K1 >= 2) ? K1 / 2 : 1;    // ... after lane bit 16
    uint32_t a[K1], b[K2];
    // lane bit 32: the lower half of the wave keeps v[i], the upper half v[i + K/2]
#pragma unroll
    for (int i = 0; i < K1; ++i) {
        const auto s = __builtin_amdgcn_permlane32_swap(v[i], v[(K >= 2) ? i + K1 : i], false, false);
        a[i] = umax(s[0], s[1]);
    }
    // lane bit 16
#pragma unroll
    for (int i = 0; i < K2; ++i) {
        const auto s = __builtin_amdgcn_permlane16_swap(a[i], a[(K1 >= 2) ? i + K2 : i], false, false);
        b[i] = umax(s[0], s[1]);
    }
    // lane bit 8: rotate each row of 16 lanes by 8
    uint32_t x;
    if constexpr (K2 >= 2) {
        const bool up = (lane & 8) != 0;
        const uint32_t keep = up ? b[1] : b[0], send = up ? b[0] : b[1];
        x = umax(keep, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0x128, 0xf, 0xf, true));
    } else {
        x = dpp_max_step<0x128>(b[0]);
    }
    x = dpp_max_step<0x141>(x);           // row_half_mirror: lanes l and 7 - l of each 8
    x = dpp_max_step<0x4E>(x);            // quad_perm [2,3,0,1]
    x = dpp_max_step<0xB1>(x);            // quad_perm [1,0,3,2]
    return x;
}

// Lane maxima -> wave-level block maxima.  Blocks that span the whole wave (B >= 256: GROUP
// == 64) reduce all their NSTATE x NBLK values at once and read each result back from the lane
// that holds it; smaller blocks reduce value by value inside their groups of lanes.
template <int B, int NSTATE>
__device__ __forceinline__ void reduce_in_wave(uint32_t (&v)[NSTATE][Shape<B>::NBLK], int lane)
{
    using S = Shape<B>;
    if (S::GROUP == 64) {
        constexpr int K = NSTATE * S::NBLK;
        uint32_t flat[K];
#pragma unroll
        for (int st = 0; st < NSTATE; ++st)
#pragma unroll
            for (int k = 0; k < S::NBLK; ++k) flat[st * S::NBLK + k] = v[st][k];
        const uint32_t x = wave_max_many<K>(flat, lane);
#pragma unroll
        for (int st = 0; st < NSTATE; ++st)
#pragma unroll
            for (int k = 0; k < S::NBLK; ++k)
                v[st][k] = (uint32_t)__builtin_amdgcn_readlane((int)x, (64 / K) * (st * S::NBLK + k));
    } else {
#pragma unroll
        for (int st = 0; st < NSTATE; ++st)
#pragma unroll
            for (int k = 0; k < S::NBLK; ++k) v[st][k] = group_max<S::GROUP>(v[st][k], lane);
    }
}

// When a block spans WPB > 1 waves, their maxima meet in LDS.  Every wave of the
// workgroup calls this exactly once per job, with or without a tile (`have`; the
// waves of one unit agree on it); it holds the one barrier between the two phases.
// `parity` alternates between jobs so that one barrier per job suffices: a slot is
// rewritten two jobs later, after barriers that every reader has passed.
template <int B, int NSTATE>
__device__ __forceinline__ void exchange_block_max(uint32_t (&v)[NSTATE][Shape<B>::NBLK], bool have, Exchange* ex,
                                                   int parity, int wave, int lane)
{
    using S = Shape<B>;
    if (S::WPB > 1 && have && lane == 0) {
#pragma unroll
        for (int st = 0; st < NSTATE; ++st) ex->part[parity][st][wave] = v[st][0];
    }
    // Blocks inside one wave (WPB == 1) have nothing to exchange, but the barrier stays: waves of
    // a workgroup that enter the store phase of their neighbouring tiles together measured
    // 2.5-3 % faster on 10^9 parameters (B <= 1024) than waves that drift apart.
    __syncthreads();
    if (S::WPB > 1) {
        if (have) {
            const int g0 = wave & ~(S::WPB - 1);
#pragma unroll
            for (int st = 0; st < NSTATE; ++st) {
                uint32_t m = 0;
#pragma unroll
                for (int k = 0; k < S::WPB; ++k) m = max(m, ex->part[parity][st][g0 + k]);
                v[st][0] = (uint32_t)__builtin_amdgcn_readfirstlane((int)m);
            }
        }
    }
}

// Quantize the 4 x 4 values of this lane (Eq. quant1, quant2) against the block
// maxima (with their reciprocal data, one entry per block slot) and store codes and maxima.
// `base` is the first element of this wave, `part` its index inside the unit.
template <int B, bool FULL, bool SECOND>
__device__ __forceinline__ void requantize_store(const unsigned char* lds, float (&val)[kWaveRows][4],
                                                 const BlockNorm (&norms)[Shape<B>::NBLK],
                                                 gbyte* codes, gfloat* Nout,
                                                 int64_t n, int64_t base, int part, int lane)
{
    using S = Shape<B>;
    if (B >= kRow) {
        // the maxima of the tile's block slots are neighbours in memory: lane s stores slot s
        float mine = norms[0].N;
#pragma unroll
        for (int s = 1; s < S::NBLK; ++s) mine = (lane == s) ? norms[s].N : mine;
        const int64_t row0 = base + (int64_t)lane * S::RPB * kRow;
        if (part == 0 && lane < S::NBLK && (FULL || row0 < n)) Nout[row0 / B] = mine;
    }
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) {
        const BlockNorm bn = norms[s];
        const int64_t row0 = base + (int64_t)s * S::RPB * kRow;
        if (B < kRow) {
            const int64_t e0 = row0 + lane * 4;
            if ((lane % S::GROUP) == 0 && (FULL || e0 < n)) Nout[e0 / B] = bn.N;
        }
        // one wave-uniform decision per block slot keeps the common path straight-line
        const bool all_fast = (S::GROUP == 64) ? bn.fast : (__builtin_amdgcn_ballot_w64(!bn.fast) == 0);
        if (all_fast) {
#pragma unroll
            for (int rr = 0; rr < S::RPB; ++rr) {
                const int r = s * S::RPB + rr;
                const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
                const int cnt = FULL ? 4 : lane_count(n, e0);
                uint32_t packed = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    packed |= nearest_code<SECOND>(lds, div_fast(val[r][j], bn.N, bn.y)) << (8 * j);
                if (FULL || cnt > 0) store4b(codes + e0, cnt, packed);
            }
        } else {
#pragma unroll
            for (int rr = 0; rr < S::RPB; ++rr) {
                const int r = s * S::RPB + rr;
                const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
                const int cnt = FULL ? 4 : lane_count(n, e0);
                uint32_t packed = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    packed |= nearest_code<SECOND>(lds, div_any(val[r][j], bn.N)) << (8 * j);
                if (FULL || cnt > 0) store4b(codes + e0, cnt, packed);
            }
        }
    }
}

// Old block maxima of the block slots of this wave tile.  For B >= 256 a slot's block
// index is the same in every lane: the value is loaded once and kept as a scalar.
// Below 256 each lane group reads its own block.
template <int B, bool FULL>
__device__ __forceinline__ void load_block_maxima(const float* N, int64_t n, int64_t base, int lane,
                                                  float (&out)[Shape<B>::NBLK])
{
    using S = Shape<B>;
    gcfloat* Ng = (gcfloat*)N;
    if (B >= kRow) {
        // one load for all slots: lane l reads the maximum of slot l % NBLK (neighbours in memory)
        const int64_t row0 = base + (int64_t)(lane % S::NBLK) * S::RPB * kRow;
        float v = 0.0f;
        if (FULL || row0 < n) v = Ng[row0 / B];
#pragma unroll
        for (int s = 0; s < S::NBLK; ++s) out[s] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), s));
    } else {
#pragma unroll
        for (int s = 0; s < S::NBLK; ++s) {
            const int64_t e0 = base + (int64_t)s * S::RPB * kRow + lane * 4;
            out[s] = (FULL || e0 < n) ? Ng[e0 / B] : 0.0f;
        }
    }
}

// ---------------------------------------------------------------------------
// Element arithmetic (one statement = one rounded binary32 operation).
// ---------------------------------------------------------------------------
// New states of Eq. adam.  g is updated in place when coupled decay applies.
template <int WD>
__device__ __forceinline__ void adam_states(const AdamScalars& s, float w, float g, float m_prev, float r_prev,
                                            float& m_out, float& r_out)
{
    if (WD == 1) {
        float t0 = s.wd * w;
        g = g + t0;
    }
    float t1 = s.beta1 * m_prev;
    float t2 = s.omb1 * g;
    m_out = t1 + t2;
    float t3 = s.beta2 * r_prev;
    float t4 = s.omb2 * g;
    float t5 = t4 * g;
    r_out = t3 + t5;
}

// Weight update of Eq. adam from the new 32-bit states.  BIAS: the bias-correction
// extension (the root is scaled by 1/sqrt(1 - beta2^t), one product, before eps is
// added; the step is alpha/(1 - beta1^t)); without it alpha_t == alpha.  FAST selects
// the short square root and division, valid when the caller has checked the range of
// m and r.
template <int WD, bool BIAS, bool FAST>
__device__ __forceinline__ float adam_weight(const AdamScalars& s, float w, float m, float r)
{
    const float root = FAST ? sqrt_rn_fast(r) : sqrtf(r);
    float d;
    if (BIAS) {
        const float rs = root * s.isbc2;
        d = rs + s.eps;
    } else {
        d = root + s.eps;
    }
    const float u = FAST ? div_rn_inrange(m, d) : m / d;
    const float t6 = s.alpha_t * u;
    if (WD == 2) {
        float t7 = s.alpha_wd * w;
        w = w - t7;
    }
    return w - t6;
}

template <int WD, bool BIAS>
__device__ __forceinline__ void adam_element(const AdamScalars& s, float& w, float g, float m_prev,
                                             float r_prev, float& m_out, float& r_out)
{
    float m, r;
    adam_states<WD>(s, w, g, m_prev, r_prev, m, r);
    w = adam_weight<WD, BIAS, false>(s, w, m, r);
    m_out = m;
    r_out = r;
}

template <bool WD>
__device__ __forceinline__ void sgd_element(const SgdScalars& s, float& w, float g, float m_prev, float& m_out)
{
    float wv = w;
    if (WD) {
        float t0 = s.wd * wv;
        g = g + t0;
    }
    float t1 = s.beta * m_prev;
    float m = t1 + g;
    float t2 = s.alpha * m;
    w = wv - t2;
    m_out = m;
}

// ---------------------------------------------------------------------------
// Wave tiles, in two phases around the exchange of block maxima.  `base` = first
// element of this wave inside the tensor.  What a tile carries from the first phase
// (update: load, dequantize, new states, new weights stored, lane maxima reduced
// inside the wave) to the second (re-quantization and stores of codes and maxima):
// the new states of its 4 x 4 elements per lane and the maxima of its block slots.
// ---------------------------------------------------------------------------
template <int B, int NSTATE>
struct Carry {
    float val[NSTATE][kWaveRows][4];
    uint32_t amax[NSTATE][Shape<B>::NBLK];
};

template <int B, typename WT, bool FULL, int WD, bool BIAS>
__device__ __forceinline__ void adam8_update(const TensorDesc& d, int64_t base, const unsigned char* lds,
                                             const AdamScalars& sc, int lane, Carry<B, 2>& c)
{
    using S = Shape<B>;
    const int64_t n = d.n;
    typename Wide<WT>::ptr w = (typename Wide<WT>::ptr)d.w;
    typename Wide<WT>::cptr g = (typename Wide<WT>::cptr)d.g;
    gcbyte* m_q = (gcbyte*)d.m_q;
    gcbyte* r_q = (gcbyte*)d.r_q;
    Raw4<WT> wraw[kWaveRows], graw[kWaveRows];
    uint32_t mq[kWaveRows], rq[kWaveRows];
    float Nm_old[S::NBLK], Nr_old[S::NBLK];
#pragma unroll
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        if (FULL || cnt > 0) {
            load4raw<WT>(w + e0, cnt, wraw[r]);
            load4raw<WT>(g + e0, cnt, graw[r]);
            mq[r] = load4b(m_q + e0, cnt);
            rq[r] = load4b(r_q + e0, cnt);
        } else {
            zero4raw(wraw[r]);
            zero4raw(graw[r]);
            mq[r] = 0; rq[r] = 0;
        }
    }
    load_block_maxima<B, FULL>(d.N_m, n, base, lane, Nm_old);
    load_block_maxima<B, FULL>(d.N_r, n, base, lane, Nr_old);
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) { c.amax[0][s] = 0; c.amax[1][s] = 0; }
    // new states of all rows; `lo` collects the smallest |m| and r of the tile
    float lo = kFastHi;
#pragma unroll
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        const int slot = r / S::RPB;
        float wv[4], gv[4];
        widen4(wraw[r], wv);
        widen4(graw[r], gv);
        float (&mnew)[4] = c.val[0][r];
        float (&rnew)[4] = c.val[1][r];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m_prev = dequant<false>(lds, (mq[r] >> (8 * j)) & 0xff, Nm_old[slot]);
            const float r_prev = dequant<true>(lds, (rq[r] >> (8 * j)) & 0xff, Nr_old[slot]);
            adam_states<WD>(sc, wv[j], gv[j], m_prev, r_prev, mnew[j], rnew[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (!FULL && j >= cnt) { mnew[j] = 0.0f; rnew[j] = 0.0f; }
        c.amax[0][slot] = absmax4(c.amax[0][slot], mnew);
        c.amax[1][slot] = absmax4(c.amax[1][slot], rnew);
        lo = __builtin_fminf(__builtin_fminf(lo, __builtin_fabsf(mnew[0])), __builtin_fabsf(mnew[1]));
        lo = __builtin_fminf(__builtin_fminf(lo, __builtin_fabsf(mnew[2])), __builtin_fabsf(mnew[3]));
        lo = __builtin_fminf(__builtin_fminf(lo, rnew[0]), rnew[1]);
        lo = __builtin_fminf(__builtin_fminf(lo, rnew[2]), rnew[3]);
    }
    // One wave-uniform test per tile: every |m| and r within [kFastLo, kFastHi] (the lane maxima
    // bound them from above).  A tile that holds an exact zero, e.g. a ragged one, or values
    // outside the range takes the general square root and division.
    float hi = 0.0f;
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s)
        hi = __builtin_fmaxf(__builtin_fmaxf(hi, __uint_as_float(c.amax[0][s])), __uint_as_float(c.amax[1][s]));
    const bool general = !(lo >= kFastLo) || !(hi <= kFastHi) || !sc.fast_ok;
    const bool fast = __builtin_amdgcn_ballot_w64(general) == 0;
#pragma unroll
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        float wv[4];
        widen4(wraw[r], wv);
        if (fast) {
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = adam_weight<WD, BIAS, true>(sc, wv[j], c.val[0][r][j], c.val[1][r][j]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = adam_weight<WD, BIAS, false>(sc, wv[j], c.val[0][r][j], c.val[1][r][j]);
        }
        if (FULL || cnt > 0) store4w<WT>(w + e0, cnt, wv);
    }
    reduce_in_wave<B, 2>(c.amax, lane);
}

template <int B, bool FULL>
__device__ __forceinline__ void adam8_requantize(const TensorDesc& d, int64_t base, int part, const unsigned char* lds,
                                                 int lane, Carry<B, 2>& c)
{
    using S = Shape<B>;
    BlockNorm bn[2][S::NBLK];
    norms_of<B, 2>(c.amax, bn, lane);
    requantize_store<B, FULL, false>(lds, c.val[0], bn[0], (gbyte*)d.m_q, (gfloat*)d.N_m, d.n, base, part, lane);
    requantize_store<B, FULL, true>(lds, c.val[1], bn[1], (gbyte*)d.r_q, (gfloat*)d.N_r, d.n, base, part, lane);
}

template <int B, typename WT, bool FULL, bool WD>
__device__ __forceinline__ void sgd8_update(const TensorDesc& d, int64_t base, const unsigned char* lds,
                                            const SgdScalars& sc, int lane, Carry<B, 1>& c)
{
    using S = Shape<B>;
    const int64_t n = d.n;
    typename Wide<WT>::ptr w = (typename Wide<WT>::ptr)d.w;
    typename Wide<WT>::cptr g = (typename Wide<WT>::cptr)d.g;
    gcbyte* m_q = (gcbyte*)d.m_q;
    float wv[kWaveRows][4], gv[kWaveRows][4];
    uint32_t mq[kWaveRows];
    float Nm_old[S::NBLK];
#pragma unroll
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        if (FULL || cnt > 0) {
            load4w<WT>(w + e0, cnt, wv[r]);
            load4w<WT>(g + e0, cnt, gv[r]);
            mq[r] = load4b(m_q + e0, cnt);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) { wv[r][j] = 0.0f; gv[r][j] = 0.0f; }
            mq[r] = 0;
        }
    }
    load_block_maxima<B, FULL>(d.N_m, n, base, lane, Nm_old);
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) c.amax[0][s] = 0;
#pragma unroll
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        const int slot = r / S::RPB;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m_prev = dequant<false>(lds, (mq[r] >> (8 * j)) & 0xff, Nm_old[slot]);
            float m_new;
            sgd_element<WD>(sc, wv[r][j], gv[r][j], m_prev, m_new);
            if (!FULL && j >= cnt) m_new = 0.0f;
            c.val[0][r][j] = m_new;
        }
        c.amax[0][slot] = absmax4(c.amax[0][slot], c.val[0][r]);
        if (FULL || cnt > 0) store4w<WT>(w + e0, cnt, wv[r]);
    }
    reduce_in_wave<B, 1>(c.amax, lane);
}

template <int B, bool FULL>
__device__ __forceinline__ void sgd8_requantize(const TensorDesc& d, int64_t base, int part, const unsigned char* lds,
                                                int lane, Carry<B, 1>& c)
{
    using S = Shape<B>;
    BlockNorm bn[1][S::NBLK];
    norms_of<B, 1>(c.amax, bn, lane);
    requantize_store<B, FULL, false>(lds, c.val[0], bn[0], (gbyte*)d.m_q, (gfloat*)d.N_m, d.n, base, part, lane);
}

// Tensors that keep 32-bit states: same formulas, no quantization; one wave
// handles its 1024 elements.
template <typename WT, bool ADAM>
__device__ __forceinline__ void f32_tile(const TensorDesc& d, int64_t base, const AdamScalars& as,
                                         const SgdScalars& ss, int lane)
{
    const int64_t n = d.n;
    typename Wide<WT>::ptr w = (typename Wide<WT>::ptr)d.w;
    typename Wide<WT>::cptr g = (typename Wide<WT>::cptr)d.g;
    gfloat* m = (gfloat*)d.m_f32;
    gfloat* rr = (gfloat*)d.r_f32;
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = lane_count(n, e0);
        if (cnt == 0) continue;
        float wv[4], gv[4], mv[4], rv[4] = {0.f, 0.f, 0.f, 0.f};
        load4w<WT>(w + e0, cnt, wv);
        load4w<WT>(g + e0, cnt, gv);
        load4f(m + e0, cnt, mv);
        if (ADAM) load4f(rr + e0, cnt, rv);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (ADAM) {
                if (as.bias) {
                    if (as.wd_mode == 1) adam_element<1, true>(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
                    else if (as.wd_mode == 2) adam_element<2, true>(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
                    else adam_element<0, true>(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
                } else {
                    if (as.wd_mode == 1) adam_element<1, false>(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
                    else if (as.wd_mode == 2) adam_element<2, false>(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
                    else adam_element<0, false>(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
                }
            } else {
                if (ss.wd != 0.0f) sgd_element<true>(ss, wv[j], gv[j], mv[j], mv[j]);
                else sgd_element<false>(ss, wv[j], gv[j], mv[j], mv[j]);
            }
        }
        store4w<WT>(w + e0, cnt, wv);
        store4f(m + e0, cnt, mv);
        if (ADAM) store4f(rr + e0, cnt, rv);
    }
}

template <int B, bool FULL>
__device__ __forceinline__ void quant_load(gcfloat* T, int64_t n, int64_t base, int lane, Carry<B, 1>& c)
{
    using S = Shape<B>;
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) c.amax[0][s] = 0;
#pragma unroll
    for (int r = 0; r < kWaveRows; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        if (FULL || cnt > 0) {
            load4f(T + e0, cnt, c.val[0][r]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) c.val[0][r][j] = 0.0f;
        }
        c.amax[0][r / S::RPB] = absmax4(c.amax[0][r / S::RPB], c.val[0][r]);
    }
    reduce_in_wave<B, 1>(c.amax, lane);
}

template <int B, bool FULL>
__device__ __forceinline__ void quant_store(gbyte* TQ, gfloat* N, int64_t n, int64_t base, int part,
                                            const unsigned char* lds, int lane, Carry<B, 1>& c)
{
    using S = Shape<B>;
    BlockNorm bn[1][S::NBLK];
    norms_of<B, 1>(c.amax, bn, lane);
    requantize_store<B, FULL, false>(lds, c.val[0], bn[0], TQ, N, n, base, part, lane);
}

// ---------------------------------------------------------------------------
// Scheduling.  A job is kWavesPerWg consecutive wave tiles, i.e. UPJ consecutive
// units; workgroups are persistent and take jobs until none is left.
//
// Dynamic (sched != nullptr): thread 0 of a workgroup draws job indices from
// `sched->next` and publishes them through LDS (two slots used alternately, so one
// barrier per draw suffices).  Every workgroup leaves the loop at its first
// out-of-range draw, without having another atomic in flight; the last one to
// leave (counted in `sched->done`) zeroes both counters, so the counter is ready for
// the next launch that is given it.  The host gives a counter only to launches that
// cannot overlap with another user of the same counter.
//
// Static (sched == nullptr): the host had no counter to give; draw number i of
// workgroup b is job (b + i * gridDim.x), published the same way.  Nothing is
// shared between launches then.
// ---------------------------------------------------------------------------

struct JobBox { long long job[2]; };

// One draw hands a workgroup SPAN consecutive jobs.  The first draw is issued at the
// very start of the kernel, before the tables are staged, so that its latency hides
// behind the staging.  With AHEAD the atomic of every following draw is issued as soon
// as the current one has been read, which hides its latency too but lets every
// workgroup hold a claim one draw ahead (a wider address window); the optimizer steps
// measured faster without it, the light stand-alone quantizer faster with it.
template <int SPAN>
__device__ __forceinline__ long long draw(Sched* sched, int round)
{
    // the first draw of every workgroup is its own index (no atomic: the whole grid starts at
    // once and would queue up on the one counter); the counter hands out what follows
    if (sched && round > 0)
        return (long long)gridDim.x * SPAN + (long long)atomicAdd(&sched->next, (unsigned long long)SPAN);
    return ((long long)blockIdx.x + (long long)round * gridDim.x) * SPAN;
}

template <int SPAN>
__device__ __forceinline__ void first_draw(Sched* sched, JobBox* box)
{
    if (threadIdx.x == 0) box->job[0] = draw<SPAN>(sched, 0);
}

// `round` = number of this draw (0 = the one first_draw has already issued); its LDS
// slot is round & 1.
template <int SPAN, bool AHEAD>
__device__ __forceinline__ int64_t next_draw(Sched* sched, JobBox* box, int round, int64_t njobs)
{
    const int parity = round & 1;
    if (!AHEAD && round > 0 && threadIdx.x == 0) box->job[parity] = draw<SPAN>(sched, round);
    __syncthreads();
    const long long j = box->job[parity];
    const int lo = __builtin_amdgcn_readfirstlane((int)j);
    const int hi = __builtin_amdgcn_readfirstlane((int)(j >> 32));
    const int64_t job = ((int64_t)hi << 32) | (uint32_t)lo;
    if (AHEAD && job < njobs && threadIdx.x == 0) box->job[parity ^ 1] = draw<SPAN>(sched, round + 1);
    return job;
}

// A launch with no more draws' worth of jobs than workgroups gives every workgroup
// exactly one draw: nobody needs to ask a second time.
template <int SPAN>
__device__ __forceinline__ bool single_draw(int64_t njobs)
{
    return njobs <= (int64_t)gridDim.x * SPAN;
}

__device__ __forceinline__ void leave(Sched* sched)
{
    if (sched && threadIdx.x == 0) {
        const unsigned long long before = atomicAdd(&sched->done, 1ULL);
        if (before == gridDim.x - 1) {
            atomicExch(&sched->next, 0ULL);
            atomicExch(&sched->done, 0ULL);
        }
    }
}


// Unit -> (tensor descriptor, unit index inside the tensor).  The tables are read
// through the constant address space with wave-uniform indices, i.e. by scalar
// loads into SGPRs (they are complete before the launch that reads them starts).
#define Q8_CONSTANT __attribute__((address_space(4)))
__device__ __forceinline__ TensorDesc resolve(const StepArgs& a, int64_t u, int64_t& unit_in_tensor)
{
    if (a.tiles) {
        Q8_CONSTANT const int32_t* ref = (Q8_CONSTANT const int32_t*)a.tiles + 2 * u;
        const int ti = ref[0];
        unit_in_tensor = ref[1];
        Q8_CONSTANT const uint64_t* f = (Q8_CONSTANT const uint64_t*)(a.descs + ti);
        TensorDesc d;
        d.w = (void*)f[0];
        d.g = (const void*)f[1];
        d.m_q = (uint8_t*)f[2];
        d.r_q = (uint8_t*)f[3];
        d.N_m = (float*)f[4];
        d.N_r = (float*)f[5];
        d.m_f32 = (float*)f[6];
        d.r_f32 = (float*)f[7];
        d.n = (int64_t)f[8];
        return d;
    }
    unit_in_tensor = u;
    return a.single;
}
static_assert(sizeof(TensorDesc) == 72 && sizeof(TileRef) == 8, "descriptor layout");

struct Lds {
    unsigned char tab[kLdsBytes];
    JobBox box;
    Exchange ex;
};

constexpr int kStepSpan = 1;        // jobs per draw of the optimizer-step kernels (binary32 storage; see Occupancy)
constexpr int kQuantSpan = 4;       // the stand-alone quantizer does far less work per job

// What a wave holds in one job: nothing, a tile of a tensor with 32-bit states (done in
// the first phase), or an 8-bit tile that ends inside the tensor (full) or at its end.
enum TileKind { kNoTile = 0, kFullTile = 1, kRaggedTile = 2 };

template <int B, typename WT, int WD, bool BIAS>
__device__ __forceinline__ void adam8_walk(const StepArgs& a, const AdamScalars& sc, Lds* lds)
{
    using S = Shape<B>;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int part = wave % S::WPB;
    const int64_t njobs = (a.nunits + S::UPJ - 1) / S::UPJ;
    SgdScalars none{};
    constexpr int SPAN = Occupancy<WT>::kSpan;
    const bool once = single_draw<SPAN>(njobs);
    int xpar = 0;
    for (int round = 0;; ++round) {
        if (once && round > 0) break;
        const int64_t j0 = next_draw<SPAN, false>(a.sched, &lds->box, round, njobs);
        if (j0 >= njobs) break;
        for (int k = 0; k < SPAN && j0 + k < njobs; ++k, xpar ^= 1) {
            const int64_t u = (j0 + k) * S::UPJ + wave / S::WPB;
            int kind = kNoTile;
            TensorDesc d{};
            int64_t base = 0;
            Carry<B, 2> c;
            if (u < a.nunits) {
                int64_t ut;
                d = resolve(a, u, ut);
                base = ut * S::UNIT + (int64_t)part * kWaveElems;
                if (d.m_f32) {
                    f32_tile<WT, true>(d, base, sc, none, lane);
                } else if (base + kWaveElems <= d.n) {
                    kind = kFullTile;
                    adam8_update<B, WT, true, WD, BIAS>(d, base, lds->tab, sc, lane, c);
                } else {
                    kind = kRaggedTile;
                    adam8_update<B, WT, false, WD, BIAS>(d, base, lds->tab, sc, lane, c);
                }
            }
            exchange_block_max<B, 2>(c.amax, kind != kNoTile, &lds->ex, xpar, wave, lane);
            if (kind == kFullTile) adam8_requantize<B, true>(d, base, part, lds->tab, lane, c);
            else if (kind == kRaggedTile) adam8_requantize<B, false>(d, base, part, lds->tab, lane, c);
        }
    }
}

template <int B, typename WT>
__global__ __launch_bounds__(kWgThreads, ((B < 256 && Occupancy<WT>::kWgPerCu == 2) ? 2 : 2 * Occupancy<WT>::kWgPerCu)) void adam8_kernel(StepArgs a, AdamScalars sc)
{
    __shared__ __attribute__((aligned(16))) Lds lds;
    first_draw<Occupancy<WT>::kSpan>(a.sched, &lds.box);
    stage_tables(lds.tab, a.qtab_s, a.qtab_u, threadIdx.x);
    __syncthreads();
    if (sc.bias) {
        if (sc.wd_mode == 0) adam8_walk<B, WT, 0, true>(a, sc, &lds);
        else if (sc.wd_mode == 1) adam8_walk<B, WT, 1, true>(a, sc, &lds);
        else adam8_walk<B, WT, 2, true>(a, sc, &lds);
    } else {
        if (sc.wd_mode == 0) adam8_walk<B, WT, 0, false>(a, sc, &lds);
        else if (sc.wd_mode == 1) adam8_walk<B, WT, 1, false>(a, sc, &lds);
        else adam8_walk<B, WT, 2, false>(a, sc, &lds);
    }
    leave(a.sched);
}

template <int B, typename WT, bool WD>
__device__ __forceinline__ void sgd8_walk(const StepArgs& a, const SgdScalars& sc, Lds* lds)
{
    using S = Shape<B>;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int part = wave % S::WPB;
    const int64_t njobs = (a.nunits + S::UPJ - 1) / S::UPJ;
    AdamScalars none{};
    constexpr int SPAN = Occupancy<WT>::kSpan;
    const bool once = single_draw<SPAN>(njobs);
    int xpar = 0;
    for (int round = 0;; ++round) {
        if (once && round > 0) break;
        const int64_t j0 = next_draw<SPAN, false>(a.sched, &lds->box, round, njobs);
        if (j0 >= njobs) break;
        for (int k = 0; k < SPAN && j0 + k < njobs; ++k, xpar ^= 1) {
            const int64_t u = (j0 + k) * S::UPJ + wave / S::WPB;
            int kind = kNoTile;
            TensorDesc d{};
            int64_t base = 0;
            Carry<B, 1> c;
            if (u < a.nunits) {
                int64_t ut;
                d = resolve(a, u, ut);
                base = ut * S::UNIT + (int64_t)part * kWaveElems;
                if (d.m_f32) {
                    f32_tile<WT, false>(d, base, none, sc, lane);
                } else if (base + kWaveElems <= d.n) {
                    kind = kFullTile;
                    sgd8_update<B, WT, true, WD>(d, base, lds->tab, sc, lane, c);
                } else {
                    kind = kRaggedTile;
                    sgd8_update<B, WT, false, WD>(d, base, lds->tab, sc, lane, c);
                }
            }
            exchange_block_max<B, 1>(c.amax, kind != kNoTile, &lds->ex, xpar, wave, lane);
            if (kind == kFullTile) sgd8_requantize<B, true>(d, base, part, lds->tab, lane, c);
            else if (kind == kRaggedTile) sgd8_requantize<B, false>(d, base, part, lds->tab, lane, c);
        }
    }
}

template <int B, typename WT>
__global__ __launch_bounds__(kWgThreads, ((B < 256 && Occupancy<WT>::kWgPerCu == 2) ? 2 : 2 * Occupancy<WT>::kWgPerCu)) void sgd8_kernel(StepArgs a, SgdScalars sc)
{
    __shared__ __attribute__((aligned(16))) Lds lds;
    first_draw<Occupancy<WT>::kSpan>(a.sched, &lds.box);
    stage_tables(lds.tab, a.qtab_s, nullptr, threadIdx.x);
    __syncthreads();
    if (sc.wd != 0.0f) sgd8_walk<B, WT, true>(a, sc, &lds);
    else sgd8_walk<B, WT, false>(a, sc, &lds);
    leave(a.sched);
}

template <int B>
__global__ __launch_bounds__(kWgThreads, ((B < 256) ? 2 : kMinWavesPerEu)) void quantize_kernel(const void* qtab, const float* T,
                                                                              uint8_t* TQ, float* N, int64_t n,
                                                                              int64_t nunits, Sched* sched)
{
    using S = Shape<B>;
    __shared__ __attribute__((aligned(16))) Lds lds;
    first_draw<kQuantSpan>(sched, &lds.box);
    stage_tables(lds.tab, qtab, nullptr, threadIdx.x);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int part = wave % S::WPB;
    const int64_t njobs = (nunits + S::UPJ - 1) / S::UPJ;
    int xpar = 0;
    for (int round = 0;; ++round) {
        const int64_t j0 = next_draw<kQuantSpan, true>(sched, &lds.box, round, njobs);
        if (j0 >= njobs) break;
        for (int k = 0; k < kQuantSpan && j0 + k < njobs; ++k, xpar ^= 1) {
            const int64_t u = (j0 + k) * S::UPJ + wave / S::WPB;
            const int64_t base = u * S::UNIT + (int64_t)part * kWaveElems;
            int kind = kNoTile;
            Carry<B, 1> c;
            if (u < nunits) {
                if (base + kWaveElems <= n) {
                    kind = kFullTile;
                    quant_load<B, true>((gcfloat*)T, n, base, lane, c);
                } else {
                    kind = kRaggedTile;
                    quant_load<B, false>((gcfloat*)T, n, base, lane, c);
                }
            }
            exchange_block_max<B, 1>(c.amax, kind != kNoTile, &lds.ex, xpar, wave, lane);
            if (kind == kFullTile) quant_store<B, true>((gbyte*)TQ, (gfloat*)N, n, base, part, lds.tab, lane, c);
            else if (kind == kRaggedTile) quant_store<B, false>((gbyte*)TQ, (gfloat*)N, n, base, part, lds.tab, lane, c);
        }
    }
    leave(sched);
}

// ---------------------------------------------------------------------------
// Launch helpers (host).
// ---------------------------------------------------------------------------

// Persistent grid: enough workgroups to fill every CU to the kernel's
// occupancy, never more than there are jobs.
// `per_cu` caches the occupancy query of one kernel (0 = not asked yet; the
// answer is the same on every device of one model, so one cache serves all).
// `*slot` != nullptr on entry: the caller brings its own counter; otherwise one is acquired
// for `stream` (possibly none: fixed order).
template <typename K>
q8_status grid_for(K kernel, std::atomic<int>& per_cu, int64_t njobs, hipStream_t stream, int& grid, Sched** slot,
                   int wg_per_cu_cap = 2)
{
    int cus = 0;
    q8_status st = device_cus(cus);
    if (st != Q8_OK) return st;
    int occ = per_cu.load(std::memory_order_relaxed);
    if (occ <= 0) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, kWgThreads, 0) != hipSuccess || occ <= 0)
            return Q8_ELAUNCH;
        per_cu.store(occ, std::memory_order_relaxed);
    }
    if (occ > wg_per_cu_cap) occ = wg_per_cu_cap;
    int64_t want = njobs;
    int64_t cap = (int64_t)cus * occ;
    grid = (int)(want < cap ? want : cap);
    if (grid < 1) grid = 1;
    return *slot ? Q8_OK : acquire_sched(stream, slot);
}

inline q8_status launch_status()
{
    return hipGetLastError() == hipSuccess ? Q8_OK : Q8_ELAUNCH;
}

#define Q8_DISPATCH_B(B, CALL)                 \
    switch (B) {                               \
    case 64: { constexpr int kB = 64; CALL; } break;     \
    case 128: { constexpr int kB = 128; CALL; } break;   \
    case 256: { constexpr int kB = 256; CALL; } break;   \
    case 512: { constexpr int kB = 512; CALL; } break;   \
    case 1024: { constexpr int kB = 1024; CALL; } break; \
    case 2048: { constexpr int kB = 2048; CALL; } break; \
    case 4096: { constexpr int kB = 4096; CALL; } break; \
    default: return Q8_EBLOCK;                 \
    }

template <int B, typename WT>
q8_status launch_adam(StepArgs a, const AdamScalars& sc, hipStream_t stream)
{
    static std::atomic<int> per_cu{0};
    int grid;
    q8_status st = grid_for(adam8_kernel<B, WT>, per_cu, (a.nunits + Shape<B>::UPJ - 1) / Shape<B>::UPJ, stream, grid, &a.sched,
                            Occupancy<WT>::kWgPerCu);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL((adam8_kernel<B, WT>), dim3(grid), dim3(kWgThreads), 0, stream, a, sc);
    return launch_status();
}

template <int B, typename WT>
q8_status launch_sgd(StepArgs a, const SgdScalars& sc, hipStream_t stream)
{
    static std::atomic<int> per_cu{0};
    int grid;
    q8_status st = grid_for(sgd8_kernel<B, WT>, per_cu, (a.nunits + Shape<B>::UPJ - 1) / Shape<B>::UPJ, stream, grid, &a.sched,
                            Occupancy<WT>::kWgPerCu);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL((sgd8_kernel<B, WT>), dim3(grid), dim3(kWgThreads), 0, stream, a, sc);
    return launch_status();
}

template <int B>
q8_status launch_quantize(const void* qtab, const float* T, uint8_t* TQ, float* N, int64_t n, hipStream_t stream)
{
    const int64_t nunits = (n + Shape<B>::UNIT - 1) / Shape<B>::UNIT;
    static std::atomic<int> per_cu{0};
    int grid;
    Sched* slot = nullptr;
    q8_status st = grid_for(quantize_kernel<B>, per_cu, (nunits + Shape<B>::UPJ - 1) / Shape<B>::UPJ, stream, grid, &slot);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL(quantize_kernel<B>, dim3(grid), dim3(kWgThreads), 0, stream, qtab, T, TQ, N, n, nunits, slot);
    return launch_status();
}

}  // namespace
}  // namespace q8

#endif  // Q8OPT_DEVICE_H

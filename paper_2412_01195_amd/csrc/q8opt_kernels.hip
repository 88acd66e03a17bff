// gfx950 kernels and device entry points of the fused 8-bit optimizer step
// (Sec. IV of the paper: Eq. sgd, Eq. adam, Eq. quant1-quant3).
//
// Work decomposition: one wave64 owns one "tile" of TILE = max(B, 2048)
// consecutive elements of one tensor, i.e. whole quantization blocks.  The tile is
// read as ROWS rows of 256 elements; lane l of the wave holds elements
// [256 r + 4 l, 256 r + 4 l + 4) of row r, so every fp32 access is one coalesced
// 128-bit load/store per lane and every code access one coalesced 32-bit one.
// New states stay in registers between the update and the re-quantization; the
// block absmax needs only cross-lane DPP steps inside the wave (no barrier, no
// LDS traffic).  Workgroups of 4 waves are persistent: they stage the two search
// tables into LDS once and then walk over tiles with a grid stride.
//
// Exact arithmetic: the update formulas are written one operation per statement
// and the file is compiled with -ffp-contract=off.  The normalisation x = m / N
// (Eq. quant1) is a correctly rounded quotient: N is uniform over a block, so
// y = RN(1/N) is formed once and each element takes a multiply and two
// residual-correction fma pairs (the classical Newton/Markstein division
// sequence); blocks whose N lies outside [2^-60, 2^60] use the plain divide.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "q8opt.h"
#include "q8opt_internal.h"

using namespace q8;

namespace {

constexpr int kWgThreads = 256;
constexpr int kWavesPerWg = 4;
constexpr int kRow = 256;                 // elements per wave row: 64 lanes x 4

struct TensorDesc {                       // device-side mirror of q8_tensor
    float* w;
    const float* g;
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
    int coupled_wd, decoupled_wd;
};
struct SgdScalars { float alpha, beta, wd; };

// ---------------------------------------------------------------------------
// LDS view of one staged search table.
// ---------------------------------------------------------------------------
struct QView {
    const float* qmap;
    const float* thr;
    const unsigned char* lut;
    uint32_t shift, width, kbase, L;
};

__device__ __forceinline__ void stage_qtable(unsigned char* lds, const void* qtab, int tid)
{
    const uint4* src = static_cast<const uint4*>(qtab);
    uint4* dst = reinterpret_cast<uint4*>(lds);
    for (int i = tid; i < kQTabBytes / 16; i += kWgThreads) dst[i] = src[i];
}

__device__ __forceinline__ QView make_view(const unsigned char* lds)
{
    const QTabHeader* h = reinterpret_cast<const QTabHeader*>(lds);
    QView v;
    v.qmap = reinterpret_cast<const float*>(lds + kOffQmap);
    v.thr = reinterpret_cast<const float*>(lds + kOffThr);
    v.lut = lds + kOffLut;
    v.shift = __builtin_amdgcn_readfirstlane(h->shift);
    v.width = __builtin_amdgcn_readfirstlane(h->width);
    v.kbase = __builtin_amdgcn_readfirstlane(h->kbase);
    v.L = __builtin_amdgcn_readfirstlane(h->L);
    return v;
}

// Nearest code of x (Eq. quant2) by bucket lookup + one exact threshold compare.
template <bool NONNEG>
__device__ __forceinline__ uint32_t nearest_code(const QView& q, float x)
{
    const uint32_t bits = __float_as_uint(x);
    const uint32_t a = __builtin_amdgcn_ubfe(bits, q.shift, q.width);
    int idx = (int)a - (int)q.kbase;
    idx = min(max(idx, 0), (int)q.L - 1);
    if (!NONNEG) idx += (bits >> 31) ? (int)q.L : 0;
    const uint32_t c = q.lut[idx];
    const float t = q.thr[c];
    return c + ((x >= t) ? 1u : 0u);
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

// Correctly rounded a / N for a block-uniform N.  `fast` says N is in
// [2^-60, 2^60] and y = RN(1/N); then for every |a| <= N either the quotient is
// computed exactly as RN(a/N) (|a| >= 2^-102, no underflow in the residuals), or
// |a / N| < 2^-40, far below the smallest threshold, where any tiny value gives
// the same code.
__device__ __forceinline__ float div_by_block_max(float a, float N, float y, bool fast)
{
    if (fast) {
        float q = a * y;
        float r = __builtin_fmaf(-q, N, a);
        q = __builtin_fmaf(r, y, q);
        r = __builtin_fmaf(-q, N, a);
        q = __builtin_fmaf(r, y, q);
        return q;
    }
    return (N == 0.0f) ? 0.0f : a / N;
}

struct BlockNorm { float N, y; bool fast; };

__device__ __forceinline__ BlockNorm make_norm(uint32_t nbits)
{
    BlockNorm b;
    b.N = __uint_as_float(nbits);
    b.fast = (nbits >= 0x21800000u) && (nbits <= 0x5d800000u);   // 2^-60 .. 2^60
    b.y = b.fast ? 1.0f / b.N : 0.0f;
    return b;
}

// ---------------------------------------------------------------------------
// Per-lane row access.  cnt = number of valid elements (0..4) of this lane in
// the row; FULL tiles have cnt == 4 everywhere.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int lane_count(int64_t n, int64_t e0)
{
    int64_t left = n - e0;
    return left >= 4 ? 4 : (left <= 0 ? 0 : (int)left);
}

__device__ __forceinline__ void load4f(const float* __restrict__ p, int cnt, float (&v)[4])
{
    if (cnt == 4) {
        float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (j < cnt) ? p[j] : 0.0f;
    }
}

__device__ __forceinline__ void store4f(float* __restrict__ p, int cnt, const float (&v)[4])
{
    if (cnt == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < cnt) p[j] = v[j];
    }
}

__device__ __forceinline__ uint32_t load4b(const uint8_t* __restrict__ p, int cnt)
{
    if (cnt == 4) return *reinterpret_cast<const uint32_t*>(p);
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (j < cnt) v |= (uint32_t)p[j] << (8 * j);
    return v;
}

__device__ __forceinline__ void store4b(uint8_t* __restrict__ p, int cnt, uint32_t v)
{
    if (cnt == 4) {
        *reinterpret_cast<uint32_t*>(p) = v;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < cnt) p[j] = (uint8_t)(v >> (8 * j));
    }
}

template <int B>
struct Shape {
    static constexpr int TILE = (B > 2048) ? B : 2048;
    static constexpr int ROWS = TILE / kRow;
    static constexpr int RPB = (B >= kRow) ? B / kRow : 1;      // rows per block
    static constexpr int BPR = (B >= kRow) ? 1 : kRow / B;      // blocks per row
    static constexpr int GROUP = (B >= kRow) ? 64 : B / 4;      // lanes per block in a row
    static constexpr int NBLK = ROWS / RPB;                     // block slots per lane
};

// Re-quantize the ROWS x 4 values of this lane (Eq. quant1, quant2) and store
// codes and block maxima.  `val` holds the new state, `amax` the per-slot lane
// maxima of |val| as bit patterns.
template <int B, bool FULL, bool NONNEG>
__device__ __forceinline__ void requantize_store(const QView& q, float (&val)[Shape<B>::ROWS][4],
                                                 uint32_t (&amax)[Shape<B>::NBLK],
                                                 uint8_t* __restrict__ codes, float* __restrict__ Nout,
                                                 int64_t n, int64_t base, int lane)
{
    using S = Shape<B>;
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) {
        const uint32_t nbits = group_max<S::GROUP>(amax[s], lane);
        const BlockNorm bn = make_norm(nbits);
        const int64_t row0 = base + (int64_t)s * S::RPB * kRow;
        // block index and writer lane
        if (B >= kRow) {
            if ((FULL || row0 < n) && lane == 0) Nout[row0 / B] = bn.N;
        } else {
            const int64_t e0 = row0 + lane * 4;
            if ((FULL || e0 < n) && (lane % S::GROUP) == 0) Nout[e0 / B] = bn.N;
        }
#pragma unroll
        for (int rr = 0; rr < S::RPB; ++rr) {
            const int r = s * S::RPB + rr;
            const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
            const int cnt = FULL ? 4 : lane_count(n, e0);
            if (!FULL && cnt == 0) continue;
            uint32_t packed = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x = div_by_block_max(val[r][j], bn.N, bn.y, bn.fast);
                packed |= nearest_code<NONNEG>(q, x) << (8 * j);
            }
            store4b(codes + e0, cnt, packed);
        }
    }
}

// Old block maximum for row r of the tile (uniform for B >= 256, per lane group below).
template <int B, bool FULL>
__device__ __forceinline__ float load_block_max(const float* __restrict__ N, int64_t n, int64_t base,
                                                int r, int lane)
{
    const int64_t row0 = base + (int64_t)r * kRow;
    if (B >= kRow) {
        if (!FULL && row0 >= n) return 0.0f;
        return N[row0 / B];
    }
    const int64_t e0 = row0 + lane * 4;
    if (!FULL && e0 >= n) return 0.0f;
    return N[e0 / B];
}

// ---------------------------------------------------------------------------
// Element arithmetic (one statement = one rounded binary32 operation).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void adam_element(const AdamScalars& s, float& w, float g, float m_prev,
                                             float r_prev, float& m_out, float& r_out)
{
    float wv = w;
    if (s.coupled_wd) {
        float t0 = s.wd * wv;
        g = g + t0;
    }
    float t1 = s.beta1 * m_prev;
    float t2 = s.omb1 * g;
    float m = t1 + t2;
    float t3 = s.beta2 * r_prev;
    float t4 = s.omb2 * g;
    float t5 = t4 * g;
    float r = t3 + t5;
    float root = sqrtf(r);
    float rs = root * s.isbc2;            // isbc2 == 1 unless bias correction: exact
    float d = rs + s.eps;
    float u = m / d;
    float t6 = s.alpha_t * u;
    if (s.decoupled_wd) {
        float t7 = s.alpha_wd * wv;
        wv = wv - t7;
    }
    w = wv - t6;
    m_out = m;
    r_out = r;
}

__device__ __forceinline__ void sgd_element(const SgdScalars& s, float& w, float g, float m_prev, float& m_out)
{
    float wv = w;
    if (s.wd != 0.0f) {
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
// Tiles.
// ---------------------------------------------------------------------------
template <int B, bool FULL>
__device__ __forceinline__ void adam8_tile(const TensorDesc& d, int64_t tile, const QView& qs, const QView& qu,
                                           const AdamScalars& sc, int lane)
{
    using S = Shape<B>;
    const int64_t base = tile * S::TILE;
    const int64_t n = d.n;
    float wv[S::ROWS][4], gv[S::ROWS][4];
    uint32_t mq[S::ROWS], rq[S::ROWS];
    float Nm_old[S::ROWS], Nr_old[S::ROWS];
#pragma unroll
    for (int r = 0; r < S::ROWS; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        if (FULL || cnt > 0) {
            load4f(d.w + e0, cnt, wv[r]);
            load4f(d.g + e0, cnt, gv[r]);
            mq[r] = load4b(d.m_q + e0, cnt);
            rq[r] = load4b(d.r_q + e0, cnt);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) { wv[r][j] = 0.0f; gv[r][j] = 0.0f; }
            mq[r] = 0; rq[r] = 0;
        }
        Nm_old[r] = load_block_max<B, FULL>(d.N_m, n, base, r, lane);
        Nr_old[r] = load_block_max<B, FULL>(d.N_r, n, base, r, lane);
    }
    uint32_t amax_m[S::NBLK], amax_r[S::NBLK];
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) { amax_m[s] = 0; amax_r[s] = 0; }
    // after this loop gv holds the new m and wv is reused for the new r
#pragma unroll
    for (int r = 0; r < S::ROWS; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        float rnew[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m_prev = qs.qmap[(mq[r] >> (8 * j)) & 0xff] * Nm_old[r];
            const float r_prev = qu.qmap[(rq[r] >> (8 * j)) & 0xff] * Nr_old[r];
            float m_new, r_new;
            adam_element(sc, wv[r][j], gv[r][j], m_prev, r_prev, m_new, r_new);
            if (!FULL && j >= cnt) { m_new = 0.0f; r_new = 0.0f; }
            gv[r][j] = m_new;
            rnew[j] = r_new;
            amax_m[r / S::RPB] = max(amax_m[r / S::RPB], __float_as_uint(m_new) & 0x7fffffffu);
            amax_r[r / S::RPB] = max(amax_r[r / S::RPB], __float_as_uint(r_new));
        }
        if (FULL || cnt > 0) store4f(d.w + e0, cnt, wv[r]);
#pragma unroll
        for (int j = 0; j < 4; ++j) wv[r][j] = rnew[j];
    }
    requantize_store<B, FULL, false>(qs, gv, amax_m, d.m_q, d.N_m, n, base, lane);
    requantize_store<B, FULL, true>(qu, wv, amax_r, d.r_q, d.N_r, n, base, lane);
}

template <int B, bool FULL>
__device__ __forceinline__ void sgd8_tile(const TensorDesc& d, int64_t tile, const QView& qs,
                                          const SgdScalars& sc, int lane)
{
    using S = Shape<B>;
    const int64_t base = tile * S::TILE;
    const int64_t n = d.n;
    float wv[S::ROWS][4], gv[S::ROWS][4];
    uint32_t mq[S::ROWS];
    float Nm_old[S::ROWS];
#pragma unroll
    for (int r = 0; r < S::ROWS; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        if (FULL || cnt > 0) {
            load4f(d.w + e0, cnt, wv[r]);
            load4f(d.g + e0, cnt, gv[r]);
            mq[r] = load4b(d.m_q + e0, cnt);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) { wv[r][j] = 0.0f; gv[r][j] = 0.0f; }
            mq[r] = 0;
        }
        Nm_old[r] = load_block_max<B, FULL>(d.N_m, n, base, r, lane);
    }
    uint32_t amax_m[S::NBLK];
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) amax_m[s] = 0;
#pragma unroll
    for (int r = 0; r < S::ROWS; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float m_prev = qs.qmap[(mq[r] >> (8 * j)) & 0xff] * Nm_old[r];
            float m_new;
            sgd_element(sc, wv[r][j], gv[r][j], m_prev, m_new);
            if (!FULL && j >= cnt) m_new = 0.0f;
            gv[r][j] = m_new;
            amax_m[r / S::RPB] = max(amax_m[r / S::RPB], __float_as_uint(m_new) & 0x7fffffffu);
        }
        if (FULL || cnt > 0) store4f(d.w + e0, cnt, wv[r]);
    }
    requantize_store<B, FULL, false>(qs, gv, amax_m, d.m_q, d.N_m, n, base, lane);
}

// Tensors that keep 32-bit states: same formulas, no quantization.  Processed
// in the same 2048-element wave tiles.
template <bool ADAM>
__device__ __forceinline__ void f32_tile(const TensorDesc& d, int64_t tile, int tile_elems,
                                         const AdamScalars& as, const SgdScalars& ss, int lane)
{
    const int64_t base = tile * tile_elems;
    const int64_t n = d.n;
    for (int r = 0; r < tile_elems / kRow; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = lane_count(n, e0);
        if (cnt == 0) continue;
        float wv[4], gv[4], mv[4], rv[4] = {0.f, 0.f, 0.f, 0.f};
        load4f(d.w + e0, cnt, wv);
        load4f(d.g + e0, cnt, gv);
        load4f(d.m_f32 + e0, cnt, mv);
        if (ADAM) load4f(d.r_f32 + e0, cnt, rv);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (ADAM) adam_element(as, wv[j], gv[j], mv[j], rv[j], mv[j], rv[j]);
            else sgd_element(ss, wv[j], gv[j], mv[j], mv[j]);
        }
        store4f(d.w + e0, cnt, wv);
        store4f(d.m_f32 + e0, cnt, mv);
        if (ADAM) store4f(d.r_f32 + e0, cnt, rv);
    }
}

template <int B, bool FULL>
__device__ __forceinline__ void quant_tile(const float* __restrict__ T, uint8_t* __restrict__ TQ,
                                           float* __restrict__ N, int64_t n, int64_t tile, const QView& q, int lane)
{
    using S = Shape<B>;
    const int64_t base = tile * S::TILE;
    float v[S::ROWS][4];
    uint32_t amax[S::NBLK];
#pragma unroll
    for (int s = 0; s < S::NBLK; ++s) amax[s] = 0;
#pragma unroll
    for (int r = 0; r < S::ROWS; ++r) {
        const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
        const int cnt = FULL ? 4 : lane_count(n, e0);
        if (FULL || cnt > 0) {
            load4f(T + e0, cnt, v[r]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[r][j] = 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            amax[r / S::RPB] = max(amax[r / S::RPB], __float_as_uint(v[r][j]) & 0x7fffffffu);
    }
    requantize_store<B, FULL, false>(q, v, amax, TQ, N, n, base, lane);
}

// ---------------------------------------------------------------------------
// Persistent tile walk.  Workgroup ids are dealt round-robin to the 8 XCDs, so
// ids are re-numbered to give every XCD one contiguous run of tiles per pass.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int64_t first_tile(int& stride)
{
    const int G = gridDim.x;
    int vb = blockIdx.x;
    if ((G & 7) == 0) vb = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
    stride = G * kWavesPerWg;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    return (int64_t)vb * kWavesPerWg + wave;
}

struct StepArgs {
    const TensorDesc* descs;      // device list, or nullptr: use `single`
    const TileRef* tiles;         // device tile table for lists, else nullptr
    TensorDesc single;
    int64_t ntiles;
    const void* qtab_s;
    const void* qtab_u;
};

__device__ __forceinline__ TensorDesc resolve(const StepArgs& a, int64_t t, int64_t& tile_in_tensor)
{
    if (a.tiles) {
        const TileRef ref = a.tiles[t];
        const int ti = __builtin_amdgcn_readfirstlane(ref.tensor);
        tile_in_tensor = __builtin_amdgcn_readfirstlane(ref.tile);
        return a.descs[ti];
    }
    tile_in_tensor = t;
    return a.single;
}

template <int B>
__global__ __launch_bounds__(kWgThreads) void adam8_kernel(StepArgs a, AdamScalars sc)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kQTabBytes];
    stage_qtable(lds, a.qtab_s, threadIdx.x);
    stage_qtable(lds + kQTabBytes, a.qtab_u, threadIdx.x);
    __syncthreads();
    const QView qs = make_view(lds), qu = make_view(lds + kQTabBytes);
    const int lane = threadIdx.x & 63;
    int stride;
    SgdScalars none{};
    for (int64_t t = first_tile(stride); t < a.ntiles; t += stride) {
        int64_t tt;
        const TensorDesc d = resolve(a, t, tt);
        if (d.m_f32) {
            f32_tile<true>(d, tt, Shape<B>::TILE, sc, none, lane);
        } else if ((tt + 1) * Shape<B>::TILE <= d.n) {
            adam8_tile<B, true>(d, tt, qs, qu, sc, lane);
        } else {
            adam8_tile<B, false>(d, tt, qs, qu, sc, lane);
        }
    }
}

template <int B>
__global__ __launch_bounds__(kWgThreads) void sgd8_kernel(StepArgs a, SgdScalars sc)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kQTabBytes];
    stage_qtable(lds, a.qtab_s, threadIdx.x);
    __syncthreads();
    const QView qs = make_view(lds);
    const int lane = threadIdx.x & 63;
    int stride;
    AdamScalars none{};
    for (int64_t t = first_tile(stride); t < a.ntiles; t += stride) {
        int64_t tt;
        const TensorDesc d = resolve(a, t, tt);
        if (d.m_f32) {
            f32_tile<false>(d, tt, Shape<B>::TILE, none, sc, lane);
        } else if ((tt + 1) * Shape<B>::TILE <= d.n) {
            sgd8_tile<B, true>(d, tt, qs, sc, lane);
        } else {
            sgd8_tile<B, false>(d, tt, qs, sc, lane);
        }
    }
}

template <int B>
__global__ __launch_bounds__(kWgThreads) void quantize_kernel(const void* qtab, const float* __restrict__ T,
                                                              uint8_t* __restrict__ TQ, float* __restrict__ N,
                                                              int64_t n, int64_t ntiles)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kQTabBytes];
    stage_qtable(lds, qtab, threadIdx.x);
    __syncthreads();
    const QView q = make_view(lds);
    const int lane = threadIdx.x & 63;
    int stride;
    for (int64_t t = first_tile(stride); t < ntiles; t += stride) {
        if ((t + 1) * Shape<B>::TILE <= n) quant_tile<B, true>(T, TQ, N, n, t, q, lane);
        else quant_tile<B, false>(T, TQ, N, n, t, q, lane);
    }
}

// Eq. quant3.  One thread handles 4 consecutive elements per step; the block
// index of an element is (index >> log2 B).
__global__ __launch_bounds__(kWgThreads) void dequantize_kernel(const void* qtab, const uint8_t* __restrict__ TQ,
                                                                const float* __restrict__ N, int64_t n, int log2B,
                                                                float* __restrict__ TD)
{
    __shared__ float qmap[256];
    qmap[threadIdx.x] = reinterpret_cast<const float*>(static_cast<const unsigned char*>(qtab) + kOffQmap)[threadIdx.x];
    __syncthreads();
    const int64_t nvec = (n + 3) >> 2;
    const int64_t stride = (int64_t)gridDim.x * kWgThreads;
    for (int64_t v = (int64_t)blockIdx.x * kWgThreads + threadIdx.x; v < nvec; v += stride) {
        const int64_t e0 = v * 4;
        const int cnt = lane_count(n, e0);
        const uint32_t c = load4b(TQ + e0, cnt);
        const float Nb = N[e0 >> log2B];          // B >= 64 is a multiple of 4: one block per vector
        float out[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = qmap[(c >> (8 * j)) & 0xff] * Nb;
        store4f(TD + e0, cnt, out);
    }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
bool valid_block(int B) { return B >= 64 && B <= 4096 && (B & (B - 1)) == 0; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }
int tile_elems(int B) { return B > 2048 ? B : 2048; }

struct DeviceInfo { int cus; };

q8_status device_info(DeviceInfo& out)
{
    static int cached_dev = -1;
    static DeviceInfo cached{};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return Q8_ELAUNCH;
    if (dev != cached_dev) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return Q8_ELAUNCH;
        cached.cus = cus;
        cached_dev = dev;
    }
    out = cached;
    return Q8_OK;
}

// Persistent grid: enough workgroups to fill every CU to the kernel's
// occupancy, never more than there are 4-tile groups of work.
// `per_cu` caches the occupancy query of one kernel (0 = not asked yet).
template <typename K>
q8_status grid_for(K kernel, int& per_cu, int64_t ntiles, int& grid)
{
    DeviceInfo di;
    q8_status st = device_info(di);
    if (st != Q8_OK) return st;
    if (per_cu <= 0) {
        int v = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, kernel, kWgThreads, 0) != hipSuccess || v <= 0)
            return Q8_ELAUNCH;
        per_cu = v;
    }
    int64_t want = (ntiles + kWavesPerWg - 1) / kWavesPerWg;
    int64_t cap = (int64_t)di.cus * per_cu;
    grid = (int)(want < cap ? want : cap);
    if (grid < 1) grid = 1;
    return Q8_OK;
}

q8_status launch_status()
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

q8_status make_adam_scalars(float alpha, float beta1, float beta2, float eps, float wd, int64_t t, int flags,
                            AdamScalars& s)
{
    if (flags & ~(Q8_FLAG_BIAS_CORRECTION | Q8_FLAG_DECOUPLED_WD)) return Q8_EINVAL;
    s.beta1 = beta1; s.beta2 = beta2; s.eps = eps; s.wd = wd;
    s.omb1 = 1.0f - beta1;
    s.omb2 = 1.0f - beta2;
    s.alpha_t = alpha;
    s.isbc2 = 1.0f;
    if (flags & Q8_FLAG_BIAS_CORRECTION) {
        if (t < 1) return Q8_EINVAL;
        // beta^t in binary64 by left-to-right square-and-multiply
        auto ipow = [](double base, int64_t e) {
            double r = 1.0;
            int top = 62;
            while (top > 0 && !((e >> top) & 1)) --top;
            for (int b = top; b >= 0; --b) {
                r = r * r;
                if ((e >> b) & 1) r = r * base;
            }
            return r;
        };
        const double bc1 = 1.0 - ipow((double)beta1, t);
        const double bc2 = 1.0 - ipow((double)beta2, t);
        s.alpha_t = (float)((double)alpha / bc1);
        s.isbc2 = (float)(1.0 / sqrt(bc2));
    }
    s.alpha_wd = alpha * wd;
    s.coupled_wd = (wd != 0.0f) && !(flags & Q8_FLAG_DECOUPLED_WD);
    s.decoupled_wd = (wd != 0.0f) && (flags & Q8_FLAG_DECOUPLED_WD);
    return Q8_OK;
}

template <int B>
q8_status launch_adam(const StepArgs& a, const AdamScalars& sc, hipStream_t stream)
{
    static int per_cu = 0;
    int grid;
    q8_status st = grid_for(adam8_kernel<B>, per_cu, a.ntiles, grid);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL(adam8_kernel<B>, dim3(grid), dim3(kWgThreads), 0, stream, a, sc);
    return launch_status();
}

template <int B>
q8_status launch_sgd(const StepArgs& a, const SgdScalars& sc, hipStream_t stream)
{
    static int per_cu = 0;
    int grid;
    q8_status st = grid_for(sgd8_kernel<B>, per_cu, a.ntiles, grid);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL(sgd8_kernel<B>, dim3(grid), dim3(kWgThreads), 0, stream, a, sc);
    return launch_status();
}

template <int B>
q8_status launch_quantize(const void* qtab, const float* T, uint8_t* TQ, float* N, int64_t n, hipStream_t stream)
{
    const int64_t ntiles = (n + Shape<B>::TILE - 1) / Shape<B>::TILE;
    static int per_cu = 0;
    int grid;
    q8_status st = grid_for(quantize_kernel<B>, per_cu, ntiles, grid);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL(quantize_kernel<B>, dim3(grid), dim3(kWgThreads), 0, stream, qtab, T, TQ, N, n, ntiles);
    return launch_status();
}

}  // namespace

struct q8_plan {
    TensorDesc* d_descs;
    TileRef* d_tiles;
    int64_t ntiles;
    int count;
    int B;
    bool has_r;        // every tensor carries second-state storage (usable with Adam)
};

extern "C" q8_status q8_quantize_blockwise(const void* qtable, const float* T, int64_t n, int B,
                                           uint8_t* TQ, float* N, void* stream)
{
    if (n < 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    if (n == 0) return Q8_OK;
    if (!qtable || !T || !TQ || !N) return Q8_EINVAL;
    if (!aligned(qtable, 16) || !aligned(T, 16) || !aligned(TQ, 4) || !aligned(N, 4)) return Q8_EALIGN;
    Q8_DISPATCH_B(B, return launch_quantize<kB>(qtable, T, TQ, N, n, static_cast<hipStream_t>(stream)));
    return Q8_OK;
}

extern "C" q8_status q8_dequantize_blockwise(const void* qtable, const uint8_t* TQ, const float* N,
                                             int64_t n, int B, float* TD, void* stream)
{
    if (n < 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    if (n == 0) return Q8_OK;
    if (!qtable || !TQ || !N || !TD) return Q8_EINVAL;
    if (!aligned(qtable, 16) || !aligned(TD, 16) || !aligned(TQ, 4) || !aligned(N, 4)) return Q8_EALIGN;
    DeviceInfo di;
    q8_status st = device_info(di);
    if (st != Q8_OK) return st;
    const int64_t nvec = (n + 3) / 4;
    int64_t want = (nvec + kWgThreads - 1) / kWgThreads;
    int64_t cap = (int64_t)di.cus * 8;
    const int grid = (int)(want < cap ? want : cap);
    hipLaunchKernelGGL(dequantize_kernel, dim3(grid), dim3(kWgThreads), 0, static_cast<hipStream_t>(stream),
                       qtable, TQ, N, n, ilog2(B), TD);
    return launch_status();
}

extern "C" q8_status q8_adam8bit_step(float* w, const float* g, uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
                                      const void* qtable_signed, const void* qtable_unsigned, int64_t n, int B,
                                      float alpha, float beta1, float beta2, float eps, float weight_decay,
                                      int64_t t, int flags, void* stream)
{
    if (n < 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    AdamScalars sc;
    q8_status st = make_adam_scalars(alpha, beta1, beta2, eps, weight_decay, t, flags, sc);
    if (st != Q8_OK) return st;
    if (n == 0) return Q8_OK;
    if (!w || !g || !m_q || !r_q || !N_m || !N_r || !qtable_signed || !qtable_unsigned) return Q8_EINVAL;
    if (!aligned(w, 16) || !aligned(g, 16) || !aligned(m_q, 4) || !aligned(r_q, 4) || !aligned(N_m, 4) ||
        !aligned(N_r, 4) || !aligned(qtable_signed, 16) || !aligned(qtable_unsigned, 16))
        return Q8_EALIGN;
    StepArgs a{};
    a.single = TensorDesc{w, g, m_q, r_q, N_m, N_r, nullptr, nullptr, n};
    a.ntiles = (n + tile_elems(B) - 1) / tile_elems(B);
    a.qtab_s = qtable_signed;
    a.qtab_u = qtable_unsigned;
    Q8_DISPATCH_B(B, return launch_adam<kB>(a, sc, static_cast<hipStream_t>(stream)));
    return Q8_OK;
}

extern "C" q8_status q8_sgd8bit_step(float* w, const float* g, uint8_t* m_q, float* N_m, const void* qtable_signed,
                                     int64_t n, int B, float alpha, float beta, float weight_decay, void* stream)
{
    if (n < 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    if (n == 0) return Q8_OK;
    if (!w || !g || !m_q || !N_m || !qtable_signed) return Q8_EINVAL;
    if (!aligned(w, 16) || !aligned(g, 16) || !aligned(m_q, 4) || !aligned(N_m, 4) || !aligned(qtable_signed, 16))
        return Q8_EALIGN;
    StepArgs a{};
    a.single = TensorDesc{w, g, m_q, nullptr, N_m, nullptr, nullptr, nullptr, n};
    a.ntiles = (n + tile_elems(B) - 1) / tile_elems(B);
    a.qtab_s = qtable_signed;
    SgdScalars sc{alpha, beta, weight_decay};
    Q8_DISPATCH_B(B, return launch_sgd<kB>(a, sc, static_cast<hipStream_t>(stream)));
    return Q8_OK;
}

extern "C" q8_status q8_plan_create(const q8_tensor* list, int count, int B, q8_plan** out)
{
    if (!out) return Q8_EINVAL;
    *out = nullptr;
    if (!list || count <= 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    const int64_t te = tile_elems(B);
    int64_t ntiles = 0;
    bool has_r = true;
    for (int i = 0; i < count; ++i) {
        const q8_tensor& t = list[i];
        if (t.n < 0 || !t.w || !t.g) return Q8_EINVAL;
        if (!aligned(t.w, 16) || !aligned(t.g, 16)) return Q8_EALIGN;
        if (t.m_f32) {
            if (!aligned(t.m_f32, 16) || !aligned(t.r_f32, 16)) return Q8_EALIGN;
            if (!t.r_f32) has_r = false;
        } else {
            if (!t.m_q || !t.N_m) return Q8_EINVAL;
            if (!aligned(t.m_q, 4) || !aligned(t.N_m, 4) || !aligned(t.r_q, 4) || !aligned(t.N_r, 4)) return Q8_EALIGN;
            if (!t.r_q || !t.N_r) has_r = false;
        }
        const int64_t nt = (t.n + te - 1) / te;
        if (nt > INT32_MAX) return Q8_EINVAL;
        ntiles += nt;
    }
    TensorDesc* h_descs = new (std::nothrow) TensorDesc[count];
    TileRef* h_tiles = new (std::nothrow) TileRef[ntiles > 0 ? ntiles : 1];
    q8_plan* p = new (std::nothrow) q8_plan{};
    if (!h_descs || !h_tiles || !p) { delete[] h_descs; delete[] h_tiles; delete p; return Q8_ENOMEM; }
    int64_t k = 0;
    for (int i = 0; i < count; ++i) {
        const q8_tensor& t = list[i];
        h_descs[i] = TensorDesc{t.w, t.g, t.m_q, t.r_q, t.N_m, t.N_r, t.m_f32, t.r_f32, t.n};
        const int64_t nt = (t.n + te - 1) / te;
        for (int64_t j = 0; j < nt; ++j) h_tiles[k++] = TileRef{i, (int32_t)j};
    }
    q8_status st = Q8_OK;
    if (hipMalloc(&p->d_descs, sizeof(TensorDesc) * count) != hipSuccess) st = Q8_ENOMEM;
    if (st == Q8_OK && hipMalloc(&p->d_tiles, sizeof(TileRef) * (ntiles > 0 ? ntiles : 1)) != hipSuccess) st = Q8_ENOMEM;
    if (st == Q8_OK && hipMemcpy(p->d_descs, h_descs, sizeof(TensorDesc) * count, hipMemcpyHostToDevice) != hipSuccess)
        st = Q8_ELAUNCH;
    if (st == Q8_OK && ntiles > 0 &&
        hipMemcpy(p->d_tiles, h_tiles, sizeof(TileRef) * ntiles, hipMemcpyHostToDevice) != hipSuccess)
        st = Q8_ELAUNCH;
    delete[] h_descs;
    delete[] h_tiles;
    if (st != Q8_OK) {
        (void)hipGetLastError();
        if (p->d_descs) (void)hipFree(p->d_descs);
        if (p->d_tiles) (void)hipFree(p->d_tiles);
        delete p;
        return st;
    }
    p->ntiles = ntiles;
    p->count = count;
    p->B = B;
    p->has_r = has_r;
    *out = p;
    return Q8_OK;
}

extern "C" q8_status q8_plan_destroy(q8_plan* plan)
{
    if (!plan) return Q8_EINVAL;
    q8_status st = Q8_OK;
    if (hipFree(plan->d_descs) != hipSuccess) st = Q8_ELAUNCH;
    if (hipFree(plan->d_tiles) != hipSuccess) st = Q8_ELAUNCH;
    delete plan;
    return st;
}

extern "C" q8_status q8_multi_adam8bit_step(q8_plan* plan, const void* qtable_signed, const void* qtable_unsigned,
                                            float alpha, float beta1, float beta2, float eps, float weight_decay,
                                            int64_t t, int flags, void* stream)
{
    if (!plan || !qtable_signed || !qtable_unsigned || !plan->has_r) return Q8_EINVAL;
    if (!aligned(qtable_signed, 16) || !aligned(qtable_unsigned, 16)) return Q8_EALIGN;
    AdamScalars sc;
    q8_status st = make_adam_scalars(alpha, beta1, beta2, eps, weight_decay, t, flags, sc);
    if (st != Q8_OK) return st;
    if (plan->ntiles == 0) return Q8_OK;
    StepArgs a{};
    a.descs = plan->d_descs;
    a.tiles = plan->d_tiles;
    a.ntiles = plan->ntiles;
    a.qtab_s = qtable_signed;
    a.qtab_u = qtable_unsigned;
    Q8_DISPATCH_B(plan->B, return launch_adam<kB>(a, sc, static_cast<hipStream_t>(stream)));
    return Q8_OK;
}

extern "C" q8_status q8_multi_sgd8bit_step(q8_plan* plan, const void* qtable_signed, float alpha, float beta,
                                           float weight_decay, void* stream)
{
    if (!plan || !qtable_signed) return Q8_EINVAL;
    if (!aligned(qtable_signed, 16)) return Q8_EALIGN;
    if (plan->ntiles == 0) return Q8_OK;
    StepArgs a{};
    a.descs = plan->d_descs;
    a.tiles = plan->d_tiles;
    a.ntiles = plan->ntiles;
    a.qtab_s = qtable_signed;
    SgdScalars sc{alpha, beta, weight_decay};
    Q8_DISPATCH_B(plan->B, return launch_sgd<kB>(a, sc, static_cast<hipStream_t>(stream)));
    return Q8_OK;
}

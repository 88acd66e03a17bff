// Host side of the library: C-ABI entry points, argument checks, the job-counter ring, and
// the kernels that do not depend on the storage type of w and g (stand-alone quantize and
// dequantize).  The optimizer-step kernels are instantiated in q8opt_steps.hip, once per
// storage type.
#include "q8opt_device.h"

#include <math.h>

#include <mutex>
#include <new>

using namespace q8;

namespace q8 {

// step kernels by storage type (q8opt_steps.hip)
q8_status run_adam_f32(int B, StepArgs a, const AdamScalars& sc, hipStream_t stream);
q8_status run_sgd_f32(int B, StepArgs a, const SgdScalars& sc, hipStream_t stream);
q8_status run_adam_bf16(int B, StepArgs a, const AdamScalars& sc, hipStream_t stream);
q8_status run_sgd_bf16(int B, StepArgs a, const SgdScalars& sc, hipStream_t stream);
q8_status run_adam_f16(int B, StepArgs a, const AdamScalars& sc, hipStream_t stream);
q8_status run_sgd_f16(int B, StepArgs a, const SgdScalars& sc, hipStream_t stream);

// Job counters of the dynamic scheduler (device memory that belongs to the library: module
// data, nothing is allocated).  A kernel leaves its counter zeroed.  Two kernels must never
// use one counter at the same time, so a counter is tied to what orders its users:
//   - eager launches: one counter per stream (launches on one stream run in order); the
//     per-thread default stream counts as one stream per host thread.  When more streams
//     have been seen than there are counters, the device is synchronized once (nothing is
//     in flight then) and the table starts again;
//   - launches recorded by stream capture: one counter per (capture, stream) pair, reserved
//     for good, because the recorded graph can be replayed later on any stream; launches
//     recorded from one stream in one capture run in order in every replay.
// When no counter can be given (the reserved ones are used up, or the device cannot be
// synchronized because some stream is being captured), the launch gets none and its
// kernel walks the jobs in a fixed order instead: slower on large tensors, never wrong.
constexpr int kEagerSlots = 192;
constexpr int kGraphSlots = 64;
__device__ Sched g_sched[kEagerSlots + kGraphSlots];

struct SlotKey { hipStream_t stream; unsigned long long id; };

// One record per device, filled on the first call with that device current
// (every GPU holds its own copy of g_sched at its own address).  Host threads
// may call the library concurrently.
struct DeviceRec {
    int cus;                         // 0: not asked yet
    Sched* sched;
    int eager_used, graph_used;
    SlotKey eager[kEagerSlots];
    SlotKey graph[kGraphSlots];
};
constexpr int kMaxDevices = 64;
std::mutex g_dev_mutex;
DeviceRec g_dev[kMaxDevices];

// caller holds g_dev_mutex
q8_status device_rec(DeviceRec** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return Q8_ELAUNCH;
    DeviceRec& r = g_dev[dev];
    if (r.cus == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return Q8_ELAUNCH;
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_sched)) != hipSuccess || !p) return Q8_ELAUNCH;
        r.sched = static_cast<Sched*>(p);
        r.cus = cus;
    }
    *out = &r;
    return Q8_OK;
}

q8_status device_cus(int& cus)
{
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    DeviceRec* r = nullptr;
    q8_status st = device_rec(&r);
    if (st == Q8_OK) cus = r->cus;
    return st;
}

// small unique number of the calling host thread (keys the per-thread default stream)
unsigned long long thread_tag()
{
    static std::atomic<unsigned long long> next{1};
    thread_local unsigned long long mine = next.fetch_add(1);
    return mine;
}

int find_key(const SlotKey* keys, int used, const SlotKey& k)
{
    for (int i = 0; i < used; ++i)
        if (keys[i].stream == k.stream && keys[i].id == k.id) return i;
    return -1;
}

q8_status acquire_sched(hipStream_t stream, Sched** out)
{
    *out = nullptr;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    unsigned long long cap_id = 0;
    if (hipStreamGetCaptureInfo(stream, &cap, &cap_id) != hipSuccess) {
        (void)hipGetLastError();
        return Q8_ELAUNCH;
    }
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    DeviceRec* r = nullptr;
    q8_status st = device_rec(&r);
    if (st != Q8_OK) return st;
    if (cap != hipStreamCaptureStatusNone) {
        if (cap != hipStreamCaptureStatusActive) return Q8_ELAUNCH;          // an invalidated capture
        const SlotKey k{stream, cap_id};
        int i = find_key(r->graph, r->graph_used, k);
        if (i < 0 && r->graph_used < kGraphSlots) {
            i = r->graph_used++;
            r->graph[i] = k;
        }
        if (i >= 0) *out = r->sched + kEagerSlots + i;
        return Q8_OK;                                                        // else: fixed order
    }
    const SlotKey k{stream, stream == hipStreamPerThread ? thread_tag() : 0ULL};
    int i = find_key(r->eager, r->eager_used, k);
    if (i < 0) {
        if (r->eager_used == kEagerSlots) {
            if (hipDeviceSynchronize() != hipSuccess) {
                (void)hipGetLastError();
                return Q8_OK;                                                // fixed order
            }
            r->eager_used = 0;
        }
        i = r->eager_used++;
        r->eager[i] = k;
    }
    *out = r->sched + i;
    return Q8_OK;
}

}  // namespace q8

namespace {

// Eq. quant3.  A workgroup of 512 threads handles 4096 consecutive elements in two steps of
// 2048, one 4-element vector per thread and step (a 32-bit code access and a 128-bit access of
// the result, both non-temporal); the block index of an element is (index >> log2 B).  Launched
// flat (one workgroup per chunk), so the hardware dispatcher hands the chunks out in address
// order; a persistent variant that draws jobs from the job counter measured slower (this
// kernel does so little per byte that the counter's ~80 M draws/s become the limit, and
// drawing several jobs at once widens the window of addresses in flight).  The code and
// block-maximum loads are issued before the codebook is staged, so the staging latency hides
// behind them.  Measured on 10^9 codes: 2 steps 0.79 ms, 1 step 1.01 ms, 3 steps 0.94 ms,
// 4 steps 0.93 ms; 128, 256 and 512 threads within 2 % of each other.
constexpr int kDequantSteps = 2;
constexpr int kDequantThreads = 512;
constexpr int kDequantChunk = 4 * kDequantThreads * kDequantSteps;

template <bool FULL>
__device__ __forceinline__ void dequantize_chunk(const void* qtab, gcbyte* TQ, gcfloat* N, int64_t n, int log2B,
                                                 gfloat* TD, int64_t chunk0, float* qmap)
{
    uint32_t c[kDequantSteps];
    float Nb[kDequantSteps];
    int cnt[kDequantSteps];
#pragma unroll
    for (int i = 0; i < kDequantSteps; ++i) {
        const int64_t e0 = chunk0 + i * (4 * kDequantThreads) + threadIdx.x * 4;
        cnt[i] = FULL ? 4 : lane_count(n, e0);
        c[i] = cnt[i] > 0 ? load4b(TQ + e0, cnt[i]) : 0u;
        Nb[i] = cnt[i] > 0 ? N[e0 >> log2B] : 0.0f;       // B >= 64 is a multiple of 4: one block per vector
    }
    if (threadIdx.x < 256)
        qmap[threadIdx.x] = ((gcfloat*)(static_cast<const unsigned char*>(qtab) + kOffQmap))[threadIdx.x];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kDequantSteps; ++i) {
        const int64_t e0 = chunk0 + i * (4 * kDequantThreads) + threadIdx.x * 4;
        float out[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = qmap[(c[i] >> (8 * j)) & 0xff] * Nb[i];
        if (FULL || cnt[i] > 0) store4f(TD + e0, cnt[i], out);
    }
}

__global__ __launch_bounds__(kDequantThreads) void dequantize_kernel(const void* qtab, const uint8_t* TQ, const float* N,
                                                         int64_t n, int log2B, float* TD)
{
    __shared__ float qmap[256];
    const int64_t chunk0 = (int64_t)blockIdx.x * kDequantChunk;
    if (chunk0 + kDequantChunk <= n)
        dequantize_chunk<true>(qtab, (gcbyte*)TQ, (gcfloat*)N, n, log2B, (gfloat*)TD, chunk0, qmap);
    else
        dequantize_chunk<false>(qtab, (gcbyte*)TQ, (gcfloat*)N, n, log2B, (gfloat*)TD, chunk0, qmap);
}

q8_status launch_dequantize(const void* qtab, const uint8_t* TQ, const float* N, int64_t n, int B, float* TD,
                            hipStream_t stream)
{
    const int64_t grid = (n + kDequantChunk - 1) / kDequantChunk;
    if (grid > INT32_MAX) return Q8_EINVAL;
    int log2B = 0;
    while ((1 << log2B) < B) ++log2B;
    hipLaunchKernelGGL(dequantize_kernel, dim3((unsigned)grid), dim3(kDequantThreads), 0, stream, qtab, TQ, N, n, log2B, TD);
    return launch_status();
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------
enum Store { kStoreF32 = 0, kStoreBf16 = 1, kStoreF16 = 2 };      // element type of w and g

// w/g alignment: one lane vector = 4 elements of the storage type.
size_t wg_align(Store store) { return store == kStoreF32 ? 16 : 8; }

q8_status run_adam(Store store, int B, const StepArgs& a, const AdamScalars& sc, hipStream_t stream)
{
    switch (store) {
    case kStoreBf16: return run_adam_bf16(B, a, sc, stream);
    case kStoreF16: return run_adam_f16(B, a, sc, stream);
    default: return run_adam_f32(B, a, sc, stream);
    }
}

q8_status run_sgd(Store store, int B, const StepArgs& a, const SgdScalars& sc, hipStream_t stream)
{
    switch (store) {
    case kStoreBf16: return run_sgd_bf16(B, a, sc, stream);
    case kStoreF16: return run_sgd_f16(B, a, sc, stream);
    default: return run_sgd_f32(B, a, sc, stream);
    }
}

bool valid_block(int B) { return B >= 64 && B <= 4096 && (B & (B - 1)) == 0; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
int unit_elems(int B) { return B > 1024 ? B : 1024; }                 // Shape<B>::UNIT

q8_status make_adam_scalars(float alpha, float beta1, float beta2, float eps, float wd, int64_t t, int flags,
                            AdamScalars& s)
{
    if (flags & ~(Q8_FLAG_BIAS_CORRECTION | Q8_FLAG_DECOUPLED_WD)) return Q8_EINVAL;
    s.beta1 = beta1; s.beta2 = beta2; s.eps = eps; s.wd = wd;
    s.omb1 = 1.0f - beta1;
    s.omb2 = 1.0f - beta2;
    s.alpha_t = alpha;
    s.isbc2 = 1.0f;
    s.bias = (flags & Q8_FLAG_BIAS_CORRECTION) ? 1 : 0;
    if (s.bias) {
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
    s.fast_ok = (eps >= 0.0f && eps <= 1024.0f && s.isbc2 >= 1.0f && s.isbc2 <= 1024.0f) ? 1 : 0;
    s.alpha_wd = alpha * wd;
    s.wd_mode = (wd == 0.0f) ? 0 : ((flags & Q8_FLAG_DECOUPLED_WD) ? 2 : 1);
    return Q8_OK;
}

}  // namespace


struct q8_plan {
    TensorDesc* d_descs;
    TileRef* d_tiles;
    int64_t ntiles;
    int count;
    int B;
    bool has_r;        // every tensor carries second-state storage (usable with Adam)
    Store store;       // element type of every w and g
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
    return launch_dequantize(qtable, TQ, N, n, B, TD, static_cast<hipStream_t>(stream));
}

namespace {

q8_status adam_step(Store store, void* w, const void* g, uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
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
    if (!aligned(w, wg_align(store)) || !aligned(g, wg_align(store)) || !aligned(m_q, 4) || !aligned(r_q, 4) ||
        !aligned(N_m, 4) || !aligned(N_r, 4) || !aligned(qtable_signed, 16) || !aligned(qtable_unsigned, 16))
        return Q8_EALIGN;
    StepArgs a{};
    a.single = TensorDesc{w, g, m_q, r_q, N_m, N_r, nullptr, nullptr, n};
    a.nunits = (n + unit_elems(B) - 1) / unit_elems(B);
    a.qtab_s = qtable_signed;
    a.qtab_u = qtable_unsigned;
    return run_adam(store, B, a, sc, static_cast<hipStream_t>(stream));
}

q8_status sgd_step(Store store, void* w, const void* g, uint8_t* m_q, float* N_m, const void* qtable_signed,
                   int64_t n, int B, float alpha, float beta, float weight_decay, void* stream)
{
    if (n < 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    if (n == 0) return Q8_OK;
    if (!w || !g || !m_q || !N_m || !qtable_signed) return Q8_EINVAL;
    if (!aligned(w, wg_align(store)) || !aligned(g, wg_align(store)) || !aligned(m_q, 4) || !aligned(N_m, 4) ||
        !aligned(qtable_signed, 16))
        return Q8_EALIGN;
    StepArgs a{};
    a.single = TensorDesc{w, g, m_q, nullptr, N_m, nullptr, nullptr, nullptr, n};
    a.nunits = (n + unit_elems(B) - 1) / unit_elems(B);
    a.qtab_s = qtable_signed;
    const SgdScalars sc{alpha, beta, weight_decay};
    return run_sgd(store, B, a, sc, static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" q8_status q8_adam8bit_step(float* w, const float* g, uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
        const void* qtable_signed, const void* qtable_unsigned, int64_t n, int B,
        float alpha, float beta1, float beta2, float eps, float weight_decay, int64_t t, int flags, void* stream)
{
    return adam_step(kStoreF32, w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, n, B, alpha, beta1, beta2, eps,
                     weight_decay, t, flags, stream);
}

extern "C" q8_status q8_sgd8bit_step(float* w, const float* g, uint8_t* m_q, float* N_m, const void* qtable_signed,
        int64_t n, int B, float alpha, float beta, float weight_decay, void* stream)
{
    return sgd_step(kStoreF32, w, g, m_q, N_m, qtable_signed, n, B, alpha, beta, weight_decay, stream);
}

extern "C" q8_status q8_adam8bit_step_bf16(uint16_t* w, const uint16_t* g, uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
        const void* qtable_signed, const void* qtable_unsigned, int64_t n, int B,
        float alpha, float beta1, float beta2, float eps, float weight_decay, int64_t t, int flags, void* stream)
{
    return adam_step(kStoreBf16, w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, n, B, alpha, beta1, beta2, eps,
                     weight_decay, t, flags, stream);
}

extern "C" q8_status q8_sgd8bit_step_bf16(uint16_t* w, const uint16_t* g, uint8_t* m_q, float* N_m, const void* qtable_signed,
        int64_t n, int B, float alpha, float beta, float weight_decay, void* stream)
{
    return sgd_step(kStoreBf16, w, g, m_q, N_m, qtable_signed, n, B, alpha, beta, weight_decay, stream);
}

extern "C" q8_status q8_adam8bit_step_f16(uint16_t* w, const uint16_t* g, uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
        const void* qtable_signed, const void* qtable_unsigned, int64_t n, int B,
        float alpha, float beta1, float beta2, float eps, float weight_decay, int64_t t, int flags, void* stream)
{
    return adam_step(kStoreF16, w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, n, B, alpha, beta1, beta2, eps,
                     weight_decay, t, flags, stream);
}

extern "C" q8_status q8_sgd8bit_step_f16(uint16_t* w, const uint16_t* g, uint8_t* m_q, float* N_m, const void* qtable_signed,
        int64_t n, int B, float alpha, float beta, float weight_decay, void* stream)
{
    return sgd_step(kStoreF16, w, g, m_q, N_m, qtable_signed, n, B, alpha, beta, weight_decay, stream);
}

namespace {

// Argument rules of one list entry; nt = its number of units of `te` elements.
q8_status check_tensor(const q8_tensor& t, size_t wg_al, int64_t te, int64_t& nt, bool& has_r)
{
    nt = 0;
    if (t.n < 0) return Q8_EINVAL;
    if (t.n == 0) return Q8_OK;                       // an empty tensor contributes no unit; its pointers are not looked at
    if (!t.w || !t.g) return Q8_EINVAL;
    if (!aligned(t.w, wg_al) || !aligned(t.g, wg_al)) return Q8_EALIGN;
    if (t.m_f32) {
        if (!aligned(t.m_f32, 16) || !aligned(t.r_f32, 16)) return Q8_EALIGN;
        if (!t.r_f32) has_r = false;
    } else {
        if (!t.m_q || !t.N_m) return Q8_EINVAL;
        if (!aligned(t.m_q, 4) || !aligned(t.N_m, 4) || !aligned(t.r_q, 4) || !aligned(t.N_r, 4)) return Q8_EALIGN;
        if (!t.r_q || !t.N_r) has_r = false;
    }
    nt = (t.n + te - 1) / te;
    if (nt > INT32_MAX) return Q8_EINVAL;
    return Q8_OK;
}

q8_status plan_create(const q8_tensor* list, int count, int B, Store store, q8_plan** out)
{
    if (!out) return Q8_EINVAL;
    *out = nullptr;
    if (!list || count <= 0) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    const int64_t te = unit_elems(B);
    const size_t wg_al = wg_align(store);
    int64_t ntiles = 0;
    bool has_r = true;
    for (int i = 0; i < count; ++i) {
        int64_t nt = 0;
        q8_status st = check_tensor(list[i], wg_al, te, nt, has_r);
        if (st != Q8_OK) return st;
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
    p->store = store;
    *out = p;
    return Q8_OK;
}

}  // namespace

extern "C" q8_status q8_plan_create(const q8_tensor* list, int count, int B, q8_plan** out)
{
    return plan_create(list, count, B, kStoreF32, out);
}

extern "C" q8_status q8_plan_create_bf16(const q8_tensor* list, int count, int B, q8_plan** out)
{
    return plan_create(list, count, B, kStoreBf16, out);
}

extern "C" q8_status q8_plan_create_f16(const q8_tensor* list, int count, int B, q8_plan** out)
{
    return plan_create(list, count, B, kStoreF16, out);
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
    a.nunits = plan->ntiles;
    a.qtab_s = qtable_signed;
    a.qtab_u = qtable_unsigned;
    return run_adam(plan->store, plan->B, a, sc, static_cast<hipStream_t>(stream));
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
    a.nunits = plan->ntiles;
    a.qtab_s = qtable_signed;
    const SgdScalars sc{alpha, beta, weight_decay};
    return run_sgd(plan->store, plan->B, a, sc, static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------
// Multi-tensor Adam step for callers that cannot allocate: the tables a q8_plan keeps in
// allocated device memory (tensor descriptors, unit table) and the job counter live in one
// static device array instead.  The host list travels to the device inside kernel arguments,
// a chunk of descriptors per launch of a small fill kernel, so the call enqueues kernels
// only: no allocation, no memset, no copy.
// ---------------------------------------------------------------------------
namespace {

constexpr int kNoallocMaxTensors = 1024;
constexpr int kNoallocMaxUnits = 1 << 17;
constexpr size_t kScratchDescs = 256;                                                   // after the job counter
constexpr size_t kScratchTiles = kScratchDescs + sizeof(TensorDesc) * kNoallocMaxTensors;
constexpr size_t kScratchBytes = kScratchTiles + sizeof(TileRef) * kNoallocMaxUnits;   // 1 122 560 bytes
static_assert(kScratchTiles % 8 == 0 && sizeof(Sched) <= kScratchDescs, "scratch layout");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// device address of `scratch` per device (each GPU holds its own copy of the array)
unsigned char* g_scratch_ptr[kMaxDevices];

q8_status scratch_address(unsigned char** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return Q8_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (!g_scratch_ptr[dev]) {
        unsigned char* ptr = nullptr;
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return Q8_ELAUNCH;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return Q8_OK;
}

// One launch carries up to kFillChunk descriptors in its arguments (under the 4 KB limit).
constexpr int kFillChunk = 40;
struct FillArgs {
    TensorDesc desc[kFillChunk];
    int32_t first_unit[kFillChunk];     // position of the tensor's first unit in the unit table
    int32_t units[kFillChunk];
    int32_t first_tensor, count;
    int32_t clear_counter;              // the first chunk also zeroes the job counter
};
static_assert(sizeof(FillArgs) + 8 <= 3584, "kernel arguments stay well under 4 KB");

// Workgroup b writes descriptor (first_tensor + b) and that tensor's rows of the unit table.
__global__ __launch_bounds__(256) void fill_tables_kernel(FillArgs a, unsigned char* base)
{
    const int b = blockIdx.x;
    if (b >= a.count) return;
    TensorDesc* descs = reinterpret_cast<TensorDesc*>(base + kScratchDescs);
    TileRef* tiles = reinterpret_cast<TileRef*>(base + kScratchTiles);
    if (threadIdx.x == 0) {
        descs[a.first_tensor + b] = a.desc[b];
        if (a.clear_counter && b == 0) {
            Sched* s = reinterpret_cast<Sched*>(base);
            s->next = 0;
            s->done = 0;
        }
    }
    for (int j = threadIdx.x; j < a.units[b]; j += blockDim.x)
        tiles[a.first_unit[b] + j] = TileRef{a.first_tensor + b, j};
}

}  // namespace

extern "C" q8_status q8_multi_adam8bit_step_noalloc(const q8_tensor* list, int count, int B,
                                                    const void* qtable_signed, const void* qtable_unsigned,
                                                    float alpha, float beta1, float beta2, float eps,
                                                    float weight_decay, int64_t t, int flags, void* stream)
{
    if (!list || count <= 0 || !qtable_signed || !qtable_unsigned) return Q8_EINVAL;
    if (!valid_block(B)) return Q8_EBLOCK;
    if (!aligned(qtable_signed, 16) || !aligned(qtable_unsigned, 16)) return Q8_EALIGN;
    AdamScalars sc;
    q8_status st = make_adam_scalars(alpha, beta1, beta2, eps, weight_decay, t, flags, sc);
    if (st != Q8_OK) return st;
    if (count > kNoallocMaxTensors) return Q8_ELIMIT;
    const int64_t te = unit_elems(B);
    int64_t nunits = 0;
    bool has_r = true;
    for (int i = 0; i < count; ++i) {
        int64_t nt = 0;
        st = check_tensor(list[i], wg_align(kStoreF32), te, nt, has_r);
        if (st != Q8_OK) return st;
        nunits += nt;
        if (nunits > kNoallocMaxUnits) return Q8_ELIMIT;
    }
    if (!has_r) return Q8_EINVAL;
    if (nunits == 0) return Q8_OK;
    unsigned char* ptr = nullptr;
    st = scratch_address(&ptr);
    if (st != Q8_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t unit0 = 0;
    for (int first = 0; first < count; first += kFillChunk) {
        FillArgs fa{};
        fa.first_tensor = first;
        fa.count = (count - first < kFillChunk) ? count - first : kFillChunk;
        fa.clear_counter = (first == 0) ? 1 : 0;
        for (int k = 0; k < fa.count; ++k) {
            const q8_tensor& x = list[first + k];
            fa.desc[k] = TensorDesc{x.w, x.g, x.m_q, x.r_q, x.N_m, x.N_r, x.m_f32, x.r_f32, x.n};
            fa.first_unit[k] = (int32_t)unit0;
            fa.units[k] = (int32_t)((x.n + te - 1) / te);
            unit0 += fa.units[k];
        }
        hipLaunchKernelGGL(fill_tables_kernel, dim3(fa.count), dim3(256), 0, s, fa, ptr);
        if (launch_status() != Q8_OK) return Q8_ELAUNCH;
    }
    StepArgs a{};
    a.descs = reinterpret_cast<const TensorDesc*>(ptr + kScratchDescs);
    a.tiles = reinterpret_cast<const TileRef*>(ptr + kScratchTiles);
    a.nunits = nunits;
    a.qtab_s = qtable_signed;
    a.qtab_u = qtable_unsigned;
    a.sched = reinterpret_cast<Sched*>(ptr);
    return run_adam(kStoreF32, B, a, sc, s);
}

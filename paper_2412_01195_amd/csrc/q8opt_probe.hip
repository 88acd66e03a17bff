// Measurement aid, NOT part of the product library: built into libq8opt_probe.so only, which
// bench.py loads for its workload "probe1b".  The kernel moves exactly the bytes of one Adam
// (8-bit) step at B = 2048 -- same wave tiles, same scheduler, same LDS footprint and
// occupancy, same barriers per job -- with the arithmetic left out: w and both code arrays
// are written back unchanged, g is only read.  Its rate is what this access pattern can
// reach on the chip, the yardstick the step kernel is compared with.
#include "q8opt_device.h"

using namespace q8;

namespace {

__global__ __launch_bounds__(kWgThreads, kMinWavesPerEu) void traffic_probe_kernel(StepArgs a)
{
    using S = Shape<2048>;
    __shared__ __attribute__((aligned(16))) Lds lds;
    first_draw<kStepSpan>(a.sched, &lds.box);
    stage_tables(lds.tab, a.qtab_s, a.qtab_u, threadIdx.x);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int part = wave % S::WPB;
    const int64_t njobs = (a.nunits + S::UPJ - 1) / S::UPJ;
    const int64_t n = a.single.n;
    gfloat* w = (gfloat*)a.single.w;
    gcfloat* g = (gcfloat*)a.single.g;
    gbyte* m_q = (gbyte*)a.single.m_q;
    gbyte* r_q = (gbyte*)a.single.r_q;
    const bool once = single_draw<kStepSpan>(njobs);
    for (int round = 0;; ++round) {
        if (once && round > 0) break;
        const int64_t j0 = next_draw<kStepSpan, false>(a.sched, &lds.box, round, njobs);
        if (j0 >= njobs) break;
        const int64_t u = j0 * S::UPJ + wave / S::WPB;
        const int64_t base = u * S::UNIT + (int64_t)part * kWaveElems;
        float wv[kWaveRows][4], gv[kWaveRows][4];
        uint32_t mq[kWaveRows], rq[kWaveRows];
        int cnt[kWaveRows];
#pragma unroll
        for (int r = 0; r < kWaveRows; ++r) {
            const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
            cnt[r] = (u < a.nunits) ? lane_count(n, e0) : 0;
            if (cnt[r] > 0) {
                load4f(w + e0, cnt[r], wv[r]);
                load4f(g + e0, cnt[r], gv[r]);
                mq[r] = load4b(m_q + e0, cnt[r]);
                rq[r] = load4b(r_q + e0, cnt[r]);
#pragma unroll
                for (int j = 0; j < 4; ++j) asm volatile("" ::"v"(gv[r][j]));      // keep the loads of g
            }
        }
#pragma unroll
        for (int r = 0; r < kWaveRows; ++r) {
            const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
            if (cnt[r] > 0) store4f(w + e0, cnt[r], wv[r]);
        }
        __syncthreads();                               // stands for the exchange of block maxima
#pragma unroll
        for (int r = 0; r < kWaveRows; ++r) {
            const int64_t e0 = base + (int64_t)r * kRow + lane * 4;
            if (cnt[r] > 0) {
                store4b(m_q + e0, cnt[r], mq[r]);
                store4b(r_q + e0, cnt[r], rq[r]);
            }
        }
    }
    leave(a.sched);
}

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

// Device pointers; asynchronous on `stream`; w, m_q, r_q keep their contents.
extern "C" Q8_API q8_status q8_probe_adam8bit_traffic(float* w, const float* g, uint8_t* m_q, uint8_t* r_q,
                                                      const void* qtable_signed, const void* qtable_unsigned,
                                                      int64_t n, void* stream)
{
    if (n < 0) return Q8_EINVAL;
    if (n == 0) return Q8_OK;
    if (!w || !g || !m_q || !r_q || !qtable_signed || !qtable_unsigned) return Q8_EINVAL;
    if (!aligned_to(w, 16) || !aligned_to(g, 16) || !aligned_to(m_q, 4) || !aligned_to(r_q, 4) ||
        !aligned_to(qtable_signed, 16) || !aligned_to(qtable_unsigned, 16))
        return Q8_EALIGN;
    StepArgs a{};
    a.single = TensorDesc{w, g, m_q, r_q, nullptr, nullptr, nullptr, nullptr, n};
    a.nunits = (n + 2047) / 2048;
    a.qtab_s = qtable_signed;
    a.qtab_u = qtable_unsigned;
    static std::atomic<int> per_cu{0};
    int grid;
    hipStream_t s = static_cast<hipStream_t>(stream);
    q8_status st = grid_for(traffic_probe_kernel, per_cu, (a.nunits + Shape<2048>::UPJ - 1) / Shape<2048>::UPJ, s, grid,
                            &a.sched);
    if (st != Q8_OK) return st;
    hipLaunchKernelGGL(traffic_probe_kernel, dim3(grid), dim3(kWgThreads), 0, s, a);
    return launch_status();
}

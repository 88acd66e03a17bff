// Optimizer-step kernels for ONE storage type of w and g.  The build compiles this file three
// times (-DQ8_STEPS_F32, -DQ8_STEPS_BF16, -DQ8_STEPS_F16), in parallel; each object holds the
// adam8_kernel<B, WT> and sgd8_kernel<B, WT> instantiations for every block size B and the two
// functions through which q8opt_kernels.hip reaches them.
#include "q8opt_device.h"

namespace q8 {

#if defined(Q8_STEPS_F32)
#define Q8_STEPS_WT float
#define Q8_STEPS_NAME(f) f##_f32
#elif defined(Q8_STEPS_BF16)
#define Q8_STEPS_WT Bf16
#define Q8_STEPS_NAME(f) f##_bf16
#elif defined(Q8_STEPS_F16)
#define Q8_STEPS_WT F16
#define Q8_STEPS_NAME(f) f##_f16
#else
#error "define one of Q8_STEPS_F32, Q8_STEPS_BF16, Q8_STEPS_F16"
#endif

q8_status Q8_STEPS_NAME(run_adam)(int B, StepArgs a, const AdamScalars& sc, hipStream_t stream)
{
    Q8_DISPATCH_B(B, return (launch_adam<kB, Q8_STEPS_WT>(a, sc, stream)));
    return Q8_OK;
}

q8_status Q8_STEPS_NAME(run_sgd)(int B, StepArgs a, const SgdScalars& sc, hipStream_t stream)
{
    Q8_DISPATCH_B(B, return (launch_sgd<kB, Q8_STEPS_WT>(a, sc, stream)));
    return Q8_OK;
}

}  // namespace q8

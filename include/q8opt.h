/*
 * q8opt.h -- C ABI of the fused 8-bit optimizer step for MI355X (gfx950).
 *
 * The library implements the optimizer-state method of the paper's Sec. IV
 * ("Optimizer State Quantization for Deep Speaker Embedding Learning"):
 *   - block-wise 8-bit dynamic-tree quantization of optimizer states
 *     (tensor chunking, Eq. quant1 normalization, Eq. quant2 nearest value,
 *     Eq. quant3 dequantization), and
 *   - the SGD-momentum (Eq. sgd) and Adam (Eq. adam) updates applied to the
 *     dequantized states, followed by re-quantization ("SGD (8-bit)",
 *     "Adam (8-bit)").
 * Notation follows the paper: w weights, g gradient, m first state, r second
 * state, alpha learning rate, beta / beta1 / beta2 decay coefficients, eps,
 * B block size, N_b block absmax, Q^map codebook, T^Q codes.
 *
 * Conventions common to all entry points
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HBM
 *     addresses valid on the current HIP device.  The library never allocates
 *     or frees tensor storage; every buffer is owned by the caller.  Only
 *     q8_plan_create allocates (a small device table owned by the plan).
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Device entry points enqueue work on it and return without waiting.
 *   - Return value: Q8_OK or a negative q8_status.  Argument errors are
 *     reported before anything is enqueued; nothing throws or aborts.
 *   - B is a power of two in [64, 4096].  A tensor of n elements has
 *     ceil(n / B) blocks; the last block may be short (it is quantized over
 *     its valid elements only).  n == 0 is a no-op.
 *   - fp32 tensors (w, g, T, TD) must be 16-byte aligned, 16-bit w and g
 *     (the _bf16 and _f16 entry points) 8-byte aligned, code arrays and absmax arrays
 *     4-byte aligned, qtables 16-byte aligned (else Q8_EALIGN).
 *   - Inputs must be finite; results for NaN/Inf inputs are unspecified (no
 *     out-of-bounds access happens).
 *   - Zero-initialised optimizer state = every code equal to the code of 0.0
 *     (127 in the signed map, 0 in the unsigned map) and every N_b = 0.
 *   - All arithmetic is IEEE binary32, one rounding per operation, no fused
 *     multiply-add in the update formulas; divisions and square roots are
 *     correctly rounded.
 *   - Scheduling state: the step and quantize kernels hand out work through a
 *     job counter in device memory (module data of the library, nothing is
 *     allocated; a kernel leaves its counter zeroed).  Two kernels never share a
 *     counter while either runs: eager launches use one counter per stream
 *     (launches on one stream run in order; the per-thread default stream counts
 *     once per host thread), launches recorded by stream capture one counter per
 *     (capture, stream) pair that is reserved for as long as the process lives,
 *     so a recorded graph may be replayed on any stream next to any other work
 *     of this library.  192 streams and 64 (capture, stream) pairs per device
 *     are served this way.  Beyond that nothing fails and nothing is shared:
 *     when a 193rd stream appears the call synchronizes the device once and
 *     starts its table of streams afresh, and a launch that can be given no
 *     counter (a 65th capture; or that synchronization refused because a
 *     capture is under way) runs its kernel with a fixed assignment of work to
 *     workgroups, which is slower on large tensors and gives the same result.
 *     What the caller must not do: run two instances of one recorded launch at
 *     the same time (a graph replayed concurrently with itself, or two
 *     executable graphs instantiated from one capture running concurrently),
 *     or destroy a stream while a kernel of this library still runs on it.
 *     The device entry points enqueue exactly one kernel
 *     (q8_multi_adam8bit_step_noalloc: a few) and no memset or copy, so they
 *     can be captured once each kernel has been launched eagerly a first time
 *     (the first launch queries occupancy and the counter address).
 */
#ifndef Q8OPT_H
#define Q8OPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define Q8_API __attribute__((visibility("default")))

typedef int q8_status;
enum {
    Q8_OK = 0,
    Q8_EINVAL = -1,     /* null pointer, negative size, bad count or flags   */
    Q8_EALIGN = -2,     /* a pointer violates the alignment rules above      */
    Q8_EBLOCK = -3,     /* B is not a power of two in [64, 4096]             */
    Q8_ELAUNCH = -4,    /* the HIP runtime refused the launch or a copy      */
    Q8_ENOMEM = -5,     /* q8_plan_create could not allocate its table       */
    Q8_ECODEBOOK = -6,  /* codebook not strictly increasing within [-1, 1],
                           or too fine for the search table                  */
    Q8_ELIMIT = -7      /* list too large for q8_multi_adam8bit_step_noalloc */
};

/* flags of the Adam entry points; 0 = Eq. adam exactly as printed            */
#define Q8_FLAG_BIAS_CORRECTION 1  /* step alpha/(1-beta1^t), root scaled by 1/sqrt(1-beta2^t) */
#define Q8_FLAG_DECOUPLED_WD    2  /* w <- w - alpha*wd*w instead of g <- g + wd*w            */

/* Human-readable name of a status code (static string, never NULL). */
Q8_API const char* q8_status_str(q8_status s);

/*
 * Dynamic-tree 8-bit codebook Q^map (Sec. IV-B, "Nearest value searching").
 * Writes 256 strictly increasing binary32 values into host memory `qmap_out`.
 * Bit layout behind the values: leading bit | E zero bits (decimal exponent
 * 10^-E) | indicator 1 | F linear-fraction bits selecting the centre of one of
 * 2^F equal bins of the mantissa range [0.1, 1].  is_signed != 0: leading bit is
 * the sign, F = 6 - E (for the first state m); is_signed == 0: leading bit is a
 * further fraction bit, F = 7 - E (for the non-negative second state r).  The
 * two indicator-less patterns encode 0.0 and +1.0.  A code is the rank of its
 * value in ascending order.
 */
Q8_API q8_status q8_build_codebook(int is_signed, float* qmap_out /* host [256] */);

/*
 * Search table ("qtable") of a codebook: the codebook itself, the 255 decision
 * thresholds of Eq. quant2 (the first binary32 value above each midpoint of
 * neighbouring codes, so that "x >= threshold" decides nearest-with-ties-down
 * exactly) and a bucket table indexed by the leading bits of x.  Built on the
 * host into `qtable_out` (q8_qtable_bytes() bytes, host); the caller copies the
 * bytes to 16-byte aligned device memory once and passes that device pointer
 * to the entry points below.  Any strictly increasing 256-entry codebook within
 * [-1, 1] is accepted as long as no bucket holds more than one threshold and no
 * non-zero entry is smaller than 2^-99 in magnitude (else Q8_ECODEBOOK).
 */
Q8_API size_t    q8_qtable_bytes(void);
Q8_API q8_status q8_build_qtable(const float* qmap /* host [256] */, void* qtable_out /* host */);

/* Host evaluation of the same table lookup the kernels perform; returns the
 * code of x (|x| <= 1), or a negative q8_status.  For tests of the table. */
Q8_API int       q8_host_nearest_code(const void* qtable /* host */, float x);

/*
 * Eq. quant1 + Eq. quant2: for each block b, N[b] = max |T_b| and
 * TQ[i] = argmin_j |Q^map_j - T[i] / N[b]| (ties to the lower index); an
 * all-zero block stores N[b] = 0 and the code of 0.0.
 * T: device, n floats (read).  TQ: device, n bytes (written).  N: device,
 * ceil(n/B) floats (written).
 */
Q8_API q8_status q8_quantize_blockwise(const void* qtable, const float* T, int64_t n, int B,
                                uint8_t* TQ, float* N, void* stream);

/* Eq. quant3: TD[i] = Q^map(TQ[i]) * N[i / B].  TD: device, n floats (written). */
Q8_API q8_status q8_dequantize_blockwise(const void* qtable, const uint8_t* TQ, const float* N,
                                  int64_t n, int B, float* TD, void* stream);

/*
 * Adam (8-bit): Eq. adam on dequantized states, then re-quantization.
 * Per element, each line one binary32 operation:
 *   m_prev = Qs[m_q]*N_m[b]            r_prev = Qu[r_q]*N_r[b]
 *   (wd != 0, coupled)  g = g + wd*w
 *   m = beta1*m_prev + (1-beta1)*g     r = beta2*r_prev + ((1-beta2)*g)*g
 *   w = w - alpha * ( m / (sqrt(r) + eps) )
 * then N_m[b], m_q <- quantize(m) with the signed table and N_r[b], r_q <-
 * quantize(r) with the unsigned table.  The weight update uses the new 32-bit
 * states, not their quantized values.  1-beta1 and 1-beta2 are formed in
 * binary32 on the host.  `t` (1-based step count) is used only with
 * Q8_FLAG_BIAS_CORRECTION.
 * Extensions (not printed in Eq. adam; one binary32 operation per step as above):
 *   Q8_FLAG_BIAS_CORRECTION:  rs = sqrt(r)*c;  d = rs + eps;  w = w - alpha_t*(m/d)
 *     with alpha_t = alpha/(1-beta1^t) and c = 1/sqrt(1-beta2^t), each evaluated in
 *     binary64 from the binary32 hyper-parameters and rounded once to binary32;
 *   Q8_FLAG_DECOUPLED_WD (wd != 0):  w = w - (alpha*wd)*w  before the step is
 *     subtracted, and g is left alone.
 * In place on w, m_q, r_q, N_m, N_r (device); g is read only (device).
 */
Q8_API q8_status q8_adam8bit_step(float* w, const float* g,
                           uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
                           const void* qtable_signed, const void* qtable_unsigned,
                           int64_t n, int B,
                           float alpha, float beta1, float beta2, float eps,
                           float weight_decay, int64_t t, int flags, void* stream);

/*
 * SGD (8-bit): Eq. sgd on the dequantized state, then re-quantization.
 *   m_prev = Qs[m_q]*N_m[b];  (wd != 0) g = g + wd*w;
 *   m = beta*m_prev + g;  w = w - alpha*m;   N_m[b], m_q <- quantize(m)
 * The first case of Eq. sgd (m_0 = g_0) follows from the zero state.
 */
Q8_API q8_status q8_sgd8bit_step(float* w, const float* g, uint8_t* m_q, float* N_m,
                          const void* qtable_signed, int64_t n, int B,
                          float alpha, float beta, float weight_decay, void* stream);

/*
 * Weights and gradients stored in 16 bits (an extension; the paper keeps both in
 * binary32): bfloat16 (the upper 16 bits of a binary32; _bf16) or IEEE binary16
 * (_f16, subnormals kept, overflow rounds to infinity), passed as uint16_t.
 * Each stored w and g is widened exactly, the step runs in binary32 exactly as
 * in the entry points above (same formulas, same 8-bit states and block maxima),
 * and the new weight is rounded once, to nearest-even, back to the storage
 * type.  An update smaller than half a unit in the last place of its stored
 * weight therefore leaves that weight unchanged; the states still advance.
 * Arguments as above except for the element type of w (in place) and g.
 */
Q8_API q8_status q8_adam8bit_step_bf16(uint16_t* w, const uint16_t* g,
                                uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
                                const void* qtable_signed, const void* qtable_unsigned,
                                int64_t n, int B,
                                float alpha, float beta1, float beta2, float eps,
                                float weight_decay, int64_t t, int flags, void* stream);
Q8_API q8_status q8_sgd8bit_step_bf16(uint16_t* w, const uint16_t* g, uint8_t* m_q, float* N_m,
                               const void* qtable_signed, int64_t n, int B,
                               float alpha, float beta, float weight_decay, void* stream);
Q8_API q8_status q8_adam8bit_step_f16(uint16_t* w, const uint16_t* g,
                               uint8_t* m_q, uint8_t* r_q, float* N_m, float* N_r,
                               const void* qtable_signed, const void* qtable_unsigned,
                               int64_t n, int B,
                               float alpha, float beta1, float beta2, float eps,
                               float weight_decay, int64_t t, int flags, void* stream);
Q8_API q8_status q8_sgd8bit_step_f16(uint16_t* w, const uint16_t* g, uint8_t* m_q, float* N_m,
                              const void* qtable_signed, int64_t n, int B,
                              float alpha, float beta, float weight_decay, void* stream);

/*
 * Multi-tensor launch: the networks of Sec. V-B / Sec. VI-B (ResNets and RevNets
 * under SGD with momentum, DF-ResNets and DF-RevNets under AdamW) hold hundreds
 * of parameter tensors, each chunked on its own (Sec. IV-B, block-wise
 * quantization); one kernel launch updates a whole list of parameter
 * tensors (blocks never span tensors).  A tensor with m_f32 != NULL keeps
 * 32-bit states (m_f32, and r_f32 for Adam; same update formulas, no
 * quantization; m_q/r_q/N_m/N_r ignored); otherwise it uses 8-bit states.
 * All pointers in q8_tensor are device pointers with the alignment rules
 * above.  q8_plan_create copies the list into a device table it owns
 * (synchronous); the tensors themselves stay owned by the caller and must
 * outlive the plan's use.  r_q/N_r/r_f32 may be NULL for a plan that is only
 * used with the SGD entry point.  A tensor with n == 0 is accepted and skipped
 * (its pointers are not examined).  w and g of every tensor of a plan hold
 * binary32 (q8_plan_create), bfloat16 (q8_plan_create_bf16) or binary16
 * (q8_plan_create_f16), with the semantics of the 16-bit steps above; the
 * 32-bit states m_f32/r_f32 stay binary32.
 */
typedef struct q8_tensor {
    void*        w;
    const void*  g;
    int64_t      n;
    uint8_t*     m_q;
    uint8_t*     r_q;
    float*       N_m;
    float*       N_r;
    float*       m_f32;
    float*       r_f32;
} q8_tensor;

typedef struct q8_plan q8_plan;

Q8_API q8_status q8_plan_create(const q8_tensor* list /* host */, int count, int B, q8_plan** out);
Q8_API q8_status q8_plan_create_bf16(const q8_tensor* list /* host */, int count, int B, q8_plan** out);
Q8_API q8_status q8_plan_create_f16(const q8_tensor* list /* host */, int count, int B, q8_plan** out);
Q8_API q8_status q8_plan_destroy(q8_plan* plan);

Q8_API q8_status q8_multi_adam8bit_step(q8_plan* plan,
                                 const void* qtable_signed, const void* qtable_unsigned,
                                 float alpha, float beta1, float beta2, float eps,
                                 float weight_decay, int64_t t, int flags, void* stream);
Q8_API q8_status q8_multi_sgd8bit_step(q8_plan* plan, const void* qtable_signed,
                                float alpha, float beta, float weight_decay, void* stream);

/*
 * For callers that cannot allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid it: q8_multi_adam8bit_step without a
 * plan.  Same update, same results as q8_plan_create + q8_multi_adam8bit_step on
 * the same list (w and g binary32), but the tables a plan keeps in memory it
 * allocated (tensor descriptors, unit table) and the job counter live in a static
 * device array of the library (1 122 560 bytes per GPU, held until the process
 * ends).  `list` is host memory and is consumed before the call returns (it
 * travels inside kernel arguments); the call enqueues only kernels on `stream`
 * (ceil(count / 40) small table-fill launches, then the step): no hipMalloc, no
 * hipFree, no memset, no copy, so it may be recorded by stream capture.
 * Limits: count <= 1024 tensors and at most 131 072 units of max(B, 1024)
 * elements in total (e.g. 134 million parameters at B <= 1024, 268 million at
 * B = 2048), else Q8_ELIMIT and nothing is enqueued.  All calls on one GPU share
 * the one array: calls that overlap in time on one GPU (two streams, or a graph
 * replayed next to an eager call) race and give wrong results; calls on one
 * stream, or otherwise ordered, are safe.  Other arguments and errors as for
 * q8_plan_create and q8_multi_adam8bit_step.
 */
Q8_API q8_status q8_multi_adam8bit_step_noalloc(const q8_tensor* list /* host */, int count, int B,
                                         const void* qtable_signed, const void* qtable_unsigned,
                                         float alpha, float beta1, float beta2, float eps,
                                         float weight_decay, int64_t t, int flags, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* Q8OPT_H */

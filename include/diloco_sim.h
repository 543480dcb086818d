/*
 * diloco_sim.h - harness entry points: the noisy quadratic stand-in problem and
 * launch tuning.  Same conventions as diloco.h (device pointers owned by the
 * caller, element strides, asynchronous on `stream`, validation before launch).
 *
 * The paper's workers run forward/backward passes of a language model (lines 3-4
 * of Algorithms 1-3); here a separable quadratic
 *     L(theta) = 0.5 * sum_i h_i (theta_i - theta*_i)^2
 * stands in for it, and each replica's gradient is made inside the kernel:
 *     g_m[i] = h_i (theta_m[i] - theta*_i) + noise_std * z(seed, step, m, i)
 * z is a counter-based standard normal: elements 2j and 2j+1 of replica m at
 * step t share the 64-bit word x = mix64(key + (j+1)*0x9E3779B97F4A7C15), where
 * mix64 is the splitmix64 output function (Steele, Lea, Flood 2014) and
 * key = mix64(mix64(seed + (t+1)*G) + (m+1)*G), G the same odd constant;
 * u1 = ((x >> 40) + 1) / 2^24, u2 = ((x >> 16) & 0xFFFFFF) / 2^24,
 * r = sqrt(-2 ln u1), z_2j = r cos(2 pi u2), z_2j+1 = r sin(2 pi u2).
 */
#ifndef DILOCO_SIM_H
#define DILOCO_SIM_H

#include <stdint.h>

#include "diloco.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Lines 3-5 of Algorithms 1-3 on the quadratic: gradient made in registers, then the
 * AdamW step of diloco_inner_adamw, for every replica.  theta, m1, m2: [M][stride]
 * fp32 in place.  h, theta_star: [n] fp32 shared.  index_base is the global index of
 * element 0 of this window (so windows of one buffer draw the noise of their own
 * elements); it must be a multiple of 4.  step >= 1.
 */
int diloco_sim_quadratic_inner(float* theta, float* m1, float* m2,
                               int M, int64_t n, int64_t stride,
                               const float* h, const float* theta_star,
                               double noise_std, uint64_t seed, int64_t index_base,
                               double lr, double beta1, double beta2, double eps,
                               double weight_decay, int64_t step, void* stream);

/*
 * `steps` consecutive calls of diloco_sim_quadratic_inner, for step = step_first,
 * step_first + 1, ..., in one pass: every replica's theta, m1, m2 are read once, stepped in
 * registers and written once (legitimate for this separable stand-in problem only: a real
 * model's gradient needs the whole parameter vector of the previous step).  The results are
 * bit-identical to the separate calls.  0 <= steps <= DILOCO_SIM_MAX_FUSED_STEPS (longer
 * phases take several calls); the other arguments are those of diloco_sim_quadratic_inner.
 */
#define DILOCO_SIM_MAX_FUSED_STEPS 64
int diloco_sim_quadratic_phase(float* theta, float* m1, float* m2, int M, int64_t n,
                               int64_t stride, const float* h, const float* theta_star,
                               double noise_std, uint64_t seed, int64_t index_base,
                               double lr, double beta1, double beta2, double eps,
                               double weight_decay, int64_t step_first, int steps, void* stream);

/* Number of fp64 partial sums diloco_sim_quadratic_loss needs for n elements. */
int64_t diloco_sim_loss_workspace(int64_t n);

/*
 * loss_out[0] <- 0.5 * sum_i h_i (tbar_i - theta*_i)^2 with tbar = (1/M) sum_m theta_m
 * (fp64 accumulation, fixed order: deterministic).  theta: [M][stride] fp32.
 * partials: device workspace of n_partials >= diloco_sim_loss_workspace(n) doubles,
 * overwritten.  loss_out: one device double.
 */
int diloco_sim_quadratic_loss(const float* theta, int M, int64_t n, int64_t stride,
                              const float* h, const float* theta_star,
                              double* partials, int64_t n_partials, double* loss_out,
                              void* stream);

/*
 * diloco_sim_quadratic_loss for callers that cannot allocate and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The partial sums
 * live in a 64 KB array that is part of the library's device image (8192 doubles, one copy per GPU
 * the library runs on, held until the process ends); the call allocates nothing, on the device or
 * through any library.  Same kernels, same order of summation: the result has the bits of
 * diloco_sim_quadratic_loss.  n <= DILOCO_SIM_STATIC_LOSS_MAX_N, DILOCO_ERR_SHAPE beyond.  The
 * first call on a GPU looks the array's address up (make that call outside a graph capture).
 * All calls on one GPU share the array: calls that may overlap on one GPU (different streams
 * without an ordering between them) race on it; calls on one stream are safe back to back, since
 * every slot a call reads it has written itself.
 */
#define DILOCO_SIM_STATIC_LOSS_MAX_N ((int64_t)1 << 40)
int diloco_sim_quadratic_loss_static(const float* theta, int M, int64_t n, int64_t stride,
                                     const float* h, const float* theta_star, double* loss_out,
                                     void* stream);

/*
 * Launch shape of one call, for measurements.  The entry points of diloco.h choose their shape
 * themselves; the *_shaped variants below run the same call (same validation, same kernels, same
 * results bit for bit) in the shape the caller names, so that a harness can compare shapes
 * without any state outside the call.  launch == NULL means the automatic choice.
 *   block         threads per workgroup of the streaming kernels: 64..512, a power of two; 0 lets
 *                 the launch choose (one-wavefront workgroups, throttled as wg_per_cu -1 says).
 *   xcd_remap     0/1: give each of the 8 XCDs a contiguous slice of the index space.
 *   wg_per_cu     at most this many workgroups of the kernel resident on a compute unit (1..32,
 *                 enforced with dynamic LDS the kernel never touches); 0: no cap; -1: with block 0
 *                 the cap that puts about 32-64 KB of loads in flight per compute unit, with an
 *                 explicit block no cap.
 *   generic_path  eager step only: 0 = register-resident kernel for M <= 8, beyond that the first
 *                 40 replicas staged in LDS and the rest read twice; 1 = for every M, up to 80
 *                 staged; 2 = for every M, none staged.
 * A field out of range is DILOCO_ERR_HYPER.
 */
typedef struct diloco_launch {
    int block;
    int xcd_remap;
    int wg_per_cu;
    int generic_path;
} diloco_launch;

int diloco_inner_adamw_shaped(void* theta, void* m1, void* m2, const void* grad,
                              int M, int64_t n, int64_t stride,
                              diloco_dtype param_dtype, diloco_dtype grad_dtype,
                              double lr, double beta1, double beta2, double eps,
                              double weight_decay, int64_t step, void* stream,
                              const diloco_launch* launch);
int diloco_outer_sync_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                             float* anchor, float* vel, float* mean_out,
                             double outer_lr, double outer_momentum, int nesterov, int comm,
                             void* stream, const diloco_launch* launch);
int diloco_outer_eager_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                              float* anchor, float* vel, float* prev_local, int64_t state_stride,
                              float* prev_mean,
                              double outer_lr, double outer_momentum, int nesterov,
                              int variant, int apply_update, void* stream,
                              const diloco_launch* launch);
int diloco_outer_eager_packed_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                     int64_t stride, float* state,
                                     double outer_lr, double outer_momentum, int nesterov,
                                     int variant, int apply_update, void* stream,
                                     const diloco_launch* launch);
int diloco_outer_eager_pingpong_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                       int64_t stride, const float* state_in, float* state_out,
                                       double outer_lr, double outer_momentum, int nesterov,
                                       int variant, int apply_update, void* stream,
                                       const diloco_launch* launch);

/*
 * Measurement aid: dst[i] <- src[i] for n fp32 elements with the same 128-bit
 * non-temporal accesses and launch shape as the sweep kernels (moves 8n bytes).  The
 * rate it reaches is the practical HBM ceiling the sweeps are compared with.
 * dst, src: 16-byte aligned, non-overlapping.  launch: as above, NULL = automatic.
 */
int diloco_sim_stream_copy(float* dst, const float* src, int64_t n, void* stream,
                           const diloco_launch* launch);

/*
 * In-place sweep over K rows of n floats, `stride` floats apart: each 16-byte piece of every
 * row is read and written back unchanged, with the access shape of the outer steps (a lane
 * touches all K rows at one index).  No arithmetic: the rate it reaches is what the memory
 * system gives a read-modify-write over K separated streams, the ceiling the eager outer
 * step (K = 4M + 1) is compared with.  K in {1, 2, 4, 5, 8, 9, 16, 17, 33}; n a multiple of 4;
 * base 16-byte aligned, stride a multiple of 4.  launch: as above, NULL = automatic.
 */
int diloco_sim_stream_rmw(float* base, int K, int64_t n, int64_t stride, void* stream,
                          const diloco_launch* launch);

/*
 * The same sweep with its two halves apart, to tell which of them the memory system limits:
 * DILOCO_SIM_SWEEP_RMW is diloco_sim_stream_rmw; DILOCO_SIM_SWEEP_READ only reads the K rows
 * (moves 4Kn bytes, writes nothing); DILOCO_SIM_SWEEP_WRITE only writes them, every element set
 * to `fill` (moves 4Kn bytes).  Other modes: DILOCO_ERR_DTYPE.  Arguments as above.
 */
#define DILOCO_SIM_SWEEP_RMW 0
#define DILOCO_SIM_SWEEP_READ 1
#define DILOCO_SIM_SWEEP_WRITE 2
int diloco_sim_stream_sweep(float* base, int K, int64_t n, int64_t stride, int mode, float fill,
                            void* stream, const diloco_launch* launch);

/*
 * The launch shape that calls WITHOUT an explicit shape use on the calling thread (test aid): the
 * fields of diloco_launch by name, "block", "xcd_remap", "wg_per_cu", "generic_path", with the
 * same ranges.  The setting is per thread (thread-local storage): a thread never sees another
 * thread's values, and a new thread starts from the automatic choice.  Results do not depend
 * on any of them.  Returns DILOCO_OK, or DILOCO_ERR_HYPER for an unknown key / value
 * (diloco_tune_get: -1 for an unknown key; wg_per_cu may itself read -1).
 */
int diloco_tune(const char* key, int value);
int diloco_tune_get(const char* key);

#ifdef __cplusplus
}
#endif
#endif /* DILOCO_SIM_H */

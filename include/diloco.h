/*
 * diloco.h - C ABI of the DiLoCo optimizer sweep for one AMD MI355X (gfx950).
 *
 * The library runs, on flat parameter buffers of M simulated replicas that
 * all live in one GPU's memory, the per-parameter work of DiLoCo with
 * overlapped communication ("Eager Updates For Overlapped Communication and
 * Computation in DiLoCo", arXiv 2502.12996):
 *
 *   diloco_inner_adamw   line 5 of Algorithms 1-3 (InnerOpt = AdamW) for all replicas
 *   diloco_outer_sync    Algorithm 1, lines 7-10 (standard DiLoCo outer step)
 *   diloco_outer_eager   Algorithm 3, lines 7-12 (eager updates) and
 *                        Algorithm 2, lines 7-11 (naive delayed outer gradients)
 *   diloco_reset         the assignment theta_m <- outer parameters on its own
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer into memory owned by the caller.  The
 *     library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.  The caller keeps the buffers alive until `stream` has
 *     passed the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued asynchronously; the library never synchronises.
 *   - Buffers with a replica axis are laid out [M][stride]: replica m starts at
 *     base + m*stride elements and holds n <= stride meaningful elements.
 *     Sizes and strides count ELEMENTS.  Any (base + offset, n) window of a
 *     larger buffer is a valid argument, so a caller can sweep fragments of a
 *     model on different schedules.
 *   - Arithmetic is fp32 (bf16 buffers are widened exactly on load and rounded
 *     to nearest-even on store).  The mean over replicas is accumulated in fp64
 *     in the fixed order m = 0, 1, ..., M-1 and rounded once to fp32.
 *   - Arguments are validated before anything is launched: a call that returns
 *     an error has had no effect.  n == 0 is a successful no-op.
 *   - Pointers must be aligned to their element size.  128-bit accesses are
 *     used when every pointer is 16-byte aligned (8-byte for bf16) and every
 *     stride is a multiple of 4 elements; otherwise an element-wise path runs.
 *   - Return value: DILOCO_OK (0) or one of the diloco_status codes below.
 */
#ifndef DILOCO_H
#define DILOCO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DILOCO_F32 = 0, DILOCO_BF16 = 1 } diloco_dtype;

/* Which outer gradient OuterOpt is fed (diloco_outer_eager).  The `variant` argument is an int:
 * one of these two values in its low byte, with the DILOCO_COMM_* / DILOCO_STATE_* flag bits
 * below OR-ed in (an enum-typed parameter could not legally hold those bits). */
typedef enum {
    DILOCO_EAGER = 0,   /* Algorithm 3 line 11: (Delta_m - Delta_m_prev)/M + Delta_prev */
    DILOCO_DELAYED = 1  /* Algorithm 2 line 11: Delta_prev                              */
} diloco_variant;

/*
 * Quantised communication (Section 3.2, "Quantized Communication"): OR this flag into the
 * `variant` argument and every replica's outer gradient is rounded to bfloat16 (nearest even)
 * before it enters the mean, as if it had crossed the wire in bf16:
 *   prev_mean <- (1/M) sum_m bf16(Delta_m),  prev_local_m <- bf16(Delta_m)  (what was sent, so
 *   that next phase's eager combination removes exactly the replica's own stale share),
 * while the replica's own fresh Delta_m enters its eager combination unrounded.
 */
#define DILOCO_COMM_BF16 0x100

/*
 * The same section names float8 and float4 wire formats of the "ExMy" kind without fixing them.
 * DILOCO_COMM_EXMY(E, MN, BIAS), OR-ed into `variant` instead of DILOCO_COMM_BF16, rounds the
 * outer gradients to the format with one sign bit, E exponent bits, MN mantissa bits and exponent
 * bias BIAS, read this way: the values are +-2^(e-BIAS) (1 + f/2^MN) for exponent codes
 * e = 1 .. 2^E - 1 and +-2^(1-BIAS) f/2^MN for e = 0 (zero and subnormals), f = 0 .. 2^MN - 1;
 * every code is a number (no infinities, no NaNs); rounding is to the nearest value, ties to the
 * even code; magnitudes beyond the largest value saturate to it.  BIAS places the format's range
 * (a power-of-two scale chosen by the caller, e.g. E2M1 with BIAS 11 spans 2^-11 .. 1.5 * 2^-8).
 * Limits: 1 <= E <= 8, 0 <= MN <= 10, E + MN <= 15, -128 <= BIAS <= 127, and the format must lie
 * inside float32's normal range: 2^E - 1 - BIAS <= 127 and 1 - BIAS - MN >= -126; anything else is
 * DILOCO_ERR_DTYPE.  The state buffers keep the rounded values as float32.
 */
#define DILOCO_COMM_EXMY(E, MN, BIAS) \
    (0x200 | (((E) & 0xf) << 12) | (((MN) & 0xf) << 16) | (((BIAS) & 0xff) << 20))

/*
 * The previous averaged outer gradient Delta^(t-H) is, by Algorithm 3, the all-reduce (mean) of
 * the previous local outer gradients Delta_m^(t-H).  When all M replicas are in this call, as
 * they are in this one-GPU setting, it can be formed from them instead of being kept: OR this
 * flag into the `variant` of an EAGER call and prev_mean (or the mean stream of the packed
 * state) is neither read nor written; the call sums prev_local over m = 0..M-1 in fp64 and
 * rounds once, exactly as the call that stored prev_local would have formed prev_mean, so the
 * results are bit-identical to the flag-less calls as long as every call of a run carries the
 * flag or prev_mean is that mean.  One stream of 4M+1 less each way (11 % of the traffic at
 * M = 2, 3 % at M = 8).  EAGER only (DILOCO_ERR_DTYPE with DELAYED, which never reads
 * prev_local); any M (beyond 8 replicas the first 24 keep their prev_local on chip between the
 * two sums, the others' is read twice); prev_mean must still be a valid pointer.
 */
#define DILOCO_STATE_NO_MEAN 0x400

typedef enum {
    DILOCO_OK = 0,
    DILOCO_ERR_NULL = 1,   /* a required pointer is NULL                                   */
    DILOCO_ERR_SHAPE = 2,  /* M < 1, M > DILOCO_MAX_REPLICAS, n < 0, stride < n, overflow  */
    DILOCO_ERR_ALIGN = 3,  /* a pointer is not aligned to its element size                 */
    DILOCO_ERR_DTYPE = 4,  /* unknown dtype / variant code                                 */
    DILOCO_ERR_HYPER = 5,  /* non-finite scalar, beta or momentum outside [0,1), eps <= 0,
                              step < 1, negative weight decay                              */
    DILOCO_ERR_ALIAS = 6,  /* two buffers the call writes (or reads and writes) overlap    */
    DILOCO_ERR_LAUNCH = 7  /* the HIP runtime refused the launch                           */
} diloco_status;

#define DILOCO_MAX_REPLICAS 65535

/* Human-readable text for a status code (static storage, never NULL). */
const char* diloco_strerror(int status);

/* Library version, major*10000 + minor*100 + patch. */
int diloco_version(void);

/*
 * InnerOpt (Algorithms 1-3, line 5): one AdamW step on every replica.
 *   m1 <- beta1 m1 + (1-beta1) g ;  m2 <- beta2 m2 + (1-beta2) g^2
 *   theta <- theta - lr * ( (m1/(1-beta1^step)) / (sqrt(m2/(1-beta2^step)) + eps)
 *                           + weight_decay * theta )
 * theta, m1, m2: [M][stride] of param_dtype, updated in place.  grad: [M][stride]
 * of grad_dtype, read only.  step >= 1 is the caller's global step count t (it keeps
 * running across outer steps).  The bias corrections are evaluated on the host in
 * fp64.  Errors: NULL, SHAPE, ALIGN, DTYPE, HYPER, ALIAS, LAUNCH.
 */
int diloco_inner_adamw(void* theta, void* m1, void* m2, const void* grad,
                       int M, int64_t n, int64_t stride,
                       diloco_dtype param_dtype, diloco_dtype grad_dtype,
                       double lr, double beta1, double beta2, double eps,
                       double weight_decay, int64_t step, void* stream);

/*
 * Standard DiLoCo outer step (Algorithm 1, lines 7-10), fused into one pass:
 *   Delta_m = anchor - theta_m ; Delta = (1/M) sum_m Delta_m
 *   vel <- mu vel + Delta ; anchor <- anchor - lr (Delta + mu vel)     (nesterov != 0)
 *                           anchor <- anchor - lr vel                  (nesterov == 0)
 *   theta_m <- anchor  for every m
 * theta: [M][stride] of theta_dtype, overwritten.  anchor, vel: [n] fp32 shared by all
 * replicas (the outer parameters theta^(t-H) and OuterOpt's velocity), updated in
 * place.  mean_out: optional [n] fp32 that receives Delta, may be NULL.
 */
int diloco_outer_sync(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                      float* anchor, float* vel, float* mean_out,
                      double outer_lr, double outer_momentum, int nesterov, void* stream);

/*
 * The same step with quantised communication (Section 3.2, "Quantized Communication"):
 * Delta = (1/M) sum_m q(Delta_m), q the rounding to the wire format named by `comm`:
 * 0 (none: identical to diloco_outer_sync), DILOCO_COMM_BF16 or DILOCO_COMM_EXMY(E, MN, BIAS),
 * both defined below; anything else is DILOCO_ERR_DTYPE.
 */
int diloco_outer_sync_comm(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                           float* anchor, float* vel, float* mean_out,
                           double outer_lr, double outer_momentum, int nesterov, int comm,
                           void* stream);

/*
 * Eager (Algorithm 3, lines 7-12) or naive delayed (Algorithm 2, lines 7-11) outer
 * step, fused into one read-modify-write pass.  Every replica owns its outer
 * parameters and its OuterOpt state (Section 2.2: the replicas are never
 * re-synchronised):
 *   Delta_m = anchor_m - theta_m ; Delta = (1/M) sum_m Delta_m
 *   G_m = (Delta_m - prev_local_m)/M + prev_mean     (DILOCO_EAGER)
 *   G_m = prev_mean                                  (DILOCO_DELAYED)
 *   vel_m <- mu vel_m + G_m ; anchor_m <- anchor_m - lr (G_m + mu vel_m)  [Nesterov]
 *   theta_m <- anchor_m ; prev_local_m <- Delta_m ; prev_mean <- Delta
 * apply_update == 0 is the first boundary t = H, where the listings apply no outer
 * step: anchor_m <- theta_m, prev_local_m <- Delta_m, prev_mean <- Delta, and theta,
 * vel stay as they are.
 * theta: [M][stride] of theta_dtype.  anchor, vel, prev_local: [M][state_stride] fp32.
 * prev_mean: [n] fp32.  All are read and written (vel and prev_local are not read when
 * apply_update == 0; prev_local is not read for DILOCO_DELAYED).
 */
int diloco_outer_eager(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                       float* anchor, float* vel, float* prev_local, int64_t state_stride,
                       float* prev_mean,
                       double outer_lr, double outer_momentum, int nesterov,
                       int variant, int apply_update, void* stream);

/*
 * Packed outer state.  The eager / delayed outer step touches 3M+1 state streams per
 * parameter index (outer parameters, velocity and previous local outer gradient of every
 * replica, plus the previous mean).  Kept as separate [M][state_stride] rows they lie
 * gigabytes apart, and a wavefront's 3M+1 accesses land in 3M+1 different pages.  The
 * packed form is one buffer of diloco_packed_state_elems(M, n) floats laid out
 * [tile][3M+1][DILOCO_STATE_TILE]: tile t holds, for parameter indices
 * [t*8192, (t+1)*8192), in the order the kernel touches them: streams 0..M-1 = outer
 * parameters of replicas 0..M-1, stream M = the previous mean, stream M+1+2m = velocity of
 * replica m, stream M+2+2m = its previous local outer gradient.  The last tile is padded.
 * A window [off, off+n) of a larger model may be swept on its own when off is a multiple
 * of DILOCO_STATE_TILE: pass state + (off/8192)*(3M+1)*8192.
 * diloco_outer_eager_packed computes exactly what diloco_outer_eager computes (same
 * arithmetic, same order, bit-identical results); only the addresses differ.
 * state must be 16-byte aligned.
 */
#define DILOCO_STATE_TILE 8192

/* Floats in the packed state of M replicas x n parameters; -1 for invalid M or n. */
int64_t diloco_packed_state_elems(int M, int64_t n);

/* rows -> packed.  anchor, vel, prev_local: [M][state_stride] fp32; prev_mean: [n] fp32;
 * any of the four may be NULL, its streams are then left as they are.  The two conversions
 * take 3M+1 <= 65535 (M <= 21844), DILOCO_ERR_SHAPE beyond. */
int diloco_pack_state(float* state, int M, int64_t n, const float* anchor, const float* vel,
                      const float* prev_local, int64_t state_stride, const float* prev_mean,
                      void* stream);

/* packed -> rows; NULL destinations are skipped. */
int diloco_unpack_state(const float* state, int M, int64_t n, float* anchor, float* vel,
                        float* prev_local, int64_t state_stride, float* prev_mean, void* stream);

/* diloco_outer_eager on the packed state (Algorithm 3 lines 7-12 / Algorithm 2 lines 7-11). */
int diloco_outer_eager_packed(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                              int64_t stride, float* state,
                              double outer_lr, double outer_momentum, int nesterov,
                              int variant, int apply_update, void* stream);

/*
 * The same step (Algorithm 3 lines 7-12 / Algorithm 2 lines 7-11) reading the packed outer state
 * from state_in and writing the new one to state_out, two separate buffers of
 * diloco_packed_state_elems(M, n) floats that the caller swaps between boundaries.  On this chip
 * a sweep that reads one buffer and writes another streams 1-2 % faster than the same sweep in
 * place; the price is a second state buffer (with 288 GB of HBM the M = 8, 617M-parameter
 * configuration still fits twice over).  Results are bit-identical to
 * diloco_outer_eager_packed.  Every stream of state_out is written (at the first boundary,
 * apply_update == 0, the velocities are copied across), except the mean stream under
 * DILOCO_STATE_NO_MEAN, which no flagged call reads.  theta is updated in place.
 * state_in == state_out or overlapping buffers: DILOCO_ERR_ALIAS.
 */
int diloco_outer_eager_pingpong(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                int64_t stride, const float* state_in, float* state_out,
                                double outer_lr, double outer_momentum, int nesterov,
                                int variant, int apply_update, void* stream);

/*
 * Two-outer-steps overlap (Section 3.2, "Two-outer-steps overlap": the all-reduce launched at a
 * boundary is consumed two boundaries later; the paper gives no formula, reading: Algorithms 2 / 3
 * with Delta_m^(t-2H), Delta^(t-2H) in place of Delta_m^(t-H), Delta^(t-H) and `if t > 2H`) on
 * the packed state.  Two packed buffers hold the two generations in flight.  At boundary b
 * (1, 2, ...) the caller passes state_prev = the buffer written at boundary b-1 (its outer
 * parameters and velocities are the current ones) and state_cur = the buffer written at boundary
 * b-2 (its previous local / averaged outer gradients are the ones this step consumes); the call
 * writes the complete new state to state_cur.  So the caller alternates: S[(b-1) % 2], S[b % 2].
 * Both buffers start from the same packed state; apply_update == 0 at boundaries 1 and 2.
 * DILOCO_STATE_NO_MEAN is refused (DILOCO_ERR_DTYPE); everything else as
 * diloco_outer_eager_pingpong.
 */
int diloco_outer_eager_overlap2(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                int64_t stride, const float* state_prev, float* state_cur,
                                double outer_lr, double outer_momentum, int nesterov,
                                int variant, int apply_update, void* stream);

/* theta_m <- outer parameters of replica m, read from the packed state. */
int diloco_reset_packed(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                        const float* state, void* stream);

/*
 * Streaming DiLoCo schedule (Section 3 of the paper: all its experiments apply the outer
 * step to fragments of the model, e.g. 3 consecutive layers, on different schedules).  The
 * outer-step entry points accept any (pointer + offset, n) window, so a fragment is swept
 * by passing its window; these host-side helpers only say WHEN.  The paper does not give
 * the stagger; this library spreads the fragments evenly over the H inner steps:
 * fragment f of F has its outer boundaries at the steps t >= 1 with
 * t mod H == diloco_stream_offset(H, F, f) = floor(f*H/F).
 * diloco_stream_due returns 1 if step t is such a boundary, 0 if not, -1 for bad arguments
 * (H < 1, F < 1, f outside [0, F), t < 0).  diloco_stream_boundary_count returns how many
 * boundaries fragment f has had up to and including step t (the first one is the one where
 * Algorithms 2 and 3 apply no outer step), -1 for bad arguments.
 */
int64_t diloco_stream_offset(int64_t H, int F, int f);
int diloco_stream_due(int64_t t, int64_t H, int F, int f);
int64_t diloco_stream_boundary_count(int64_t t, int64_t H, int F, int f);

/*
 * theta_m <- anchor_m for every replica (the left-hand side of Algorithm 1 line 10 /
 * Algorithm 3 line 12 on its own).  anchor_stride == 0 broadcasts one shared [n]
 * buffer; otherwise anchor is [M][anchor_stride].  Idempotent.
 */
int diloco_reset(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                 const float* anchor, int64_t anchor_stride, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DILOCO_H */

// InnerOpt = AdamW (line 5 of Algorithms 1-3) for all replicas in one launch, and the same
// step with the gradient of the noisy quadratic stand-in problem made in registers.
//
// Grid: x walks the parameter index in 128-bit vectors, y is the replica.  Each thread
// reads theta, m1, m2, g once and writes theta, m1, m2 once (28 bytes per fp32 parameter).
#include "common.hpp"
#include "diloco_sim.h"

namespace diloco {

struct AdamScalars {
    float beta1, omb1;  // beta1, 1 - beta1
    float beta2, omb2;
    float inv_bc1;      // 1 / (1 - beta1^t)
    float inv_bc2;      // 1 / (1 - beta2^t)
    float eps, lr, wd;
};

// m1 <- b1 m1 + (1-b1) g ; m2 <- b2 m2 + (1-b2) g^2 ;
// theta <- theta - lr ( m1_hat / (sqrt(m2_hat) + eps) + wd theta )
template <typename T>
__device__ __forceinline__ void adamw_update(T& th, T& m1, T& m2, T g, const AdamScalars& sc, float inv_bc1,
                                             float inv_bc2) {
    m1 = fma_(splat<T>(sc.beta1), m1, sc.omb1 * g);
    m2 = fma_(splat<T>(sc.beta2), m2, (sc.omb2 * g) * g);
    const T denom = sqrt_(m2 * inv_bc2) + sc.eps;
    const T upd = (m1 * inv_bc1) / denom;
    th = fma_(splat<T>(-sc.lr), fma_(splat<T>(sc.wd), th, upd), th);
}
template <typename T>
__device__ __forceinline__ void adamw_update(T& th, T& m1, T& m2, T g, const AdamScalars& sc) {
    adamw_update(th, m1, m2, g, sc, sc.inv_bc1, sc.inv_bc2);
}

template <typename PT, typename GT>
__global__ __launch_bounds__(kMaxBlock) void adamw_vec_kernel(PT* __restrict__ theta, PT* __restrict__ m1, PT* __restrict__ m2,
                                 const GT* __restrict__ grad, int64_t n, int64_t stride,
                                 AdamScalars sc, int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    const int64_t row = (int64_t)blockIdx.y * stride;
    if (v > nvec) return;
    if (v == nvec) {
        for (int64_t i = row + (n & ~(int64_t)3); i < row + n; ++i) {
            float t = load1(theta + i), a = load1(m1 + i), b = load1(m2 + i);
            adamw_update(t, a, b, load1(grad + i), sc);
            store1(theta + i, t);
            store1(m1 + i, a);
            store1(m2 + i, b);
        }
        return;
    }
    const int64_t i = row + (v << 2);
    f4 t = load4(theta + i), a = load4(m1 + i), b = load4(m2 + i), g = load4(grad + i);
    adamw_update(t, a, b, g, sc);
    store4(theta + i, t);
    store4(m1 + i, a);
    store4(m2 + i, b);
}

template <typename PT, typename GT>
__global__ __launch_bounds__(kMaxBlock) void adamw_scalar_kernel(PT* theta, PT* m1, PT* m2, const GT* grad, int64_t n,
                                    int64_t stride, AdamScalars sc, int64_t per_xcd) {
    const int64_t e = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    if (e >= n) return;
    const int64_t i = (int64_t)blockIdx.y * stride + e;
    float t = load1(theta + i), a = load1(m1 + i), b = load1(m2 + i);
    adamw_update(t, a, b, load1(grad + i), sc);
    store1(theta + i, t);
    store1(m1 + i, a);
    store1(m2 + i, b);
}

// ---------------------------------------------------------------- noisy quadratic
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t x) {  // splitmix64 output function
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

// Two standard normals from pair index j of the stream `key` (Box-Muller on 24-bit uniforms).
__device__ __forceinline__ void normal_pair(uint64_t key, uint64_t j, float& z0, float& z1) {
    const uint64_t x = mix64(key + kGolden * (j + 1));
    const float u1 = (float)((uint32_t)(x >> 40) + 1u) * 5.9604644775390625e-8f;  // (0, 1]
    const float u2 = (float)((uint32_t)(x >> 16) & 0xFFFFFFu) * 5.9604644775390625e-8f;  // [0, 1)
    const float r = sqrtf(-2.0f * logf(u1));
    float s, c;
    sincospif(2.0f * u2, &s, &c);
    z0 = r * c;
    z1 = r * s;
}

__global__ __launch_bounds__(kMaxBlock) void quadratic_inner_kernel(float* __restrict__ theta, float* __restrict__ m1,
                                       float* __restrict__ m2, const float* __restrict__ h,
                                       const float* __restrict__ star, int M, int64_t n,
                                       int64_t stride, float noise_std, uint64_t seed_step_key,
                                       int64_t index_base, AdamScalars sc, int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    if (v > nvec) return;
    if (v == nvec) {
        for (int64_t e = n & ~(int64_t)3; e < n; ++e) {
            const float hh = h[e], ss = star[e];
            const uint64_t gi = (uint64_t)(index_base + e);
            for (int m = 0; m < M; ++m) {
                const uint64_t key = mix64(seed_step_key + kGolden * (uint64_t)(m + 1));
                float z0, z1;
                normal_pair(key, gi >> 1, z0, z1);
                const int64_t i = m * stride + e;
                float t = theta[i], a = m1[i], b = m2[i];
                const float g = fmaf(noise_std, (gi & 1) ? z1 : z0, hh * (t - ss));
                adamw_update(t, a, b, g, sc);
                theta[i] = t;
                m1[i] = a;
                m2[i] = b;
            }
        }
        return;
    }
    const int64_t e = v << 2;
    // h and theta* are re-read by every replica of this index: plain (cached) loads
    const f4 hh = *reinterpret_cast<const f4*>(h + e);
    const f4 ss = *reinterpret_cast<const f4*>(star + e);
    const uint64_t j = (uint64_t)(index_base + e) >> 1;
    for (int m = 0; m < M; ++m) {
        const uint64_t key = mix64(seed_step_key + kGolden * (uint64_t)(m + 1));
        float z0, z1, z2, z3;
        normal_pair(key, j, z0, z1);
        normal_pair(key, j + 1, z2, z3);
        const f4 z = {z0, z1, z2, z3};
        const int64_t i = m * stride + e;
        f4 t = load4(theta + i), a = load4(m1 + i), b = load4(m2 + i);
        f4 g = fma_(splat<f4>(noise_std), z, hh * (t - ss));
        adamw_update(t, a, b, g, sc);
        store4(theta + i, t);
        store4(m1 + i, a);
        store4(m2 + i, b);
    }
}

// The same steps for `steps` consecutive values of t in one pass (grid.y = replica): theta, m1, m2
// are read once, stepped in registers and written once, which leaves the noise generator, the
// square root and the division as the only cost: this kernel is bound by the vector ALU, not by
// HBM.  Per element the arithmetic is the one of quadratic_inner_kernel in the same order.
struct PhaseScalars {
    float inv_bc1[DILOCO_SIM_MAX_FUSED_STEPS];  // 1 / (1 - beta1^t) for t = step_first + s
    float inv_bc2[DILOCO_SIM_MAX_FUSED_STEPS];
};

__global__ __launch_bounds__(kMaxBlock) void quadratic_phase_kernel(
    float* __restrict__ theta, float* __restrict__ m1, float* __restrict__ m2, const float* __restrict__ h,
    const float* __restrict__ star, int64_t n, int64_t stride, float noise_std, uint64_t seed, int64_t step_first,
    int steps, int64_t index_base, AdamScalars sc, PhaseScalars ps, int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    if (v > nvec) return;
    const int m = blockIdx.y;
    if (v == nvec) {
        for (int64_t e = n & ~(int64_t)3; e < n; ++e) {
            const float hh = h[e], ss = star[e];
            const uint64_t gi = (uint64_t)(index_base + e);
            const int64_t i = m * stride + e;
            float t = theta[i], a = m1[i], b = m2[i];
            for (int s = 0; s < steps; ++s) {
                const uint64_t k0 = mix64(seed + kGolden * (uint64_t)(step_first + s + 1));
                const uint64_t key = mix64(k0 + kGolden * (uint64_t)(m + 1));
                float z0, z1;
                normal_pair(key, gi >> 1, z0, z1);
                const float g = fmaf(noise_std, (gi & 1) ? z1 : z0, hh * (t - ss));
                adamw_update(t, a, b, g, sc, ps.inv_bc1[s], ps.inv_bc2[s]);
            }
            theta[i] = t;
            m1[i] = a;
            m2[i] = b;
        }
        return;
    }
    const int64_t e = v << 2;
    const f4 hh = *reinterpret_cast<const f4*>(h + e);
    const f4 ss = *reinterpret_cast<const f4*>(star + e);
    const uint64_t j = (uint64_t)(index_base + e) >> 1;
    const int64_t i = m * stride + e;
    f4 t = load4(theta + i), a = load4(m1 + i), b = load4(m2 + i);
    for (int s = 0; s < steps; ++s) {
        const uint64_t k0 = mix64(seed + kGolden * (uint64_t)(step_first + s + 1));
        const uint64_t key = mix64(k0 + kGolden * (uint64_t)(m + 1));
        float z0, z1, z2, z3;
        normal_pair(key, j, z0, z1);
        normal_pair(key, j + 1, z2, z3);
        const f4 z = {z0, z1, z2, z3};
        const f4 g = fma_(splat<f4>(noise_std), z, hh * (t - ss));
        adamw_update(t, a, b, g, sc, ps.inv_bc1[s], ps.inv_bc2[s]);
    }
    store4(theta + i, t);
    store4(m1 + i, a);
    store4(m2 + i, b);
}

// ---------------------------------------------------------------- host side
static int check_adam_hyper(double lr, double b1, double b2, double eps, double wd, int64_t step) {
    if (!is_finite(lr) || !in_unit(b1) || !in_unit(b2) || !is_finite(eps) || eps <= 0.0 ||
        !is_finite(wd) || wd < 0.0 || step < 1)
        return DILOCO_ERR_HYPER;
    return DILOCO_OK;
}
static AdamScalars make_adam(double lr, double b1, double b2, double eps, double wd, int64_t step) {
    AdamScalars sc;
    sc.beta1 = (float)b1;
    sc.omb1 = (float)(1.0 - b1);
    sc.beta2 = (float)b2;
    sc.omb2 = (float)(1.0 - b2);
    sc.inv_bc1 = (float)(1.0 / (1.0 - std::pow(b1, (double)step)));
    sc.inv_bc2 = (float)(1.0 / (1.0 - std::pow(b2, (double)step)));
    sc.eps = (float)eps;
    sc.lr = (float)lr;
    sc.wd = (float)wd;
    return sc;
}

template <typename PT, typename GT>
static int launch_adamw(void* theta, void* m1, void* m2, const void* grad, int M, int64_t n,
                        int64_t stride, const AdamScalars& sc, bool vec_ok, hipStream_t st, const Tuning& t) {
    // a wavefront of the vector kernel loads theta, m1, m2 and the gradient of 256 parameters
    const Shape shape = launch_shape(t, (int64_t)64 * 4 * (3 * sizeof(PT) + sizeof(GT)), kInFlightTarget, false);
    const int block = shape.block;
    const int64_t threads = vec_ok ? (n >> 2) + ((n & 3) ? 1 : 0) : n;
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    if (vec_ok) {
        if (!grant_lds(&adamw_vec_kernel<PT, GT>, shape.lds)) return DILOCO_ERR_LAUNCH;
        return launch(adamw_vec_kernel<PT, GT>, dim3(g.blocks, M), dim3(block), shape.lds, st,
                      static_cast<PT*>(theta), static_cast<PT*>(m1), static_cast<PT*>(m2),
                      static_cast<const GT*>(grad), n, stride, sc, g.per_xcd);
    }
    return launch(adamw_scalar_kernel<PT, GT>, dim3(g.blocks, M), dim3(block), 0, st, static_cast<PT*>(theta),
                  static_cast<PT*>(m1), static_cast<PT*>(m2), static_cast<const GT*>(grad), n, stride, sc,
                  g.per_xcd);
}

static int inner_adamw_impl(void* theta, void* m1, void* m2, const void* grad, int M, int64_t n, int64_t stride,
                            int param_dtype, int grad_dtype, double lr, double beta1, double beta2, double eps,
                            double weight_decay, int64_t step, void* stream, const Tuning& t);

}  // namespace diloco

using namespace diloco;

extern "C" int diloco_inner_adamw(void* theta, void* m1, void* m2, const void* grad, int M,
                                  int64_t n, int64_t stride, diloco_dtype param_dtype,
                                  diloco_dtype grad_dtype, double lr, double beta1, double beta2,
                                  double eps, double weight_decay, int64_t step, void* stream) {
    return inner_adamw_impl(theta, m1, m2, grad, M, n, stride, param_dtype, grad_dtype, lr, beta1, beta2, eps,
                            weight_decay, step, stream, tuning());
}

extern "C" int diloco_inner_adamw_shaped(void* theta, void* m1, void* m2, const void* grad, int M,
                                         int64_t n, int64_t stride, diloco_dtype param_dtype,
                                         diloco_dtype grad_dtype, double lr, double beta1, double beta2,
                                         double eps, double weight_decay, int64_t step, void* stream,
                                         const diloco_launch* launch_arg) {
    Tuning t;
    if (!resolve_launch(launch_arg, t)) return DILOCO_ERR_HYPER;
    return inner_adamw_impl(theta, m1, m2, grad, M, n, stride, param_dtype, grad_dtype, lr, beta1, beta2, eps,
                            weight_decay, step, stream, t);
}

static int diloco::inner_adamw_impl(void* theta, void* m1, void* m2, const void* grad, int M, int64_t n,
                                    int64_t stride, int param_dtype, int grad_dtype, double lr, double beta1,
                                    double beta2, double eps, double weight_decay, int64_t step, void* stream,
                                    const Tuning& t) {
    if (!theta || !m1 || !m2 || !grad) return DILOCO_ERR_NULL;
    if (!valid_dtype(param_dtype) || !valid_dtype(grad_dtype)) return DILOCO_ERR_DTYPE;
    if (int e = check_shape(M, n, stride)) return e;
    if (int e = check_adam_hyper(lr, beta1, beta2, eps, weight_decay, step)) return e;
    const int ps = elem_size(param_dtype), gs = elem_size(grad_dtype);
    if (!aligned_to(theta, ps) || !aligned_to(m1, ps) || !aligned_to(m2, ps) || !aligned_to(grad, gs))
        return DILOCO_ERR_ALIGN;
    Range r[4] = {{theta, extent_bytes(M, n, stride, ps), true},
                  {m1, extent_bytes(M, n, stride, ps), true},
                  {m2, extent_bytes(M, n, stride, ps), true},
                  {grad, extent_bytes(M, n, stride, gs), false}};
    if (int e = check_alias(r, 4)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(theta, 4 * ps) && aligned_to(m1, 4 * ps) && aligned_to(m2, 4 * ps) &&
                        aligned_to(grad, 4 * gs) && (M == 1 || stride % 4 == 0);
    const AdamScalars sc = make_adam(lr, beta1, beta2, eps, weight_decay, step);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (param_dtype == DILOCO_F32 && grad_dtype == DILOCO_F32)
        return launch_adamw<float, float>(theta, m1, m2, grad, M, n, stride, sc, vec_ok, st, t);
    if (param_dtype == DILOCO_F32)
        return launch_adamw<float, __bf16>(theta, m1, m2, grad, M, n, stride, sc, vec_ok, st, t);
    if (grad_dtype == DILOCO_F32)
        return launch_adamw<__bf16, float>(theta, m1, m2, grad, M, n, stride, sc, vec_ok, st, t);
    return launch_adamw<__bf16, __bf16>(theta, m1, m2, grad, M, n, stride, sc, vec_ok, st, t);
}

extern "C" int diloco_sim_quadratic_inner(float* theta, float* m1, float* m2, int M, int64_t n,
                                          int64_t stride, const float* h, const float* theta_star,
                                          double noise_std, uint64_t seed, int64_t index_base,
                                          double lr, double beta1, double beta2, double eps,
                                          double weight_decay, int64_t step, void* stream) {
    if (!theta || !m1 || !m2 || !h || !theta_star) return DILOCO_ERR_NULL;
    if (int e = check_shape(M, n, stride)) return e;
    if (index_base < 0 || (index_base & 3)) return DILOCO_ERR_SHAPE;
    if (int e = check_adam_hyper(lr, beta1, beta2, eps, weight_decay, step)) return e;
    if (!is_finite(noise_std) || noise_std < 0.0) return DILOCO_ERR_HYPER;
    // this entry point has no element-wise variant: 16-byte alignment is required
    if (!aligned_to(theta, 16) || !aligned_to(m1, 16) || !aligned_to(m2, 16) || !aligned_to(h, 16) ||
        !aligned_to(theta_star, 16) || (M > 1 && stride % 4 != 0))
        return DILOCO_ERR_ALIGN;
    Range r[5] = {{theta, extent_bytes(M, n, stride, 4), true},
                  {m1, extent_bytes(M, n, stride, 4), true},
                  {m2, extent_bytes(M, n, stride, 4), true},
                  {h, n * 4, false},
                  {theta_star, n * 4, false}};
    if (int e = check_alias(r, 5)) return e;
    if (n == 0) return DILOCO_OK;
    const AdamScalars sc = make_adam(lr, beta1, beta2, eps, weight_decay, step);
    const uint64_t k0 = mix64(seed + kGolden * (uint64_t)(step + 1));
    // the kernel walks the replicas one at a time: a wavefront has h, theta* and one replica's
    // theta, m1, m2 in flight, 16 B a lane each; the noise generator keeps the ALU busy for long, so
    // more wavefronts than for the plain sweeps pay (measured best at M = 4: 12 workgroups per CU)
    const Tuning& t = tuning();
    const Shape shape = launch_shape(t, (int64_t)64 * 16 * 5, 64 * 1024);
    const int block = shape.block;
    const int64_t threads = (n >> 2) + ((n & 3) ? 1 : 0);
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    if (!grant_lds(&quadratic_inner_kernel, shape.lds)) return DILOCO_ERR_LAUNCH;
    return launch(quadratic_inner_kernel, dim3(g.blocks), dim3(block), shape.lds, static_cast<hipStream_t>(stream),
                  theta, m1, m2, h, theta_star, M, n, stride, (float)noise_std, k0, index_base, sc, g.per_xcd);
}

extern "C" int diloco_sim_quadratic_phase(float* theta, float* m1, float* m2, int M, int64_t n,
                                          int64_t stride, const float* h, const float* theta_star,
                                          double noise_std, uint64_t seed, int64_t index_base,
                                          double lr, double beta1, double beta2, double eps,
                                          double weight_decay, int64_t step_first, int steps, void* stream) {
    if (!theta || !m1 || !m2 || !h || !theta_star) return DILOCO_ERR_NULL;
    if (int e = check_shape(M, n, stride)) return e;
    if (index_base < 0 || (index_base & 3)) return DILOCO_ERR_SHAPE;
    if (steps < 0 || steps > DILOCO_SIM_MAX_FUSED_STEPS) return DILOCO_ERR_SHAPE;
    if (int e = check_adam_hyper(lr, beta1, beta2, eps, weight_decay, step_first)) return e;
    if (step_first > ((int64_t)1 << 60)) return DILOCO_ERR_HYPER;
    if (!is_finite(noise_std) || noise_std < 0.0) return DILOCO_ERR_HYPER;
    if (!aligned_to(theta, 16) || !aligned_to(m1, 16) || !aligned_to(m2, 16) || !aligned_to(h, 16) ||
        !aligned_to(theta_star, 16) || (M > 1 && stride % 4 != 0))
        return DILOCO_ERR_ALIGN;
    Range r[5] = {{theta, extent_bytes(M, n, stride, 4), true},
                  {m1, extent_bytes(M, n, stride, 4), true},
                  {m2, extent_bytes(M, n, stride, 4), true},
                  {h, n * 4, false},
                  {theta_star, n * 4, false}};
    if (int e = check_alias(r, 5)) return e;
    if (n == 0 || steps == 0) return DILOCO_OK;
    const AdamScalars sc = make_adam(lr, beta1, beta2, eps, weight_decay, step_first);
    PhaseScalars ps;
    for (int s = 0; s < DILOCO_SIM_MAX_FUSED_STEPS; ++s) {
        const AdamScalars one = make_adam(lr, beta1, beta2, eps, weight_decay, step_first + (s < steps ? s : 0));
        ps.inv_bc1[s] = one.inv_bc1;
        ps.inv_bc2[s] = one.inv_bc2;
    }
    // bound by the vector ALU: full occupancy, no throttle
    const Tuning& t = tuning();
    const int block = plain_block(t);
    const int64_t threads = (n >> 2) + ((n & 3) ? 1 : 0);
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    return launch(quadratic_phase_kernel, dim3(g.blocks, M), dim3(block), 0, static_cast<hipStream_t>(stream), theta,
                  m1, m2, h, theta_star, n, stride, (float)noise_std, seed, step_first, steps, index_base, sc, ps,
                  g.per_xcd);
}

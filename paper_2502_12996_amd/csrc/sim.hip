// Loss of the quadratic stand-in problem (deterministic two-stage fp64 reduction),
// launch tuning, status strings.
#include <cstring>
#include <mutex>
#include <unordered_map>

#include "common.hpp"
#include "diloco_sim.h"

namespace diloco {

Tuning& tuning() {
    static thread_local Tuning t;  // per calling thread: no caller sees another thread's shape
    return t;
}

bool grant_lds_for(const void* kernel, size_t lds) {
    static std::mutex lock;
    static std::unordered_map<uintptr_t, size_t> granted;  // per kernel and device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> hold(lock);
    size_t& have = granted[reinterpret_cast<uintptr_t>(kernel) ^ ((uintptr_t)(dev + 1) << 56)];
    if (lds <= have) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    have = lds;
    return true;
}

constexpr int kLossBlock = 256;
constexpr int64_t kLossMaxBlocks = 8192;

// Stage 1: workgroup b sums 0.5 h (tbar - theta*)^2 over its grid-strided share in fp64,
// tbar = replica mean (left to right, fp64).  Fixed tree inside the workgroup.
__global__ void quadratic_loss_partial_kernel(const float* __restrict__ theta, int M, int64_t n,
                                              int64_t stride, const float* __restrict__ h,
                                              const float* __restrict__ star,
                                              double* __restrict__ partials, double inv_M) {
    __shared__ double red[kLossBlock];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kLossBlock + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kLossBlock) {
        double t = 0.0;
        for (int m = 0; m < M; ++m) t += (double)theta[m * stride + i];
        const double d = t * inv_M - (double)star[i];
        acc += 0.5 * (double)h[i] * d * d;
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = kLossBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[blockIdx.x] = red[0];
}

// Stage 2: one workgroup folds the partial sums, again in a fixed order.
__global__ void quadratic_loss_final_kernel(const double* __restrict__ partials, int64_t count,
                                            double* __restrict__ out) {
    __shared__ double red[kLossBlock];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += kLossBlock) acc += partials[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = kLossBlock / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = red[0];
}

__global__ __launch_bounds__(kMaxBlock) void stream_copy_kernel(float* __restrict__ dst,
                                                                const float* __restrict__ src,
                                                                int64_t n, int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    if (v > nvec) return;
    if (v == nvec) {
        for (int64_t i = n & ~(int64_t)3; i < n; ++i) store1(dst + i, load1(src + i));
        return;
    }
    store4(dst + (v << 2), load4(src + (v << 2)));
}

// In-place sweep over K rows `stride` apart: every lane loads its 16 bytes of all K rows, then
// stores them back unchanged.  No arithmetic: what is left is the memory system's rate for a
// read-modify-write over K separated streams, the access pattern of the outer steps.
// MODE 0: read every row's piece, write it back.  1: read only (the values are summed and the sum
// compared with a value no input produces, so that the loads cannot be dropped; nothing is
// written).  2: write only (every piece is filled with `fill`).
template <int K, int MODE>
__global__ __launch_bounds__(kMaxBlock) void stream_sweep_kernel(float* __restrict__ base, int64_t stride,
                                                                 int64_t n, float fill, int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    if (v >= (n >> 2)) return;
    f4 x[K];
    if (MODE != 2) {
#pragma unroll
        for (int k = 0; k < K; ++k) x[k] = load4(base + k * stride + (v << 2));
    } else {
#pragma unroll
        for (int k = 0; k < K; ++k) x[k] = f4{fill, fill, fill, fill};
    }
    if (MODE == 1) {
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k) acc += (x[k].x + x[k].y) + (x[k].z + x[k].w);
        if (acc != fill) return;  // `fill` is a NaN for this mode: never equal, the store below never happens
    }
#pragma unroll
    for (int k = 0; k < K; ++k) store4(base + k * stride + (v << 2), x[k]);
}

template <int K, int MODE>
static int launch_sweep_mode(float* base, int64_t stride, int64_t n, float fill, hipStream_t st, const Tuning& t) {
    // bytes a wavefront has in flight: its K loads, or (write only) its K stores
    const Shape shape = launch_shape(t, (int64_t)64 * 16 * K, kInFlightTarget);
    const int64_t threads = n >> 2;
    if (!grid_fits(threads, shape.block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, shape.block);
    if (!grant_lds(&stream_sweep_kernel<K, MODE>, shape.lds)) return DILOCO_ERR_LAUNCH;
    return launch(stream_sweep_kernel<K, MODE>, dim3(g.blocks), dim3(shape.block), shape.lds, st, base, stride, n, fill,
                  g.per_xcd);
}
template <int K>
static int launch_sweep(float* base, int64_t stride, int64_t n, int mode, float fill, hipStream_t st,
                        const Tuning& t) {
    if (mode == 0) return launch_sweep_mode<K, 0>(base, stride, n, 0.f, st, t);
    if (mode == 1) return launch_sweep_mode<K, 1>(base, stride, n, __builtin_nanf(""), st, t);
    return launch_sweep_mode<K, 2>(base, stride, n, fill, st, t);
}

// Partial sums of the allocation-free loss: one copy of this array per GPU the library runs on,
// held until the process ends.  In host code the name is only a handle for hipGetSymbolAddress;
// the address kernels take is looked up once per device and kept.
static __device__ __align__(256) double loss_scratch[kLossMaxBlocks];
constexpr int kMaxDevices = 64;

// Device address of the current GPU's loss_scratch (looked up on the first call on that GPU).
static int static_loss_scratch(double** out) {
    static std::mutex lock;
    static double* ptrs[kMaxDevices];  // zero-initialised: not looked up yet
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DILOCO_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(lock);
    if (!ptrs[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(loss_scratch)) != hipSuccess || !p) return DILOCO_ERR_LAUNCH;
        ptrs[dev] = static_cast<double*>(p);
    }
    *out = ptrs[dev];
    return DILOCO_OK;
}

static int64_t loss_blocks(int64_t n) {
    int64_t b = (n + kLossBlock * 4 - 1) / (kLossBlock * 4);
    if (b < 1) b = 1;
    if (b > kLossMaxBlocks) b = kLossMaxBlocks;
    return b;
}

}  // namespace diloco

using namespace diloco;

extern "C" int64_t diloco_sim_loss_workspace(int64_t n) { return n < 0 ? 0 : loss_blocks(n); }

extern "C" int diloco_sim_quadratic_loss(const float* theta, int M, int64_t n, int64_t stride,
                                         const float* h, const float* theta_star, double* partials,
                                         int64_t n_partials, double* loss_out, void* stream) {
    if (!theta || !h || !theta_star || !partials || !loss_out) return DILOCO_ERR_NULL;
    if (int e = check_shape(M, n, stride)) return e;
    if (n_partials < loss_blocks(n)) return DILOCO_ERR_SHAPE;
    if (!aligned_to(theta, 4) || !aligned_to(h, 4) || !aligned_to(theta_star, 4) ||
        !aligned_to(partials, 8) || !aligned_to(loss_out, 8))
        return DILOCO_ERR_ALIGN;
    Range r[5] = {{theta, extent_bytes(M, n, stride, 4), false},
                  {h, n * 4, false},
                  {theta_star, n * 4, false},
                  {partials, n_partials * 8, true},
                  {loss_out, 8, true}};
    if (int e = check_alias(r, 5)) return e;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nb = loss_blocks(n);
    if (int e = launch(quadratic_loss_partial_kernel, dim3((unsigned)nb), dim3(kLossBlock), 0, st, theta, M, n,
                       stride, h, theta_star, partials, 1.0 / M))
        return e;
    return launch(quadratic_loss_final_kernel, dim3(1), dim3(kLossBlock), 0, st, partials, nb, loss_out);
}

extern "C" int diloco_sim_quadratic_loss_static(const float* theta, int M, int64_t n, int64_t stride,
                                                const float* h, const float* theta_star, double* loss_out,
                                                void* stream) {
    if (!theta || !h || !theta_star || !loss_out) return DILOCO_ERR_NULL;
    if (int e = check_shape(M, n, stride)) return e;
    if (n > DILOCO_SIM_STATIC_LOSS_MAX_N) return DILOCO_ERR_SHAPE;
    if (!aligned_to(theta, 4) || !aligned_to(h, 4) || !aligned_to(theta_star, 4) || !aligned_to(loss_out, 8))
        return DILOCO_ERR_ALIGN;
    Range r[4] = {{theta, extent_bytes(M, n, stride, 4), false},
                  {h, n * 4, false},
                  {theta_star, n * 4, false},
                  {loss_out, 8, true}};
    if (int e = check_alias(r, 4)) return e;
    double* partials = nullptr;
    if (int e = static_loss_scratch(&partials)) return e;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nb = loss_blocks(n);  // <= kLossMaxBlocks, the array's length; every slot read is written first
    if (int e = launch(quadratic_loss_partial_kernel, dim3((unsigned)nb), dim3(kLossBlock), 0, st, theta, M, n,
                       stride, h, theta_star, partials, 1.0 / M))
        return e;
    return launch(quadratic_loss_final_kernel, dim3(1), dim3(kLossBlock), 0, st, partials, nb, loss_out);
}

extern "C" int diloco_sim_stream_copy(float* dst, const float* src, int64_t n, void* stream,
                                      const diloco_launch* launch_arg) {
    Tuning t;
    if (!resolve_launch(launch_arg, t)) return DILOCO_ERR_HYPER;
    if (!dst || !src) return DILOCO_ERR_NULL;
    if (n < 0 || n > ((int64_t)1 << 60)) return DILOCO_ERR_SHAPE;
    if (!aligned_to(dst, 16) || !aligned_to(src, 16)) return DILOCO_ERR_ALIGN;
    Range r[2] = {{dst, n * 4, true}, {src, n * 4, false}};
    if (int e = check_alias(r, 2)) return e;
    if (n == 0) return DILOCO_OK;
    const Shape shape = launch_shape(t, 64 * 16, kInFlightTarget);  // one load a lane: never throttled by itself
    const int block = shape.block;
    const int64_t threads = (n >> 2) + ((n & 3) ? 1 : 0);
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    if (!grant_lds(&stream_copy_kernel, shape.lds)) return DILOCO_ERR_LAUNCH;
    return launch(stream_copy_kernel, dim3(g.blocks), dim3(block), shape.lds, static_cast<hipStream_t>(stream), dst,
                  src, n, g.per_xcd);
}

extern "C" int diloco_sim_stream_rmw(float* base, int K, int64_t n, int64_t stride, void* stream,
                                     const diloco_launch* launch_arg) {
    return diloco_sim_stream_sweep(base, K, n, stride, DILOCO_SIM_SWEEP_RMW, 0.f, stream, launch_arg);
}

extern "C" int diloco_sim_stream_sweep(float* base, int K, int64_t n, int64_t stride, int mode, float fill,
                                       void* stream, const diloco_launch* launch_arg) {
    Tuning t;
    if (!resolve_launch(launch_arg, t)) return DILOCO_ERR_HYPER;
    if (mode != DILOCO_SIM_SWEEP_RMW && mode != DILOCO_SIM_SWEEP_READ && mode != DILOCO_SIM_SWEEP_WRITE)
        return DILOCO_ERR_DTYPE;
    if (!base) return DILOCO_ERR_NULL;
    if (n < 0 || (n & 3) || stride < n || K < 1) return DILOCO_ERR_SHAPE;
    if (stride > ((int64_t)1 << 50) / K) return DILOCO_ERR_SHAPE;
    if (!aligned_to(base, 16) || (K > 1 && stride % 4 != 0)) return DILOCO_ERR_ALIGN;
    if (n == 0) return DILOCO_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (K) {
        case 1: return launch_sweep<1>(base, stride, n, mode, fill, st, t);
        case 2: return launch_sweep<2>(base, stride, n, mode, fill, st, t);
        case 4: return launch_sweep<4>(base, stride, n, mode, fill, st, t);
        case 5: return launch_sweep<5>(base, stride, n, mode, fill, st, t);
        case 8: return launch_sweep<8>(base, stride, n, mode, fill, st, t);
        case 9: return launch_sweep<9>(base, stride, n, mode, fill, st, t);
        case 16: return launch_sweep<16>(base, stride, n, mode, fill, st, t);
        case 17: return launch_sweep<17>(base, stride, n, mode, fill, st, t);
        case 33: return launch_sweep<33>(base, stride, n, mode, fill, st, t);
        default: return DILOCO_ERR_SHAPE;
    }
}

// ---------------------------------------------------------------- streaming schedule (host only)
static bool stream_args_ok(int64_t t, int64_t H, int F, int f) {
    return H >= 1 && F >= 1 && f >= 0 && f < F && t >= 0 && H <= ((int64_t)1 << 40);
}
extern "C" int64_t diloco_stream_offset(int64_t H, int F, int f) {
    if (!stream_args_ok(0, H, F, f)) return -1;
    return ((int64_t)f * H) / F;
}
extern "C" int diloco_stream_due(int64_t t, int64_t H, int F, int f) {
    if (!stream_args_ok(t, H, F, f)) return -1;
    return (t >= 1 && t % H == diloco_stream_offset(H, F, f)) ? 1 : 0;
}
extern "C" int64_t diloco_stream_boundary_count(int64_t t, int64_t H, int F, int f) {
    if (!stream_args_ok(t, H, F, f)) return -1;
    const int64_t off = diloco_stream_offset(H, F, f);
    // boundaries are off, off + H, off + 2H, ... restricted to steps >= 1
    if (off == 0) return t / H;
    return t < off ? 0 : (t - off) / H + 1;
}

extern "C" int diloco_tune(const char* key, int value) {
    if (!key) return DILOCO_ERR_NULL;
    Tuning t = tuning();
    if (!std::strcmp(key, "block"))
        t.block = value;
    else if (!std::strcmp(key, "xcd_remap"))
        t.xcd_remap = value;
    else if (!std::strcmp(key, "generic_path"))
        t.generic_path = value;
    else if (!std::strcmp(key, "wg_per_cu"))
        t.wg_per_cu = value;
    else
        return DILOCO_ERR_HYPER;
    if (!valid_tuning(t)) return DILOCO_ERR_HYPER;
    tuning() = t;
    return DILOCO_OK;
}

extern "C" int diloco_tune_get(const char* key) {
    if (!key) return -1;
    if (!std::strcmp(key, "block")) return tuning().block;
    if (!std::strcmp(key, "xcd_remap")) return tuning().xcd_remap;
    if (!std::strcmp(key, "generic_path")) return tuning().generic_path;
    if (!std::strcmp(key, "wg_per_cu")) return tuning().wg_per_cu;
    return -1;
}

extern "C" const char* diloco_strerror(int status) {
    switch (status) {
        case DILOCO_OK: return "ok";
        case DILOCO_ERR_NULL: return "a required pointer is NULL";
        case DILOCO_ERR_SHAPE: return "bad shape: M, n, stride or workspace size out of range";
        case DILOCO_ERR_ALIGN: return "a pointer or stride is not aligned as required";
        case DILOCO_ERR_DTYPE: return "unknown dtype or variant code";
        case DILOCO_ERR_HYPER: return "hyper-parameter out of range or not finite";
        case DILOCO_ERR_ALIAS: return "buffers overlap";
        case DILOCO_ERR_LAUNCH: return "the HIP runtime refused the launch";
        default: return "unknown status";
    }
}

extern "C" int diloco_version(void) { return 100; }

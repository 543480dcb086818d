// Shared device helpers and host-side argument checks for the DiLoCo sweep kernels (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>
#include <tuple>
#include <utility>

#include "diloco.h"
#include "diloco_sim.h"

namespace diloco {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf4 __attribute__((ext_vector_type(4)));

constexpr int kMaxBlock = 512;  // largest workgroup the streaming kernels are launched with
constexpr int kXcds = 8;  // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// ---------------------------------------------------------------- memory access
// Every byte of this path is touched once per call, so nothing is worth keeping in cache:
// loads carry the non-temporal hint, stores are non-temporal with device scope (`sc1 nt`),
// which this chip streams to HBM measurably faster than plain or `nt`-only stores
// (copy kernel 6.74 vs 6.57 vs 6.22 TB/s).  The compiler has no builtin that sets both bits
// on a 128-bit store, hence the asm statements; the "memory" clobber keeps every load of a
// thread ahead of its first store, which is the order the kernels want.  A store of more
// than 64 bits must be followed by a wait state before a VALU instruction may overwrite its
// data registers (CDNA3 ISA guide, manually inserted wait states); the compiler inserts it
// for its own stores but cannot see inside an asm statement, so the s_nop travels with it.
template <typename T> struct Vec4;
template <> struct Vec4<float> { using type = f4; };
template <> struct Vec4<__bf16> { using type = bf4; };

template <typename T>
__device__ __forceinline__ f4 load4(const T* p) {
    using V = typename Vec4<T>::type;
    V v = __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
    return __builtin_convertvector(v, f4);  // bf16 -> fp32 is exact
}
__device__ __forceinline__ void store4(float* p, f4 x) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store4(__bf16* p, f4 x) {
    typedef unsigned int u2 __attribute__((ext_vector_type(2)));
    bf4 v = __builtin_convertvector(x, bf4);  // fp32 -> bf16 rounds to nearest even
    u2 bits = __builtin_bit_cast(u2, v);
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(p), "v"(bits) : "memory");
}
template <typename T>
__device__ __forceinline__ float load1(const T* p) {
    return static_cast<float>(__builtin_nontemporal_load(p));
}
__device__ __forceinline__ void store1(float* p, float x) {
    asm volatile("global_store_dword %0, %1, off sc1 nt" : : "v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store1(__bf16* p, float x) {
    const unsigned int bits = __builtin_bit_cast(unsigned short, static_cast<__bf16>(x));
    asm volatile("global_store_short %0, %1, off sc1 nt" : : "v"(p), "v"(bits) : "memory");
}

// ---------------------------------------------------------------- fp32 math on 1 or 4 lanes
__device__ __forceinline__ float fma_(float a, float b, float c) { return fmaf(a, b, c); }
__device__ __forceinline__ f4 fma_(f4 a, f4 b, f4 c) { return __builtin_elementwise_fma(a, b, c); }
__device__ __forceinline__ float sqrt_(float x) { return sqrtf(x); }
__device__ __forceinline__ f4 sqrt_(f4 x) { return f4{sqrtf(x.x), sqrtf(x.y), sqrtf(x.z), sqrtf(x.w)}; }
template <typename T> __device__ __forceinline__ T splat(float x);
template <> __device__ __forceinline__ float splat<float>(float x) { return x; }
template <> __device__ __forceinline__ f4 splat<f4>(float x) { return f4{x, x, x, x}; }

// Logical workgroup index.  per_xcd == 0: identity.  Otherwise the grid holds 8*per_xcd
// workgroups and die k (hardware id % 8) walks the contiguous slice [k*per_xcd, (k+1)*per_xcd).
__device__ __forceinline__ int64_t logical_block(int64_t per_xcd) {
    int64_t b = blockIdx.x;
    if (per_xcd == 0) return b;
    return (b % kXcds) * per_xcd + b / kXcds;
}

// ---------------------------------------------------------------- host side
struct Tuning {
    int block = 0;         // threads per workgroup of the streaming kernels; 0: chosen per launch
    int xcd_remap = 0;
    int generic_path = 0;  // grouped eager kernel: 0 where no register instantiation exists, staging 40 replicas;
                           // 1 for every M, staging 80; 2 for every M, staging none
    int wg_per_cu = -1;    // most workgroups of a streaming kernel resident on a CU; 0: no cap, -1: chosen per launch
};
// The calling thread's launch shape (diloco_tune): what an entry point without an explicit shape uses.
Tuning& tuning();
// Range checks shared by diloco_tune and the explicit-shape entry points.
inline bool valid_block(int v) { return v == 0 || (v >= 64 && v <= kMaxBlock && (v & (v - 1)) == 0); }
inline bool valid_tuning(const Tuning& t) {
    return valid_block(t.block) && (t.xcd_remap == 0 || t.xcd_remap == 1) && t.generic_path >= 0 &&
           t.generic_path <= 2 && t.wg_per_cu >= -1 && t.wg_per_cu <= 32;
}
// The shape of a *_shaped call: the caller's struct, or the thread's shape for NULL.  false if a
// field is out of range.
inline bool resolve_launch(const diloco_launch* l, Tuning& out) {
    if (!l) {
        out = tuning();
        return true;
    }
    out.block = l->block;
    out.xcd_remap = l->xcd_remap;
    out.wg_per_cu = l->wg_per_cu;
    out.generic_path = l->generic_path;
    return valid_tuning(out);
}

constexpr int kLdsPerCu = 160 * 1024;  // gfx950

// Workgroup size and occupancy throttle of one launch.
//
// This chip's HBM pipeline is fastest with a few tens of KB of loads in flight per CU, and gets
// slower, not faster, with full occupancy (measured: AdamW 6.2 -> 6.6 TB/s, standard outer step
// 5.8 -> 6.4 TB/s at M = 8).  The throttle is dynamic LDS the kernel never touches, sized so that
// only `cap` workgroups fit a CU's 160 KB.  Left to itself (block 0, wg_per_cu -1) a launch uses
// one-wavefront workgroups and as many of them per CU as bring `target_bytes` of loads in flight,
// given that a wavefront issues `wave_load_bytes` before its first store (at least 2; from 4 up a
// multiple of 4, one SIMD's share each; no throttle from 32 up).  An explicit block size
// switches the throttle off unless wg_per_cu is set too.
struct Shape {
    int block;
    size_t lds;
};
// Loads in flight per CU at which the streaming sweeps measured fastest (eager step M = 1..8 fp32
// and bf16, standard step M = 1..64, AdamW): 30-50 KB.
constexpr int64_t kInFlightTarget = 36 * 1024;
// Smallest dynamic LDS size of which cap + 1 workgroups no longer fit a CU (0: no cap), so that at
// most `cap` are resident whatever the allocation granule.
inline size_t cap_lds_bytes(int cap) {
    if (cap <= 0) return 0;
    const size_t b = (size_t)kLdsPerCu / (size_t)(cap + 1) + 1;
    return (b + 255) & ~(size_t)255;
}
// even_simds = false keeps the computed cap as it is (AdamW: 9 one-wavefront workgroups per CU measured
// 1.2-1.9 % ahead of 8 and 0.8-2.4 % ahead of 10).
inline Shape launch_shape(const Tuning& t, int64_t wave_load_bytes, int64_t target_bytes, bool even_simds = true) {
    Shape s{t.block ? t.block : 64, 0};
    int cap = t.wg_per_cu;
    if (cap < 0) {
        cap = 0;
        if (!t.block) {
            cap = (int)((target_bytes + wave_load_bytes - 1) / wave_load_bytes);
            if (cap >= 4 && even_simds) cap = (cap + 2) / 4 * 4;  // the same number of wavefronts on each of the 4 SIMDs
            cap = cap < 2 ? 2 : (cap >= 32 ? 0 : cap);
        }
    }
    s.lds = cap_lds_bytes(cap);
    return s;
}
// Workgroup size of the kernels that take no throttle.
inline int plain_block(const Tuning& t) { return t.block ? t.block : 256; }
// More than 48 KB of dynamic LDS has to be granted per kernel, once: the largest size granted so
// far is remembered per kernel and device, so that a launch in steady state sets no attribute.
// false if the runtime refuses.
bool grant_lds_for(const void* kernel, size_t lds);
template <typename K>
inline bool grant_lds(K kernel, size_t lds) {
    return lds <= 48 * 1024 || grant_lds_for(reinterpret_cast<const void*>(kernel), lds);
}

struct Range {
    const void* p;
    int64_t bytes;
    bool written;
};

inline bool is_finite(double x) { return std::isfinite(x); }
inline bool in_unit(double x) { return std::isfinite(x) && x >= 0.0 && x < 1.0; }
inline int elem_size(int dtype) { return dtype == DILOCO_F32 ? 4 : 2; }
inline bool valid_dtype(int dtype) { return dtype == DILOCO_F32 || dtype == DILOCO_BF16; }

// [M][stride] buffer with n meaningful elements per row: bytes spanned from the base.
inline int64_t extent_bytes(int M, int64_t n, int64_t stride, int esize) {
    return ((int64_t)(M - 1) * stride + n) * esize;
}
// M, n, stride sanity incl. overflow of the largest element offset.
inline int check_shape(int M, int64_t n, int64_t stride) {
    if (M < 1 || M > DILOCO_MAX_REPLICAS || n < 0) return DILOCO_ERR_SHAPE;
    if (stride < n && M > 1) return DILOCO_ERR_SHAPE;
    if (stride < 0) return DILOCO_ERR_SHAPE;
    const int64_t lim = (int64_t)1 << 60;
    if (n > lim || stride > lim / M) return DILOCO_ERR_SHAPE;
    return DILOCO_OK;
}
inline bool aligned_to(const void* p, int a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int check_alias(const Range* r, int count) {
    for (int i = 0; i < count; ++i)
        for (int j = i + 1; j < count; ++j) {
            if (!r[i].p || !r[j].p || r[i].bytes == 0 || r[j].bytes == 0) continue;
            if (!r[i].written && !r[j].written) continue;
            const char* a0 = static_cast<const char*>(r[i].p);
            const char* b0 = static_cast<const char*>(r[j].p);
            if (a0 < b0 + r[j].bytes && b0 < a0 + r[i].bytes) return DILOCO_ERR_ALIAS;
        }
    return DILOCO_OK;
}

// Grid for `threads` work items, `block` threads per workgroup; per_xcd as logical_block wants it.
struct Grid {
    unsigned blocks;
    int64_t per_xcd;
};
inline Grid make_grid(const Tuning& t, int64_t threads, int block) {
    int64_t nb = (threads + block - 1) / block;
    Grid g;
    if (t.xcd_remap && nb >= 4 * kXcds) {
        g.per_xcd = (nb + kXcds - 1) / kXcds;
        g.blocks = (unsigned)(g.per_xcd * kXcds);
    } else {
        g.per_xcd = 0;
        g.blocks = (unsigned)nb;
    }
    return g;
}
// 2^31-1 workgroups per grid dimension.
inline bool grid_fits(int64_t threads, int block) {
    return (threads + block - 1) / block + kXcds < ((int64_t)1 << 31);
}

// Enqueues one kernel and reports the status of THIS launch: the thread's last-error slot is
// neither read nor cleared, so an unrelated earlier error is neither reported nor swallowed.
template <typename... KArgs, typename... Args, size_t... I>
inline int launch_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
                       std::index_sequence<I...>, Args&&... args) {
    std::tuple<KArgs...> vals(static_cast<KArgs>(std::forward<Args>(args))...);
    void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, st) == hipSuccess
               ? DILOCO_OK
               : DILOCO_ERR_LAUNCH;
}
template <typename... KArgs, typename... Args>
inline int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, Args&&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count does not match the kernel's");
    return launch_impl(kernel, grid, block, lds, st, std::index_sequence_for<KArgs...>{},
                       std::forward<Args>(args)...);
}

}  // namespace diloco

// Outer-step kernels: standard DiLoCo (Algorithm 1, lines 7-10), eager updates
// (Algorithm 3, lines 7-12), naive delayed outer gradients (Algorithm 2, lines 7-11)
// and the re-seeding of replicas from their outer parameters.
//
// One thread owns 4 consecutive parameters (one 128-bit access per fp32 stream) of ALL
// replicas, so the cross-replica mean is a register accumulation in the fixed order
// m = 0..M-1 with no cross-lane traffic.  The whole outer step is one read-modify-write
// pass: each byte of theta_m, the outer parameters, the velocity, the previous local
// and previous averaged outer gradient is read once and written once.
//
// The per-replica outer state (outer parameters a_m, velocity u_m, previous local outer
// gradient P_m) and the previous mean D are reached through a "state view":
//   RowState    the caller's [M][state_stride] rows and [n] mean;
//   TiledState  one library-defined buffer [tile][3M+1][8192 elements]: the 3M+1 state
//               streams of 8192 consecutive parameters sit next to each other, in the order
//               the kernel touches them (a_0..a_{M-1}, D, u_0, P_0, u_1, P_1, ...), so a
//               wavefront's 3M+1 state accesses fall into one or two 2 MB pages instead of
//               3M+1 pages that are gigabytes apart (fewer address-translation misses).
// Every kernel takes two views: `sv`, where the state is read, and `so`, where the new state is
// written.  They are the same buffer for the in-place entry points; the ping-pong entry point
// passes two packed buffers (a read-modify-write in place streams 1-2 % slower on this chip
// than the same sweep reading one buffer and writing another).
#include "common.hpp"

namespace diloco {

struct OuterScalars {
    float mu;        // outer momentum
    float c_g;       // coefficient of G in the parameter step: lr (Nesterov) or 0
    float c_u;       // coefficient of the new velocity: lr*mu (Nesterov) or lr
    float inv_M;     // 1/M in fp32 (eager combination)
    double inv_M_d;  // 1/M in fp64 (mean)
    int comm;        // wire format of the outer gradients (Section 3.2): COMM_F32 / COMM_BF16 / COMM_EXMY
    int q_mant;      // ExMy: mantissa bits
    int q_emin;      // ExMy: exponent of the spacing of the subnormals, 1 - bias - mantissa bits
    int q_bias;      // ExMy: exponent bias
    int no_mean;     // eager only: the previous mean is not kept; it is formed from the previous locals
    float q_max;     // ExMy: largest value of the format
};
enum { COMM_F32 = 0, COMM_BF16 = 1, COMM_EXMY = 2 };

// Nearest value of the small-float format, ties to the even code, saturating.  Around |d| the
// format's values are the multiples of q = 2^max(floor(log2|d|) - mantissa bits, q_emin); |d|/q is
// exact (a power-of-two scaling) and at most 2^(mantissa bits + 1), so rint() of it takes the
// rounding decision exactly as the definition does.  Rounding up into the next binade lands on a
// value of the format, or beyond q_max, where it saturates.  Without mantissa bits the parity of
// |d|/q says nothing about the code, so the one possible tie (1.5 q) looks at the exponent code.
__device__ __forceinline__ float round_exmy(float d, const OuterScalars& sc) {
    const float ax = __builtin_fabsf(d);
    const int k = (int)(__float_as_uint(ax) >> 23) - 127;
    int qe = k - sc.q_mant;
    qe = qe < sc.q_emin ? sc.q_emin : (qe > 126 ? 126 : qe);
    const float q = __uint_as_float((uint32_t)(qe + 127) << 23);
    const float iq = __uint_as_float((uint32_t)(127 - qe) << 23);
    const float t = ax * iq;
    float c = __builtin_rintf(t);
    if (sc.q_mant == 0 && t == 1.5f) c = ((qe + sc.q_bias) & 1) ? 2.f : 1.f;
    float r = c * q;
    r = r > sc.q_max ? sc.q_max : r;
    return __builtin_copysignf(r, d);
}

// What a replica sends into the all-reduce: Delta_m itself, or Delta_m rounded to the wire format.
__device__ __forceinline__ float sent(float d, const OuterScalars& sc) {
    if (sc.comm == COMM_F32) return d;
    if (sc.comm == COMM_BF16) return static_cast<float>(static_cast<__bf16>(d));
    return round_exmy(d, sc);
}
__device__ __forceinline__ f4 sent(f4 d, const OuterScalars& sc) {
    if (sc.comm == COMM_F32) return d;
    if (sc.comm == COMM_BF16) return __builtin_convertvector(__builtin_convertvector(d, bf4), f4);
    f4 r = {round_exmy(d.x, sc), round_exmy(d.y, sc), round_exmy(d.z, sc), round_exmy(d.w, sc)};
    return r;
}

enum { MODE_RECORD = 0, MODE_EAGER = 1, MODE_DELAYED = 2 };

constexpr int kMinStagedWaves = 2;     // replicas are staged in LDS only while this many wavefronts fit a CU
constexpr int kTileShift = 13;  // DILOCO_STATE_TILE = 8192 elements
constexpr int64_t kTile = (int64_t)1 << kTileShift;
static_assert(kTile == DILOCO_STATE_TILE, "header and kernels disagree on the state tile");

struct RowState {
    float* anchor;
    float* vel;
    float* P;
    float* D;
    int64_t ss;
    __device__ __forceinline__ float* a(int m, int64_t i) const { return anchor + m * ss + i; }
    __device__ __forceinline__ float* u(int m, int64_t i) const { return vel + m * ss + i; }
    __device__ __forceinline__ float* p(int m, int64_t i) const { return P + m * ss + i; }
    __device__ __forceinline__ float* d(int64_t i) const { return D + i; }
    __device__ __forceinline__ bool same_as(const RowState& o) const { return anchor == o.anchor; }
};

// `base` holds the outer parameters and velocities, `hist` the previous local and averaged outer
// gradients: one and the same buffer, except when the call reads the two from different
// generations of the state (2-outer-steps overlap).
struct TiledState {
    float* base;
    float* hist;
    int64_t M;  // replicas; streams per tile: 3M + 1
    __device__ __forceinline__ int64_t off(int64_t s, int64_t i) const {
        return (((i >> kTileShift) * (3 * M + 1) + s) << kTileShift) | (i & (kTile - 1));
    }
    __device__ __forceinline__ float* a(int m, int64_t i) const { return base + off(m, i); }
    __device__ __forceinline__ float* d(int64_t i) const { return hist + off(M, i); }
    __device__ __forceinline__ float* u(int m, int64_t i) const { return base + off(M + 1 + 2 * m, i); }
    __device__ __forceinline__ float* p(int m, int64_t i) const { return hist + off(M + 2 + 2 * m, i); }
    __device__ __forceinline__ bool same_as(const TiledState& o) const { return base == o.base; }
};

// OuterOpt on one value (or 4): u <- mu u + G ; a <- a - (c_g G + c_u u).
template <typename T>
__device__ __forceinline__ void outer_opt(T& a, T& u, T G, const OuterScalars& sc) {
    u = fma_(splat<T>(sc.mu), u, G);
    a = a - fma_(splat<T>(sc.c_u), u, sc.c_g * G);
}
// Algorithm 3 line 11: (Delta_m - Delta_m_prev)/M + Delta_prev.
template <typename T>
__device__ __forceinline__ T eager_gradient(T d, T p, T Dold, const OuterScalars& sc) {
    return fma_(d - p, splat<T>(sc.inv_M), Dold);
}

// ------------------------------------------------------------------ element-wise path
// Runtime M, one parameter index, two passes over the replicas (the second re-reads
// theta_m and a_m).  Serves misaligned buffers and the ragged tail of the vector kernels;
// same arithmetic, same order.
template <typename TT, int MODE, typename SV>
__device__ void eager_element(TT* theta, SV sv, SV so, int M, int64_t stride, int64_t i,
                              const OuterScalars& sc) {
    double s = 0.0;
    for (int m = 0; m < M; ++m) {
        float a = load1(sv.a(m, i));
        float th = load1(theta + m * stride + i);
        s += (double)sent(a - th, sc);
    }
    const float dbar = (float)(s * sc.inv_M_d);
    float Dold = 0.f;
    if (MODE == MODE_EAGER && sc.no_mean) {
        double t = 0.0;
        for (int m = 0; m < M; ++m) t += (double)load1(sv.p(m, i));
        Dold = (float)(t * sc.inv_M_d);
    } else if (MODE != MODE_RECORD) {
        Dold = load1(sv.d(i));
    }
    for (int m = 0; m < M; ++m) {
        float a = load1(sv.a(m, i));
        float th = load1(theta + m * stride + i);
        float d = a - th;
        if (MODE == MODE_RECORD) {
            store1(so.a(m, i), th);
            if (!sv.same_as(so)) store1(so.u(m, i), load1(sv.u(m, i)));  // the velocity moves along unchanged
        } else {
            float u = load1(sv.u(m, i));
            float G = Dold;
            if (MODE == MODE_EAGER) G = eager_gradient(d, load1(sv.p(m, i)), Dold, sc);
            outer_opt(a, u, G, sc);
            store1(theta + m * stride + i, a);
            store1(so.a(m, i), a);
            store1(so.u(m, i), u);
        }
        store1(so.p(m, i), sent(d, sc));
    }
    if (!sc.no_mean) store1(so.d(i), dbar);
}

template <typename TT, int MODE, typename SV>
__global__ __launch_bounds__(kMaxBlock) void outer_eager_scalar_kernel(TT* theta, SV sv, SV so, int M, int64_t n,
                                                                       int64_t stride, OuterScalars sc,
                                                                       int64_t per_xcd) {
    int64_t i = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    if (i < n) eager_element<TT, MODE, SV>(theta, sv, so, M, stride, i, sc);
}

// Tail of a vector kernel: the thread right after the last full vector sweeps n % 4 elements.
template <typename TT, int MODE, typename SV>
__device__ __forceinline__ void eager_tail(TT* theta, SV sv, SV so, int M, int64_t n, int64_t stride,
                                           const OuterScalars& sc) {
    for (int64_t i = n & ~(int64_t)3; i < n; ++i) eager_element<TT, MODE, SV>(theta, sv, so, M, stride, i, sc);
}

// ------------------------------------------------------------------ register path
// M known at compile time: a_m and Delta_m of all replicas stay in registers between the
// reduction and the update (2*M*4 VGPRs), nothing is read twice.
template <int M, typename TT, int MODE, typename SV>
__global__ __launch_bounds__(kMaxBlock) void outer_eager_reg_kernel(TT* __restrict__ theta, SV sv, SV so, int64_t n,
                                                                    int64_t stride, OuterScalars sc,
                                                                    int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    if (v >= nvec) {
        if (v == nvec) eager_tail<TT, MODE, SV>(theta, sv, so, M, n, stride, sc);
        return;
    }
    const int64_t i = v << 2;
    f4 a[M], d[M], u[M], p[M];
    f4 Dold = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < M; ++m) {
        a[m] = load4(sv.a(m, i));
        d[m] = load4(theta + m * stride + i);  // theta for now
    }
    const bool form_mean = MODE == MODE_EAGER && sc.no_mean;  // the previous mean from the previous locals
    if (MODE != MODE_RECORD) {
        if (!form_mean) Dold = load4(sv.d(i));
#pragma unroll
        for (int m = 0; m < M; ++m) {
            u[m] = load4(sv.u(m, i));
            if (MODE == MODE_EAGER) p[m] = load4(sv.p(m, i));
        }
    }
    if (form_mean) {  // the sum the previous call took, in its order: the same bits it would have stored
        double t0 = 0.0, t1 = 0.0, t2 = 0.0, t3 = 0.0;
#pragma unroll
        for (int m = 0; m < M; ++m) {
            t0 += (double)p[m].x;
            t1 += (double)p[m].y;
            t2 += (double)p[m].z;
            t3 += (double)p[m].w;
        }
        Dold = f4{(float)(t0 * sc.inv_M_d), (float)(t1 * sc.inv_M_d), (float)(t2 * sc.inv_M_d),
                  (float)(t3 * sc.inv_M_d)};
    }
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    f4 th[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        th[m] = d[m];
        d[m] = a[m] - th[m];
        const f4 q = sent(d[m], sc);
        s0 += (double)q.x;
        s1 += (double)q.y;
        s2 += (double)q.z;
        s3 += (double)q.w;
    }
    f4 dbar = {(float)(s0 * sc.inv_M_d), (float)(s1 * sc.inv_M_d), (float)(s2 * sc.inv_M_d),
               (float)(s3 * sc.inv_M_d)};
    // Stores leave in address order: the theta rows, then the state streams as the packed
    // layout holds them (a_0..a_{M-1}, D, u_0, P_0, u_1, ...).  Against stores interleaved per
    // replica this measured between equal and 6 % faster on t550m, depending on where the
    // buffers happen to lie in memory; it was never slower.
    if (MODE == MODE_RECORD) {
        const bool carry = !sv.same_as(so);  // another buffer: the velocity moves along unchanged
        if (carry) {
#pragma unroll
            for (int m = 0; m < M; ++m) u[m] = load4(sv.u(m, i));
        }
#pragma unroll
        for (int m = 0; m < M; ++m) store4(so.a(m, i), th[m]);
        if (!sc.no_mean) store4(so.d(i), dbar);
#pragma unroll
        for (int m = 0; m < M; ++m) {
            if (carry) store4(so.u(m, i), u[m]);
            store4(so.p(m, i), sent(d[m], sc));
        }
        return;
    }
#pragma unroll
    for (int m = 0; m < M; ++m) {
        f4 G = Dold;
        if (MODE == MODE_EAGER) G = eager_gradient(d[m], p[m], Dold, sc);
        outer_opt(a[m], u[m], G, sc);
    }
#pragma unroll
    for (int m = 0; m < M; ++m) store4(theta + m * stride + i, a[m]);
#pragma unroll
    for (int m = 0; m < M; ++m) store4(so.a(m, i), a[m]);
    if (!sc.no_mean) store4(so.d(i), dbar);
#pragma unroll
    for (int m = 0; m < M; ++m) {
        store4(so.u(m, i), u[m]);
        store4(so.p(m, i), sent(d[m], sc));
    }
}

// ------------------------------------------------------------------ any M: replicas in groups
// For replica counts without a register instantiation the sweep walks the replicas in groups of
// kGroup, every group's loads issued together (a wavefront that waits for one replica at a time
// needs far more resident wavefronts than the staging leaves room for).  Sum and update keep the
// order m = 0, 1, ... of the register kernel: same bits.
constexpr int kGroup = 8;

// First pass over one group: Delta_m = a_m - theta_m into the running sum; with LDS staging the
// values the second pass needs are parked (a_m, or theta_m when only recording, and Delta_m).
// NOMEAN (eager step without a stored mean): the previous local outer gradients are read here as
// well, summed into t0..t3 in replica order, and parked with the others (a third slot).
template <typename TT, int MODE, typename SV, bool FULL, bool STAGE, bool NOMEAN>
__device__ __forceinline__ void group_reduce(const TT* __restrict__ theta, const SV& sv, int m0, int cnt,
                                             int64_t i, int64_t stride, const OuterScalars& sc, f4* stage,
                                             int tid, double (&s)[4], double (&t)[4]) {
    constexpr int kSlots = NOMEAN ? 3 : 2;
    f4 a[kGroup], th[kGroup], p[kGroup];
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
        if (FULL || j < cnt) {
            a[j] = load4(sv.a(m0 + j, i));
            th[j] = load4(theta + (m0 + j) * stride + i);
            if (NOMEAN) p[j] = load4(sv.p(m0 + j, i));
        }
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
        if (FULL || j < cnt) {
            const f4 d = a[j] - th[j];
            const f4 q = sent(d, sc);
            s[0] += (double)q.x;
            s[1] += (double)q.y;
            s[2] += (double)q.z;
            s[3] += (double)q.w;
            if (NOMEAN) {
                t[0] += (double)p[j].x;
                t[1] += (double)p[j].y;
                t[2] += (double)p[j].z;
                t[3] += (double)p[j].w;
            }
            if (STAGE) {
                stage[(kSlots * (m0 + j)) * 64 + tid] = (MODE == MODE_RECORD) ? th[j] : a[j];
                stage[(kSlots * (m0 + j) + 1) * 64 + tid] = d;
                if (NOMEAN) stage[(kSlots * (m0 + j) + 2) * 64 + tid] = p[j];
            }
        }
}

// Second pass over one group.  STAGE: a_m (theta_m) and Delta_m (and, NOMEAN, the previous local
// outer gradient) come back from LDS; otherwise they are read again.
template <typename TT, int MODE, typename SV, bool FULL, bool STAGE, bool NOMEAN>
__device__ __forceinline__ void group_update(TT* __restrict__ theta, const SV& sv, const SV& so, int m0, int cnt,
                                             int64_t i, int64_t stride, const OuterScalars& sc, const f4* stage,
                                             int tid, f4 Dold) {
    constexpr int kSlots = NOMEAN ? 3 : 2;
    f4 a[kGroup], d[kGroup], u[kGroup], p[kGroup];
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
        if (FULL || j < cnt) {
            if (!STAGE) {
                a[j] = load4(sv.a(m0 + j, i));
                d[j] = load4(theta + (m0 + j) * stride + i);  // theta for now
            }
            if (MODE != MODE_RECORD || !sv.same_as(so)) u[j] = load4(sv.u(m0 + j, i));
            if (MODE == MODE_EAGER && !(STAGE && NOMEAN)) p[j] = load4(sv.p(m0 + j, i));
        }
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
        if (FULL || j < cnt) {
            if (STAGE) {
                a[j] = stage[(kSlots * (m0 + j)) * 64 + tid];  // theta_m when only recording
                d[j] = stage[(kSlots * (m0 + j) + 1) * 64 + tid];
                if (NOMEAN) p[j] = stage[(kSlots * (m0 + j) + 2) * 64 + tid];
            } else {
                const f4 th = d[j];
                d[j] = a[j] - th;
                if (MODE == MODE_RECORD) a[j] = th;
            }
            if (MODE != MODE_RECORD) {
                f4 G = Dold;
                if (MODE == MODE_EAGER) G = eager_gradient(d[j], p[j], Dold, sc);
                outer_opt(a[j], u[j], G, sc);
            }
        }
    if (MODE != MODE_RECORD) {
#pragma unroll
        for (int j = 0; j < kGroup; ++j)
            if (FULL || j < cnt) store4(theta + (m0 + j) * stride + i, a[j]);
    }
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
        if (FULL || j < cnt) store4(so.a(m0 + j, i), a[j]);
#pragma unroll
    for (int j = 0; j < kGroup; ++j)
        if (FULL || j < cnt) {
            if (MODE != MODE_RECORD || !sv.same_as(so)) store4(so.u(m0 + j, i), u[j]);  // recording: moved along
            store4(so.p(m0 + j, i), sent(d[j], sc));
        }
}

// The first `staged` replicas (a multiple of kGroup, or all M) keep a_m and Delta_m in LDS between
// the passes (32 bytes per lane and replica, 48 with NOMEAN; a lane only reads back what it wrote
// itself, so no barrier); for the others the second pass re-reads theta_m and a_m (2 of their 8
// accesses per index happen twice; with NOMEAN the previous local outer gradient as well).  One
// wavefront per workgroup.  NOMEAN is the eager step without a stored mean (MODE_EAGER only): the
// previous mean is the fp64 sum of the previous locals in replica order, rounded once, and the
// mean stream is neither read nor written (recording without a stored mean only skips the store).
template <typename TT, int MODE, typename SV, bool NOMEAN>
__global__ __launch_bounds__(64) void outer_eager_grouped_kernel(TT* __restrict__ theta, SV sv, SV so, int M,
                                                                 int staged, int64_t n, int64_t stride,
                                                                 OuterScalars sc, int64_t per_xcd) {
    static_assert(!NOMEAN || MODE == MODE_EAGER, "only the eager combination forms the previous mean itself");
    extern __shared__ f4 stage[];  // [staged][2 or 3][64]
    const int64_t v = logical_block(per_xcd) * 64 + threadIdx.x;
    const int64_t nvec = n >> 2;
    if (v >= nvec) {
        if (v == nvec) eager_tail<TT, MODE, SV>(theta, sv, so, M, n, stride, sc);
        return;
    }
    const int64_t i = v << 2;
    const int tid = threadIdx.x;
    double s[4] = {0.0, 0.0, 0.0, 0.0}, t[4] = {0.0, 0.0, 0.0, 0.0};
    int m0 = 0;
    for (; m0 + kGroup <= M; m0 += kGroup) {
        if (m0 < staged)
            group_reduce<TT, MODE, SV, true, true, NOMEAN>(theta, sv, m0, kGroup, i, stride, sc, stage, tid, s, t);
        else
            group_reduce<TT, MODE, SV, true, false, NOMEAN>(theta, sv, m0, kGroup, i, stride, sc, stage, tid, s, t);
    }
    if (m0 < M) {
        if (m0 < staged)
            group_reduce<TT, MODE, SV, false, true, NOMEAN>(theta, sv, m0, M - m0, i, stride, sc, stage, tid, s, t);
        else
            group_reduce<TT, MODE, SV, false, false, NOMEAN>(theta, sv, m0, M - m0, i, stride, sc, stage, tid, s, t);
    }
    f4 dbar = {(float)(s[0] * sc.inv_M_d), (float)(s[1] * sc.inv_M_d), (float)(s[2] * sc.inv_M_d),
               (float)(s[3] * sc.inv_M_d)};
    f4 Dold = {0.f, 0.f, 0.f, 0.f};
    if (NOMEAN)
        Dold = f4{(float)(t[0] * sc.inv_M_d), (float)(t[1] * sc.inv_M_d), (float)(t[2] * sc.inv_M_d),
                  (float)(t[3] * sc.inv_M_d)};
    else if (MODE != MODE_RECORD)
        Dold = load4(sv.d(i));
    for (m0 = 0; m0 + kGroup <= M; m0 += kGroup) {
        if (m0 < staged)
            group_update<TT, MODE, SV, true, true, NOMEAN>(theta, sv, so, m0, kGroup, i, stride, sc, stage, tid, Dold);
        else
            group_update<TT, MODE, SV, true, false, NOMEAN>(theta, sv, so, m0, kGroup, i, stride, sc, stage, tid, Dold);
    }
    if (m0 < M) {
        if (m0 < staged)
            group_update<TT, MODE, SV, false, true, NOMEAN>(theta, sv, so, m0, M - m0, i, stride, sc, stage, tid, Dold);
        else
            group_update<TT, MODE, SV, false, false, NOMEAN>(theta, sv, so, m0, M - m0, i, stride, sc, stage, tid, Dold);
    }
    if (!sc.no_mean) store4(so.d(i), dbar);
}

// ------------------------------------------------------------------ standard DiLoCo
// Shared outer parameters: nothing per replica has to survive the reduction, so any M runs
// through one kernel, the replicas in groups of kGroup.
// K consecutive replicas' theta at one index: all K loads first, then the sum in replica order.
template <int K, typename TT>
__device__ __forceinline__ void sync_group(const TT* __restrict__ th0, int64_t stride, f4 a, const OuterScalars& sc,
                                           double& s0, double& s1, double& s2, double& s3) {
    static_assert(K <= kGroup, "group too large");
    f4 th[K];
#pragma unroll
    for (int j = 0; j < K; ++j) th[j] = load4(th0 + j * stride);
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const f4 d = sent(a - th[j], sc);
        s0 += (double)d.x;
        s1 += (double)d.y;
        s2 += (double)d.z;
        s3 += (double)d.w;
    }
}

template <typename TT>
__global__ __launch_bounds__(kMaxBlock) void outer_sync_vec_kernel(TT* __restrict__ theta, float* __restrict__ anchor,
                                                                   float* __restrict__ vel,
                                                                   float* __restrict__ mean_out, int M, int64_t n,
                                                                   int64_t stride, OuterScalars sc,
                                                                   int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    if (v > nvec) return;
    if (v == nvec) {
        for (int64_t i = n & ~(int64_t)3; i < n; ++i) {
            float a = load1(anchor + i), u = load1(vel + i);
            double s = 0.0;
            for (int m = 0; m < M; ++m) s += (double)sent(a - load1(theta + m * stride + i), sc);
            float dbar = (float)(s * sc.inv_M_d);
            outer_opt(a, u, dbar, sc);
            for (int m = 0; m < M; ++m) store1(theta + m * stride + i, a);
            store1(anchor + i, a);
            store1(vel + i, u);
            if (mean_out) store1(mean_out + i, dbar);
        }
        return;
    }
    const int64_t i = v << 2;
    f4 a = load4(anchor + i), u = load4(vel + i);
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    // replicas in groups of kGroup, a group's loads issued together; the sum runs over m = 0, 1, ...
    int m0 = 0;
    for (; m0 + kGroup <= M; m0 += kGroup) sync_group<kGroup>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3);
    switch (M - m0) {
        case 1: sync_group<1>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        case 2: sync_group<2>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        case 3: sync_group<3>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        case 4: sync_group<4>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        case 5: sync_group<5>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        case 6: sync_group<6>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        case 7: sync_group<7>(theta + m0 * stride + i, stride, a, sc, s0, s1, s2, s3); break;
        default: break;
    }
    f4 dbar = {(float)(s0 * sc.inv_M_d), (float)(s1 * sc.inv_M_d), (float)(s2 * sc.inv_M_d),
               (float)(s3 * sc.inv_M_d)};
    outer_opt(a, u, dbar, sc);
    for (int m = 0; m < M; ++m) store4(theta + m * stride + i, a);
    store4(anchor + i, a);
    store4(vel + i, u);
    if (mean_out) store4(mean_out + i, dbar);
}

template <typename TT>
__global__ __launch_bounds__(kMaxBlock) void outer_sync_scalar_kernel(TT* theta, float* anchor, float* vel,
                                                                      float* mean_out, int M, int64_t n,
                                                                      int64_t stride, OuterScalars sc,
                                                                      int64_t per_xcd) {
    const int64_t i = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float a = load1(anchor + i), u = load1(vel + i);
    double s = 0.0;
    for (int m = 0; m < M; ++m) s += (double)sent(a - load1(theta + m * stride + i), sc);
    float dbar = (float)(s * sc.inv_M_d);
    outer_opt(a, u, dbar, sc);
    for (int m = 0; m < M; ++m) store1(theta + m * stride + i, a);
    store1(anchor + i, a);
    store1(vel + i, u);
    if (mean_out) store1(mean_out + i, dbar);
}

// ------------------------------------------------------------------ reset (grid.y = replica)
struct RowAnchor {
    const float* anchor;
    int64_t as;  // 0: one shared row
    __device__ __forceinline__ const float* a(int m, int64_t i) const { return anchor + m * as + i; }
};
struct TiledAnchor {
    const float* base;
    int64_t S;  // streams per tile: 3M + 1
    __device__ __forceinline__ const float* a(int m, int64_t i) const {
        return base + ((((i >> kTileShift) * S + m) << kTileShift) | (i & (kTile - 1)));
    }
};

template <typename TT, typename AV>
__global__ __launch_bounds__(kMaxBlock) void reset_vec_kernel(TT* __restrict__ theta, AV av, int64_t n,
                                                              int64_t stride, int64_t per_xcd) {
    const int64_t v = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int64_t nvec = n >> 2;
    const int m = blockIdx.y;
    if (v > nvec) return;
    if (v == nvec) {
        for (int64_t i = n & ~(int64_t)3; i < n; ++i) store1(theta + m * stride + i, load1(av.a(m, i)));
        return;
    }
    const int64_t i = v << 2;
    store4(theta + m * stride + i, load4(av.a(m, i)));
}
template <typename TT, typename AV>
__global__ __launch_bounds__(kMaxBlock) void reset_scalar_kernel(TT* theta, AV av, int64_t n, int64_t stride,
                                                                 int64_t per_xcd) {
    const int64_t i = logical_block(per_xcd) * blockDim.x + threadIdx.x;
    const int m = blockIdx.y;
    if (i < n) store1(theta + m * stride + i, load1(av.a(m, i)));
}

// ------------------------------------------------------------------ rows <-> tiled state
// grid.y = state stream s (m < M: a_m; M: D; M+1+2m: u_m; M+2+2m: P_m).  TO_TILED: rows -> tiled.
// A NULL row buffer skips its streams.  VEC = 4 or 1.
template <bool TO_TILED, int VEC>
__global__ __launch_bounds__(kMaxBlock) void repack_kernel(float* tiled, float* anchor, float* vel, float* P,
                                                           float* D, int M, int64_t n, int64_t ss,
                                                           int64_t per_xcd) {
    const int64_t e = (logical_block(per_xcd) * blockDim.x + threadIdx.x) * VEC;
    if (e >= n) return;
    const int s = blockIdx.y;
    const int64_t S = 3 * M + 1;
    float* row;
    if (s < M) {
        row = anchor ? anchor + s * ss : nullptr;
    } else if (s == M) {
        row = D;
    } else {
        const int k = s - M - 1, m = k >> 1;
        float* b = (k & 1) ? P : vel;
        row = b ? b + m * ss : nullptr;
    }
    if (!row) return;
    float* t = tiled + ((((e >> kTileShift) * S + s) << kTileShift) | (e & (kTile - 1)));
    if (VEC == 4 && e + 4 <= n) {
        if (TO_TILED)
            store4(t, load4(row + e));
        else
            store4(row + e, load4(t));
    } else {
        for (int64_t j = 0; j < VEC && e + j < n; ++j) {
            if (TO_TILED)
                t[j] = row[e + j];
            else
                row[e + j] = t[j];
        }
    }
}

// ------------------------------------------------------------------ host dispatch
// Wire format out of the bits OR-ed into `variant` (DILOCO_COMM_BF16 / DILOCO_COMM_EXMY); false if
// they name no format this library computes.
static bool parse_comm(int variant, OuterScalars& sc) {
    sc.comm = COMM_F32;
    sc.q_mant = sc.q_emin = sc.q_bias = 0;
    sc.no_mean = 0;
    sc.q_max = 0.f;
    const bool bf16 = variant & DILOCO_COMM_BF16, exmy = variant & 0x200;
    if (bf16 && exmy) return false;
    if (bf16) sc.comm = COMM_BF16;
    if (!exmy) return (variant & ~0x1ff) == 0;
    const int E = (variant >> 12) & 0xf, Mn = (variant >> 16) & 0xf;
    const int bias = (int)(int8_t)((variant >> 20) & 0xff);
    if ((variant & ~0x0ffff3ff) != 0 || E < 1 || E > 8 || Mn > 10 || E + Mn > 15) return false;
    const int emax = (1 << E) - 1 - bias, emin_q = 1 - bias - Mn;
    if (emax > 127 || emin_q < -126) return false;
    sc.comm = COMM_EXMY;
    sc.q_mant = Mn;
    sc.q_emin = emin_q;
    sc.q_bias = bias;
    sc.q_max = (float)std::ldexp(2.0 - std::ldexp(1.0, -Mn), emax);
    return true;
}

static OuterScalars make_scalars(int M, double lr, double mu, int nesterov) {
    OuterScalars sc;
    sc.comm = COMM_F32;
    sc.q_mant = sc.q_emin = sc.q_bias = 0;
    sc.no_mean = 0;
    sc.q_max = 0.f;
    sc.mu = (float)mu;
    sc.c_g = nesterov ? (float)lr : 0.f;
    sc.c_u = nesterov ? (float)(lr * mu) : (float)lr;
    sc.inv_M = (float)(1.0 / M);
    sc.inv_M_d = 1.0 / M;
    return sc;
}

template <typename TT, int MODE, typename SV>
static int launch_eager(TT* theta, SV sv, SV so, int M, int64_t n, int64_t stride, const OuterScalars& sc,
                        bool vec_ok, hipStream_t st, const Tuning& t) {
    // a wavefront of the vector kernels loads theta_m, a_m, u_m, P_m of every replica and D: 16 B a lane each
    const Shape shape =
        launch_shape(t, (int64_t)64 * ((3 * M + 1) * 16 + M * 4 * (int64_t)sizeof(TT)), kInFlightTarget);
    const int block = shape.block;
    if (!vec_ok) {
        if (!grid_fits(n, block)) return DILOCO_ERR_SHAPE;
        Grid g = make_grid(t, n, block);
        return launch(outer_eager_scalar_kernel<TT, MODE, SV>, dim3(g.blocks), dim3(block), 0, st, theta, sv, so, M,
                      n, stride, sc, g.per_xcd);
    }
    const int64_t threads = (n >> 2) + ((n & 3) ? 1 : 0);
    if (!grid_fits(threads, 64)) return DILOCO_ERR_SHAPE;
#define DILOCO_REG_CASE(MM)                                                                             \
    case MM: {                                                                                          \
        Grid g = make_grid(t, threads, block);                                                          \
        if (!grant_lds(&outer_eager_reg_kernel<MM, TT, MODE, SV>, shape.lds)) return DILOCO_ERR_LAUNCH; \
        return launch(outer_eager_reg_kernel<MM, TT, MODE, SV>, dim3(g.blocks), dim3(block), shape.lds, st, theta,  \
                      sv, so, n, stride, sc, g.per_xcd);                                                \
    }
    // a forced generic path also replaces the register kernels
    switch (t.generic_path ? 0 : M) {
        DILOCO_REG_CASE(1)
        DILOCO_REG_CASE(2)
        DILOCO_REG_CASE(3)
        DILOCO_REG_CASE(4)
        DILOCO_REG_CASE(5)
        DILOCO_REG_CASE(6)
        DILOCO_REG_CASE(7)
        DILOCO_REG_CASE(8)
        default: break;
    }
#undef DILOCO_REG_CASE
    // Other M: the grouped kernel, one wavefront per workgroup.  It stages as many replicas in LDS
    // (2 KB each per workgroup, 3 KB when the previous mean is formed from the previous locals) as
    // leave room for kMinStagedWaves workgroups on a CU's 160 KB: all of them up to M = 40 (26), the
    // first 40 (24) beyond; the rest are read twice.  generic_path 1 stages all that one workgroup
    // per CU can hold (80 / 53), 2 stages none.  The kernel's 256 VGPRs and the staging already keep
    // it to 4 workgroups per CU or fewer; left to itself a launch that stages nothing is capped at 2.
    // Measured, of algorithmic bytes: 6.2-6.6 TB/s fully staged (M <= 40), 6.2 / 5.8 / 5.6 at
    // M = 48 / 64 / 80, 5.3-5.8 unstaged.  A cap may ask for more LDS than the staging needs, never less.
    constexpr bool kNoMeanKernel = MODE == MODE_EAGER;
    const bool nomean = kNoMeanKernel && sc.no_mean;
    const int per_replica = 64 * 16 * (nomean ? 3 : 2);
    const int room = t.generic_path == 2 ? 0 : kLdsPerCu / per_replica / (t.generic_path == 1 ? 1 : kMinStagedWaves);
    const int staged = M <= room ? M : room / kGroup * kGroup;
    const int64_t need = (int64_t)per_replica * staged;
    const int cap = t.wg_per_cu >= 0 ? t.wg_per_cu : (staged ? 0 : 2);
    const int64_t cap_lds = (int64_t)cap_lds_bytes(cap);
    const size_t lds = (size_t)(need > cap_lds ? need : cap_lds);
    Grid g = make_grid(t, threads, 64);
    if (nomean) {
        // only instantiated for the eager mode (the others never form the previous mean)
        auto kernel = outer_eager_grouped_kernel<TT, kNoMeanKernel ? MODE : MODE_EAGER, SV, true>;
        if (!grant_lds(kernel, lds)) return DILOCO_ERR_LAUNCH;
        return launch(kernel, dim3(g.blocks), dim3(64), lds, st, theta, sv, so, M, staged, n, stride, sc, g.per_xcd);
    }
    if (!grant_lds(&outer_eager_grouped_kernel<TT, MODE, SV, false>, lds)) return DILOCO_ERR_LAUNCH;
    return launch(outer_eager_grouped_kernel<TT, MODE, SV, false>, dim3(g.blocks), dim3(64), lds, st, theta, sv, so,
                  M, staged, n, stride, sc, g.per_xcd);
}

template <typename TT, typename SV>
static int dispatch_eager(void* theta, SV sv, SV so, int M, int64_t n, int64_t stride, const OuterScalars& sc,
                          bool vec_ok, int mode, hipStream_t st, const Tuning& t) {
    TT* th = static_cast<TT*>(theta);
    switch (mode) {
        case MODE_RECORD: return launch_eager<TT, MODE_RECORD, SV>(th, sv, so, M, n, stride, sc, vec_ok, st, t);
        case MODE_EAGER: return launch_eager<TT, MODE_EAGER, SV>(th, sv, so, M, n, stride, sc, vec_ok, st, t);
        default: return launch_eager<TT, MODE_DELAYED, SV>(th, sv, so, M, n, stride, sc, vec_ok, st, t);
    }
}

static int64_t packed_elems(int M, int64_t n) { return ((n + kTile - 1) >> kTileShift) * (3 * (int64_t)M + 1) * kTile; }

static int mode_of(int base, int apply_update) {
    return !apply_update ? MODE_RECORD : (base == DILOCO_EAGER ? MODE_EAGER : MODE_DELAYED);
}

// The `variant` argument of the eager entry points: base rule in the low byte, flag bits above.
struct Variant {
    int base;     // DILOCO_EAGER or DILOCO_DELAYED
    int no_mean;  // DILOCO_STATE_NO_MEAN
    OuterScalars wire;
};
static int parse_variant(int variant, Variant& v) {
    v.no_mean = (variant & DILOCO_STATE_NO_MEAN) ? 1 : 0;
    if (!parse_comm(variant & ~DILOCO_STATE_NO_MEAN & ~0xff, v.wire)) return DILOCO_ERR_DTYPE;
    v.base = variant & 0xff;
    if (v.base != DILOCO_EAGER && v.base != DILOCO_DELAYED) return DILOCO_ERR_DTYPE;
    if (v.no_mean && v.base != DILOCO_EAGER) return DILOCO_ERR_DTYPE;
    return DILOCO_OK;
}
static OuterScalars eager_scalars(int M, double lr, double mu, int nesterov, const Variant& v) {
    OuterScalars sc = make_scalars(M, lr, mu, nesterov);
    sc.comm = v.wire.comm, sc.q_mant = v.wire.q_mant, sc.q_emin = v.wire.q_emin, sc.q_bias = v.wire.q_bias;
    sc.q_max = v.wire.q_max;
    sc.no_mean = v.no_mean;
    return sc;
}

static int outer_eager_impl(void* theta, int theta_dtype, int M, int64_t n, int64_t stride, float* anchor,
                            float* vel, float* prev_local, int64_t state_stride, float* prev_mean,
                            double outer_lr, double outer_momentum, int nesterov, int variant, int apply_update,
                            void* stream, const Tuning& t) {
    if (!theta || !anchor || !vel || !prev_local || !prev_mean) return DILOCO_ERR_NULL;
    if (!valid_dtype(theta_dtype)) return DILOCO_ERR_DTYPE;
    Variant v;
    if (int e = parse_variant(variant, v)) return e;
    if (int e = check_shape(M, n, stride)) return e;
    if (int e = check_shape(M, n, state_stride)) return e;
    if (!is_finite(outer_lr) || !in_unit(outer_momentum)) return DILOCO_ERR_HYPER;
    const int es = elem_size(theta_dtype);
    if (!aligned_to(theta, es) || !aligned_to(anchor, 4) || !aligned_to(vel, 4) ||
        !aligned_to(prev_local, 4) || !aligned_to(prev_mean, 4))
        return DILOCO_ERR_ALIGN;
    Range r[5] = {{theta, extent_bytes(M, n, stride, es), true},
                  {anchor, extent_bytes(M, n, state_stride, 4), true},
                  {vel, extent_bytes(M, n, state_stride, 4), true},
                  {prev_local, extent_bytes(M, n, state_stride, 4), true},
                  {prev_mean, n * 4, true}};
    if (int e = check_alias(r, 5)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(theta, 4 * es) && aligned_to(anchor, 16) && aligned_to(vel, 16) &&
                        aligned_to(prev_local, 16) && aligned_to(prev_mean, 16) &&
                        (M == 1 || (stride % 4 == 0 && state_stride % 4 == 0));
    const OuterScalars sc = eager_scalars(M, outer_lr, outer_momentum, nesterov, v);
    const RowState sv{anchor, vel, prev_local, prev_mean, state_stride};
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int mode = mode_of(v.base, apply_update);
    if (theta_dtype == DILOCO_F32)
        return dispatch_eager<float, RowState>(theta, sv, sv, M, n, stride, sc, vec_ok, mode, st, t);
    return dispatch_eager<__bf16, RowState>(theta, sv, sv, M, n, stride, sc, vec_ok, mode, st, t);
}

// state_out == state: in place.  Otherwise the state is read from `state` and written to state_out.
// hist_from_out: the previous local and averaged outer gradients are read from state_out (the
// generation written two boundaries ago), the outer parameters and velocities from `state`.
static int outer_eager_packed_impl(void* theta, int theta_dtype, int M, int64_t n, int64_t stride, float* state,
                                   float* state_out, bool hist_from_out, double outer_lr, double outer_momentum,
                                   int nesterov, int variant, int apply_update, void* stream, const Tuning& t) {
    if (!theta || !state || !state_out) return DILOCO_ERR_NULL;
    if (!valid_dtype(theta_dtype)) return DILOCO_ERR_DTYPE;
    Variant v;
    if (int e = parse_variant(variant, v)) return e;
    if (int e = check_shape(M, n, stride)) return e;
    if (n > ((int64_t)1 << 40)) return DILOCO_ERR_SHAPE;
    if (!is_finite(outer_lr) || !in_unit(outer_momentum)) return DILOCO_ERR_HYPER;
    const int es = elem_size(theta_dtype);
    if (!aligned_to(theta, es) || !aligned_to(state, 16) || !aligned_to(state_out, 16)) return DILOCO_ERR_ALIGN;
    const bool in_place = state_out == state;
    Range r[3] = {{theta, extent_bytes(M, n, stride, es), true},
                  {state, packed_elems(M, n) * 4, in_place},
                  {in_place ? nullptr : state_out, packed_elems(M, n) * 4, true}};
    if (int e = check_alias(r, 3)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(theta, 4 * es) && (M == 1 || stride % 4 == 0);
    const OuterScalars sc = eager_scalars(M, outer_lr, outer_momentum, nesterov, v);
    const TiledState sv{state, hist_from_out ? state_out : state, (int64_t)M}, so{state_out, state_out, (int64_t)M};
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int mode = mode_of(v.base, apply_update);
    if (theta_dtype == DILOCO_F32)
        return dispatch_eager<float, TiledState>(theta, sv, so, M, n, stride, sc, vec_ok, mode, st, t);
    return dispatch_eager<__bf16, TiledState>(theta, sv, so, M, n, stride, sc, vec_ok, mode, st, t);
}

}  // namespace diloco

using namespace diloco;

extern "C" int diloco_outer_eager(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                  int64_t stride, float* anchor, float* vel, float* prev_local,
                                  int64_t state_stride, float* prev_mean, double outer_lr,
                                  double outer_momentum, int nesterov, int variant,
                                  int apply_update, void* stream) {
    return outer_eager_impl(theta, theta_dtype, M, n, stride, anchor, vel, prev_local, state_stride, prev_mean,
                            outer_lr, outer_momentum, nesterov, variant, apply_update, stream, tuning());
}

extern "C" int diloco_outer_eager_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                         int64_t stride, float* anchor, float* vel, float* prev_local,
                                         int64_t state_stride, float* prev_mean, double outer_lr,
                                         double outer_momentum, int nesterov, int variant,
                                         int apply_update, void* stream, const diloco_launch* launch) {
    Tuning t;
    if (!resolve_launch(launch, t)) return DILOCO_ERR_HYPER;
    return outer_eager_impl(theta, theta_dtype, M, n, stride, anchor, vel, prev_local, state_stride, prev_mean,
                            outer_lr, outer_momentum, nesterov, variant, apply_update, stream, t);
}

extern "C" int64_t diloco_packed_state_elems(int M, int64_t n) {
    if (M < 1 || M > DILOCO_MAX_REPLICAS || n < 0 || n > ((int64_t)1 << 40)) return -1;
    return packed_elems(M, n);
}

extern "C" int diloco_outer_eager_packed(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                         int64_t stride, float* state, double outer_lr,
                                         double outer_momentum, int nesterov, int variant,
                                         int apply_update, void* stream) {
    return outer_eager_packed_impl(theta, theta_dtype, M, n, stride, state, state, false, outer_lr, outer_momentum,
                                   nesterov, variant, apply_update, stream, tuning());
}

extern "C" int diloco_outer_eager_overlap2(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                           int64_t stride, const float* state_prev, float* state_cur,
                                           double outer_lr, double outer_momentum, int nesterov, int variant,
                                           int apply_update, void* stream) {
    if (state_prev == state_cur && state_prev) return DILOCO_ERR_ALIAS;
    if (variant & DILOCO_STATE_NO_MEAN) return DILOCO_ERR_DTYPE;  // the mean of two boundaries ago is not at hand otherwise
    return outer_eager_packed_impl(theta, theta_dtype, M, n, stride, const_cast<float*>(state_prev), state_cur, true,
                                   outer_lr, outer_momentum, nesterov, variant, apply_update, stream, tuning());
}

extern "C" int diloco_outer_eager_pingpong(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                           int64_t stride, const float* state_in, float* state_out,
                                           double outer_lr, double outer_momentum, int nesterov, int variant,
                                           int apply_update, void* stream) {
    if (state_in == state_out && state_in) return DILOCO_ERR_ALIAS;
    return outer_eager_packed_impl(theta, theta_dtype, M, n, stride, const_cast<float*>(state_in), state_out, false,
                                   outer_lr, outer_momentum, nesterov, variant, apply_update, stream, tuning());
}

extern "C" int diloco_outer_eager_pingpong_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                                  int64_t stride, const float* state_in, float* state_out,
                                                  double outer_lr, double outer_momentum, int nesterov,
                                                  int variant, int apply_update, void* stream,
                                                  const diloco_launch* launch) {
    Tuning t;
    if (!resolve_launch(launch, t)) return DILOCO_ERR_HYPER;
    if (state_in == state_out && state_in) return DILOCO_ERR_ALIAS;
    return outer_eager_packed_impl(theta, theta_dtype, M, n, stride, const_cast<float*>(state_in), state_out, false,
                                   outer_lr, outer_momentum, nesterov, variant, apply_update, stream, t);
}

extern "C" int diloco_outer_eager_packed_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                                int64_t stride, float* state, double outer_lr,
                                                double outer_momentum, int nesterov, int variant,
                                                int apply_update, void* stream, const diloco_launch* launch) {
    Tuning t;
    if (!resolve_launch(launch, t)) return DILOCO_ERR_HYPER;
    return outer_eager_packed_impl(theta, theta_dtype, M, n, stride, state, state, false, outer_lr, outer_momentum,
                                   nesterov, variant, apply_update, stream, t);
}

// rows <-> tiled.  Any of anchor / vel / prev_local / prev_mean may be NULL (skipped).
static int repack(bool to_tiled, float* state, int M, int64_t n, float* anchor, float* vel, float* prev_local,
                  int64_t state_stride, float* prev_mean, void* stream) {
    if (!state) return DILOCO_ERR_NULL;
    if (int e = check_shape(M, n, state_stride)) return e;
    if (n > ((int64_t)1 << 40) || 3 * M + 1 > 65535) return DILOCO_ERR_SHAPE;
    if (!aligned_to(state, 16) || !aligned_to(anchor, 4) || !aligned_to(vel, 4) || !aligned_to(prev_local, 4) ||
        !aligned_to(prev_mean, 4))
        return DILOCO_ERR_ALIGN;
    const int64_t rb = extent_bytes(M, n, state_stride, 4);
    Range r[5] = {{state, packed_elems(M, n) * 4, to_tiled}, {anchor, rb, !to_tiled}, {vel, rb, !to_tiled},
                  {prev_local, rb, !to_tiled}, {prev_mean, n * 4, !to_tiled}};
    if (int e = check_alias(r, 5)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(anchor, 16) && aligned_to(vel, 16) && aligned_to(prev_local, 16) &&
                        aligned_to(prev_mean, 16) && (M == 1 || state_stride % 4 == 0);
    const Tuning& t = tuning();
    const int block = plain_block(t);
    const int64_t threads = vec_ok ? (n + 3) >> 2 : n;
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    dim3 grid(g.blocks, 3 * M + 1);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (to_tiled && vec_ok)
        return launch(repack_kernel<true, 4>, grid, dim3(block), 0, st, state, anchor, vel, prev_local, prev_mean, M,
                      n, state_stride, g.per_xcd);
    if (to_tiled)
        return launch(repack_kernel<true, 1>, grid, dim3(block), 0, st, state, anchor, vel, prev_local, prev_mean, M,
                      n, state_stride, g.per_xcd);
    if (vec_ok)
        return launch(repack_kernel<false, 4>, grid, dim3(block), 0, st, state, anchor, vel, prev_local, prev_mean, M,
                      n, state_stride, g.per_xcd);
    return launch(repack_kernel<false, 1>, grid, dim3(block), 0, st, state, anchor, vel, prev_local, prev_mean, M, n,
                  state_stride, g.per_xcd);
}

extern "C" int diloco_pack_state(float* state, int M, int64_t n, const float* anchor, const float* vel,
                                 const float* prev_local, int64_t state_stride, const float* prev_mean,
                                 void* stream) {
    return repack(true, state, M, n, const_cast<float*>(anchor), const_cast<float*>(vel),
                  const_cast<float*>(prev_local), state_stride, const_cast<float*>(prev_mean), stream);
}

extern "C" int diloco_unpack_state(const float* state, int M, int64_t n, float* anchor, float* vel,
                                   float* prev_local, int64_t state_stride, float* prev_mean, void* stream) {
    return repack(false, const_cast<float*>(state), M, n, anchor, vel, prev_local, state_stride, prev_mean,
                  stream);
}

template <typename TT>
static int launch_sync(TT* theta, float* anchor, float* vel, float* mean_out, int M, int64_t n,
                       int64_t stride, const OuterScalars& sc, bool vec_ok, hipStream_t st, const Tuning& t) {
    // a wavefront of the vector kernel has the anchor, the velocity and one group of theta_m in
    // flight; measured best (n = 2^26, fp32): 12 / 8 / 8 / 4 workgroups per CU at M = 1 / 2 / 4 / >= 8
    const int grp = M < kGroup ? M : kGroup;
    const Shape shape = launch_shape(t, (int64_t)64 * (2 * 16 + grp * 4 * (int64_t)sizeof(TT)), kInFlightTarget);
    const int block = shape.block;
    const int64_t threads = vec_ok ? (n >> 2) + ((n & 3) ? 1 : 0) : n;
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    if (vec_ok) {
        if (!grant_lds(&outer_sync_vec_kernel<TT>, shape.lds)) return DILOCO_ERR_LAUNCH;
        return launch(outer_sync_vec_kernel<TT>, dim3(g.blocks), dim3(block), shape.lds, st, theta, anchor, vel,
                      mean_out, M, n, stride, sc, g.per_xcd);
    }
    return launch(outer_sync_scalar_kernel<TT>, dim3(g.blocks), dim3(block), 0, st, theta, anchor, vel, mean_out, M,
                  n, stride, sc, g.per_xcd);
}

static int outer_sync_impl(void* theta, int theta_dtype, int M, int64_t n, int64_t stride, float* anchor, float* vel,
                           float* mean_out, double outer_lr, double outer_momentum, int nesterov, int comm,
                           void* stream, const Tuning& t) {
    if (!theta || !anchor || !vel) return DILOCO_ERR_NULL;
    if (!valid_dtype(theta_dtype)) return DILOCO_ERR_DTYPE;
    OuterScalars wire;
    if ((comm & 0xff) != 0 || !parse_comm(comm, wire)) return DILOCO_ERR_DTYPE;
    if (int e = check_shape(M, n, stride)) return e;
    if (!is_finite(outer_lr) || !in_unit(outer_momentum)) return DILOCO_ERR_HYPER;
    const int es = elem_size(theta_dtype);
    if (!aligned_to(theta, es) || !aligned_to(anchor, 4) || !aligned_to(vel, 4) ||
        !aligned_to(mean_out, 4))
        return DILOCO_ERR_ALIGN;
    Range r[4] = {{theta, extent_bytes(M, n, stride, es), true},
                  {anchor, n * 4, true},
                  {vel, n * 4, true},
                  {mean_out, n * 4, true}};
    if (int e = check_alias(r, 4)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(theta, 4 * es) && aligned_to(anchor, 16) && aligned_to(vel, 16) &&
                        aligned_to(mean_out, 16) && (M == 1 || stride % 4 == 0);
    OuterScalars sc = make_scalars(M, outer_lr, outer_momentum, nesterov);
    sc.comm = wire.comm, sc.q_mant = wire.q_mant, sc.q_emin = wire.q_emin, sc.q_bias = wire.q_bias, sc.q_max = wire.q_max;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (theta_dtype == DILOCO_F32)
        return launch_sync<float>(static_cast<float*>(theta), anchor, vel, mean_out, M, n, stride, sc, vec_ok, st, t);
    return launch_sync<__bf16>(static_cast<__bf16*>(theta), anchor, vel, mean_out, M, n, stride, sc, vec_ok, st, t);
}

extern "C" int diloco_outer_sync_comm(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                      int64_t stride, float* anchor, float* vel, float* mean_out,
                                      double outer_lr, double outer_momentum, int nesterov, int comm,
                                      void* stream) {
    return outer_sync_impl(theta, theta_dtype, M, n, stride, anchor, vel, mean_out, outer_lr, outer_momentum,
                           nesterov, comm, stream, tuning());
}

extern "C" int diloco_outer_sync_shaped(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                        int64_t stride, float* anchor, float* vel, float* mean_out,
                                        double outer_lr, double outer_momentum, int nesterov, int comm,
                                        void* stream, const diloco_launch* launch) {
    Tuning t;
    if (!resolve_launch(launch, t)) return DILOCO_ERR_HYPER;
    return outer_sync_impl(theta, theta_dtype, M, n, stride, anchor, vel, mean_out, outer_lr, outer_momentum,
                           nesterov, comm, stream, t);
}

extern "C" int diloco_outer_sync(void* theta, diloco_dtype theta_dtype, int M, int64_t n,
                                 int64_t stride, float* anchor, float* vel, float* mean_out,
                                 double outer_lr, double outer_momentum, int nesterov,
                                 void* stream) {
    return diloco_outer_sync_comm(theta, theta_dtype, M, n, stride, anchor, vel, mean_out, outer_lr,
                                  outer_momentum, nesterov, 0, stream);
}

template <typename TT, typename AV>
static int launch_reset(void* theta, AV av, int M, int64_t n, int64_t stride, bool vec_ok, hipStream_t st) {
    const Tuning& t = tuning();
    const int block = plain_block(t);
    const int64_t threads = vec_ok ? (n >> 2) + ((n & 3) ? 1 : 0) : n;
    if (!grid_fits(threads, block)) return DILOCO_ERR_SHAPE;
    Grid g = make_grid(t, threads, block);
    if (vec_ok)
        return launch(reset_vec_kernel<TT, AV>, dim3(g.blocks, M), dim3(block), 0, st, static_cast<TT*>(theta), av, n,
                      stride, g.per_xcd);
    return launch(reset_scalar_kernel<TT, AV>, dim3(g.blocks, M), dim3(block), 0, st, static_cast<TT*>(theta), av, n,
                  stride, g.per_xcd);
}

extern "C" int diloco_reset(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                            const float* anchor, int64_t anchor_stride, void* stream) {
    if (!theta || !anchor) return DILOCO_ERR_NULL;
    if (!valid_dtype(theta_dtype)) return DILOCO_ERR_DTYPE;
    if (int e = check_shape(M, n, stride)) return e;
    if (anchor_stride != 0)
        if (int e = check_shape(M, n, anchor_stride)) return e;
    const int es = elem_size(theta_dtype);
    if (!aligned_to(theta, es) || !aligned_to(anchor, 4)) return DILOCO_ERR_ALIGN;
    Range r[2] = {{theta, extent_bytes(M, n, stride, es), true},
                  {anchor, anchor_stride ? extent_bytes(M, n, anchor_stride, 4) : n * 4, false}};
    if (int e = check_alias(r, 2)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(theta, 4 * es) && aligned_to(anchor, 16) &&
                        (M == 1 || (stride % 4 == 0 && anchor_stride % 4 == 0));
    const RowAnchor av{anchor, anchor_stride};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (theta_dtype == DILOCO_F32) return launch_reset<float, RowAnchor>(theta, av, M, n, stride, vec_ok, st);
    return launch_reset<__bf16, RowAnchor>(theta, av, M, n, stride, vec_ok, st);
}

extern "C" int diloco_reset_packed(void* theta, diloco_dtype theta_dtype, int M, int64_t n, int64_t stride,
                                   const float* state, void* stream) {
    if (!theta || !state) return DILOCO_ERR_NULL;
    if (!valid_dtype(theta_dtype)) return DILOCO_ERR_DTYPE;
    if (int e = check_shape(M, n, stride)) return e;
    if (n > ((int64_t)1 << 40)) return DILOCO_ERR_SHAPE;
    const int es = elem_size(theta_dtype);
    if (!aligned_to(theta, es) || !aligned_to(state, 16)) return DILOCO_ERR_ALIGN;
    Range r[2] = {{theta, extent_bytes(M, n, stride, es), true}, {state, packed_elems(M, n) * 4, false}};
    if (int e = check_alias(r, 2)) return e;
    if (n == 0) return DILOCO_OK;
    const bool vec_ok = aligned_to(theta, 4 * es) && (M == 1 || stride % 4 == 0);
    const TiledAnchor av{state, 3 * (int64_t)M + 1};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (theta_dtype == DILOCO_F32) return launch_reset<float, TiledAnchor>(theta, av, M, n, stride, vec_ok, st);
    return launch_reset<__bf16, TiledAnchor>(theta, av, M, n, stride, vec_ok, st);
}

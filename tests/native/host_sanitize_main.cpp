// Host-side checks of the library under AddressSanitizer and UndefinedBehaviorSanitizer.
//
// Linked with the library's own sources, their HOST pass compiled with
// -fsanitize=address,undefined (the device code is built as always and never runs here).  Every
// entry point is driven through its argument validation, the wire-format parser, the alias
// check, the schedule helpers, the per-thread launch shape and the launch-shape arithmetic, with
// the arguments the CPU boundary tests use: fake, suitably aligned device addresses that
// validation never dereferences.  Where a call passes validation it goes on to ask the HIP
// runtime for a launch; without a GPU that is refused (DILOCO_ERR_LAUNCH), with one the size is
// kept at zero so that nothing is launched on made-up addresses.
// Exit status 0 and "host checks passed" on success; a sanitizer report aborts the program.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>

#include "diloco.h"
#include "diloco_sim.h"

static int failures = 0;
#define EXPECT(call, want)                                                                      \
    do {                                                                                        \
        const long long got_ = (long long)(call);                                               \
        if (got_ != (long long)(want)) {                                                        \
            std::printf("line %d: %s = %lld, expected %lld\n", __LINE__, #call, got_, (long long)(want)); \
            ++failures;                                                                         \
        }                                                                                       \
    } while (0)

static void* P(int k, long off = 0) { return reinterpret_cast<void*>(0x700000000000ull + (uint64_t)k * 0x10000000ull + off); }
static float* F(int k, long off = 0) { return static_cast<float*>(P(k, off)); }

static int eager(int M, int64_t n, int64_t stride, float* a, float* pm, double mu, int var, void* theta = P(0)) {
    return diloco_outer_eager(theta, DILOCO_F32, M, n, stride, a, F(2), F(3), stride, pm, 0.7, mu, 1, var, 1, nullptr);
}

int main() {
    // status texts and version
    for (int c = 0; c < 8; ++c) EXPECT(diloco_strerror(c) != nullptr, 1);
    EXPECT(diloco_version() >= 100, 1);

    // eager / delayed: every validation branch, every flag combination the parser knows
    EXPECT(eager(2, 0, 64, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_OK);
    EXPECT(eager(2, 64, 64, nullptr, F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_NULL);
    EXPECT(eager(0, 64, 64, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_SHAPE);
    EXPECT(eager(70000, 64, 64, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_SHAPE);
    EXPECT(eager(2, -1, 64, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_SHAPE);
    EXPECT(eager(2, 64, 63, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_SHAPE);
    EXPECT(eager(2, (int64_t)1 << 61, (int64_t)1 << 61, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_SHAPE);
    EXPECT(eager(65535, (int64_t)1 << 59, (int64_t)1 << 59, F(1), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_SHAPE);
    EXPECT(eager(2, 64, 64, F(1), F(4), 1.0, DILOCO_EAGER), DILOCO_ERR_HYPER);
    EXPECT(eager(2, 64, 64, F(1, 2), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_ALIGN);
    EXPECT(eager(2, 64, 64, F(0), F(4), 0.9, DILOCO_EAGER), DILOCO_ERR_ALIAS);
    EXPECT(eager(2, 64, 64, F(1), F(3, 64), 0.9, DILOCO_EAGER), DILOCO_ERR_ALIAS);
    EXPECT(eager(2, 64, 64, F(1), F(4), 0.9, 2), DILOCO_ERR_DTYPE);
    EXPECT(eager(2, 64, 64, F(1), F(4), 0.9, 0x800), DILOCO_ERR_DTYPE);
    EXPECT(eager(2, 64, 64, F(1), F(4), 0.9, DILOCO_DELAYED | DILOCO_STATE_NO_MEAN), DILOCO_ERR_DTYPE);
    EXPECT(eager(2, 64, 64, F(1), F(4), 0.9, DILOCO_EAGER | DILOCO_COMM_BF16 | DILOCO_COMM_EXMY(4, 3, 7)), DILOCO_ERR_DTYPE);
    for (int E = 0; E <= 15; ++E)            // the whole space of format fields: parsed or refused, never UB
        for (int Mn = 0; Mn <= 15; ++Mn)
            for (int bias = -128; bias <= 127; bias += 5) {
                const int rc = eager(2, 0, 64, F(1), F(4), 0.9, DILOCO_EAGER | DILOCO_COMM_EXMY(E, Mn, bias));
                if (rc != DILOCO_OK && rc != DILOCO_ERR_DTYPE) EXPECT(rc, DILOCO_OK);
            }
    EXPECT(eager(9, 0, 64, F(1), F(4), 0.9, DILOCO_EAGER | DILOCO_STATE_NO_MEAN | DILOCO_COMM_EXMY(2, 1, 11)), DILOCO_OK);
    for (int bits = 0; bits < 32; ++bits)    // any single bit in `variant`
        (void)eager(2, 0, 64, F(1), F(4), 0.9, (int)(1u << bits));
    (void)eager(2, 0, 64, F(1), F(4), 0.9, -1);
    (void)eager(2, 0, 64, F(1), F(4), 0.9, INT32_MIN);

    // packed state, ping-pong, 2-step overlap, conversions
    EXPECT(diloco_packed_state_elems(8, 8193), 2 * 25 * 8192);
    EXPECT(diloco_packed_state_elems(0, 5), -1);
    EXPECT(diloco_packed_state_elems(65535, (int64_t)1 << 40), ((int64_t)1 << 40) * (3 * 65535LL + 1));
    EXPECT(diloco_outer_eager_packed(P(0), DILOCO_F32, 2, 0, 64, F(1), 0.7, 0.9, 1, DILOCO_EAGER, 1, nullptr), DILOCO_OK);
    EXPECT(diloco_outer_eager_packed(P(0), DILOCO_F32, 2, 64, 64, F(0, 16), 0.7, 0.9, 1, DILOCO_EAGER, 1, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_outer_eager_packed(P(0), DILOCO_BF16, 2, ((int64_t)1 << 40) + 1, ((int64_t)1 << 40) + 1, F(1), 0.7, 0.9, 1, 0, 1, nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_outer_eager_pingpong(P(0), DILOCO_F32, 2, 64, 64, F(1), F(1), 0.7, 0.9, 1, 0, 1, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_outer_eager_pingpong(P(0), DILOCO_F32, 2, 64, 64, F(1), F(1, 4 * 8192), 0.7, 0.9, 1, 0, 1, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_outer_eager_pingpong(P(0), DILOCO_F32, 2, 0, 64, F(1), F(2), 0.7, 0.9, 1, 0, 1, nullptr), DILOCO_OK);
    EXPECT(diloco_outer_eager_overlap2(P(0), DILOCO_F32, 2, 0, 64, F(1), F(2), 0.7, 0.9, 1, DILOCO_DELAYED, 1, nullptr), DILOCO_OK);
    EXPECT(diloco_outer_eager_overlap2(P(0), DILOCO_F32, 2, 64, 64, F(1), F(2), 0.7, 0.9, 1, DILOCO_STATE_NO_MEAN, 1, nullptr), DILOCO_ERR_DTYPE);
    EXPECT(diloco_pack_state(F(0), 2, 0, F(1), F(2), F(3), 64, F(4), nullptr), DILOCO_OK);
    EXPECT(diloco_pack_state(F(0), 30000, 64, F(1), F(2), F(3), 64, F(4), nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_unpack_state(F(0), 2, 64, F(0), nullptr, nullptr, 64, nullptr, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_unpack_state(F(0), 2, 0, nullptr, nullptr, nullptr, 64, nullptr, nullptr), DILOCO_OK);
    EXPECT(diloco_reset_packed(P(0), DILOCO_F32, 2, 0, 64, F(1), nullptr), DILOCO_OK);
    EXPECT(diloco_reset(P(0), DILOCO_BF16, 2, 64, 64, F(1), 5, nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_reset(P(0), DILOCO_F32, 2, 64, 64, F(0, 256), 0, nullptr), DILOCO_ERR_ALIAS);

    // standard outer step and AdamW
    EXPECT(diloco_outer_sync(P(0), DILOCO_F32, 2, 0, 64, F(1), F(2), nullptr, 0.7, 0.9, 1, nullptr), DILOCO_OK);
    EXPECT(diloco_outer_sync_comm(P(0), DILOCO_F32, 2, 64, 64, F(1), F(2), F(1), 0.7, 0.9, 1, 0, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_outer_sync_comm(P(0), DILOCO_F32, 2, 64, 64, F(1), F(2), nullptr, 0.7, 0.9, 1, 1, nullptr), DILOCO_ERR_DTYPE);
    EXPECT(diloco_inner_adamw(P(0), P(1), P(2), P(3), 2, 0, 64, DILOCO_F32, DILOCO_BF16, 4e-4, 0.9, 0.95, 1e-8, 0.1, 1, nullptr), DILOCO_OK);
    EXPECT(diloco_inner_adamw(P(0), P(1), P(2), P(0), 2, 64, 64, DILOCO_F32, DILOCO_F32, 4e-4, 0.9, 0.95, 1e-8, 0.1, 1, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_inner_adamw(P(0), P(1), P(2), P(3), 2, 64, 64, DILOCO_F32, DILOCO_F32, 4e-4, 0.9, 0.95, 0.0, 0.1, 1, nullptr), DILOCO_ERR_HYPER);
    EXPECT(diloco_inner_adamw(P(0), P(1), P(2), P(3), 2, 64, 64, DILOCO_F32, DILOCO_F32, 4e-4, 0.9, 0.95, 1e-8, 0.1, 0, nullptr), DILOCO_ERR_HYPER);

    // harness calls
    EXPECT(diloco_sim_quadratic_inner(F(0), F(1), F(2), 2, 0, 64, F(3), F(4), 0.1, 1, 0, 4e-4, 0.9, 0.95, 1e-8, 0.0, 1, nullptr), DILOCO_OK);
    EXPECT(diloco_sim_quadratic_inner(F(0), F(1), F(2), 2, 64, 64, F(3), F(4), 0.1, 1, 2, 4e-4, 0.9, 0.95, 1e-8, 0.0, 1, nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_sim_quadratic_phase(F(0), F(1), F(2), 2, 64, 64, F(3), F(4), 0.1, 1, 0, 4e-4, 0.9, 0.95, 1e-8, 0.0, 1, 65, nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_sim_quadratic_phase(F(0), F(1), F(2), 2, 64, 64, F(3), F(4), 0.1, 1, 0, 4e-4, 0.9, 0.95, 1e-8, 0.0, 1, 0, nullptr), DILOCO_OK);
    EXPECT(diloco_sim_loss_workspace(0), 1);
    EXPECT(diloco_sim_loss_workspace((int64_t)1 << 40), 8192);
    EXPECT(diloco_sim_quadratic_loss(F(0), 2, 64, 64, F(1), F(2), reinterpret_cast<double*>(P(3)), 0, reinterpret_cast<double*>(P(4)), nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_sim_quadratic_loss_static(F(0), 1, ((int64_t)1 << 40) + 1, ((int64_t)1 << 40) + 1, F(1), F(2), reinterpret_cast<double*>(P(3)), nullptr), DILOCO_ERR_SHAPE);
    EXPECT(diloco_sim_quadratic_loss_static(F(0), 2, 64, 64, F(1), F(2), reinterpret_cast<double*>(P(0, 8)), nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_sim_stream_copy(F(0), F(1), 0, nullptr, nullptr), DILOCO_OK);
    EXPECT(diloco_sim_stream_copy(F(0), F(0, 16), 64, nullptr, nullptr), DILOCO_ERR_ALIAS);
    EXPECT(diloco_sim_stream_sweep(F(0), 4, 0, 64, DILOCO_SIM_SWEEP_READ, 0.f, nullptr, nullptr), DILOCO_OK);
    EXPECT(diloco_sim_stream_sweep(F(0), 4, 64, 64, 3, 0.f, nullptr, nullptr), DILOCO_ERR_DTYPE);
    EXPECT(diloco_sim_stream_rmw(F(0), 3, 64, 64, nullptr, nullptr), DILOCO_ERR_SHAPE);

    // explicit launch shapes: the struct is read, checked, and (n = 0) never used for a launch
    const diloco_launch good = {256, 1, 2, 1}, bad_block = {100, 0, 0, 0}, bad_cap = {0, 0, 33, 0}, bad_path = {0, 0, -1, 3};
    EXPECT(diloco_outer_eager_packed_shaped(P(0), DILOCO_F32, 2, 0, 64, F(1), 0.7, 0.9, 1, 0, 1, nullptr, &good), DILOCO_OK);
    EXPECT(diloco_outer_eager_packed_shaped(P(0), DILOCO_F32, 2, 0, 64, F(1), 0.7, 0.9, 1, 0, 1, nullptr, &bad_block), DILOCO_ERR_HYPER);
    EXPECT(diloco_outer_eager_shaped(P(0), DILOCO_F32, 2, 0, 64, F(1), F(2), F(3), 64, F(4), 0.7, 0.9, 1, 0, 1, nullptr, &bad_cap), DILOCO_ERR_HYPER);
    EXPECT(diloco_outer_eager_pingpong_shaped(P(0), DILOCO_F32, 2, 0, 64, F(1), F(2), 0.7, 0.9, 1, 0, 1, nullptr, &bad_path), DILOCO_ERR_HYPER);
    EXPECT(diloco_outer_sync_shaped(P(0), DILOCO_F32, 2, 0, 64, F(1), F(2), nullptr, 0.7, 0.9, 1, 0, nullptr, &good), DILOCO_OK);
    EXPECT(diloco_inner_adamw_shaped(P(0), P(1), P(2), P(3), 2, 0, 64, DILOCO_F32, DILOCO_F32, 4e-4, 0.9, 0.95, 1e-8, 0.1, 1, nullptr, &good), DILOCO_OK);

    // the thread's launch shape: per thread, range-checked
    EXPECT(diloco_tune("block", 128), DILOCO_OK);
    EXPECT(diloco_tune("block", 100), DILOCO_ERR_HYPER);
    EXPECT(diloco_tune("nope", 1), DILOCO_ERR_HYPER);
    EXPECT(diloco_tune(nullptr, 1), DILOCO_ERR_NULL);
    EXPECT(diloco_tune_get(nullptr), -1);
    int seen_block = -1, seen_cap = -2;
    std::thread other([&] {
        seen_block = diloco_tune_get("block");
        seen_cap = diloco_tune_get("wg_per_cu");
        (void)diloco_tune("wg_per_cu", 7);
    });
    other.join();
    EXPECT(seen_block, 0);
    EXPECT(seen_cap, -1);
    EXPECT(diloco_tune_get("block"), 128);
    EXPECT(diloco_tune_get("wg_per_cu"), -1);
    EXPECT(diloco_tune("block", 0), DILOCO_OK);

    // streaming schedule: every fragment has exactly one boundary per H steps, counts add up
    for (int64_t H : {1, 2, 7, 30, 100})
        for (int Fr : {1, 2, 3, 8, 13}) {
            for (int f = 0; f < Fr; ++f) {
                int64_t count = 0;
                for (int64_t t = 0; t <= 5 * H; ++t) {
                    const int due = diloco_stream_due(t, H, Fr, f);
                    if (due < 0) EXPECT(due, 0);
                    count += due;
                    EXPECT(diloco_stream_boundary_count(t, H, Fr, f), count);
                }
                EXPECT(count >= 4 && count <= 5, 1);
                EXPECT(diloco_stream_offset(H, Fr, f) >= 0 && diloco_stream_offset(H, Fr, f) < H, 1);
            }
            EXPECT(diloco_stream_due(3, H, Fr, Fr), -1);
            EXPECT(diloco_stream_offset(0, Fr, 0), -1);
        }
    EXPECT(diloco_stream_boundary_count(INT64_MAX, (int64_t)1 << 40, 65535, 65534) > 0, 1);

    // calls that pass validation and reach the launch-shape arithmetic: every replica count's kernel
    // choice, odd strides (element-wise kernels), every workgroup size.  Without a GPU the launch is
    // refused (DILOCO_ERR_LAUNCH); on a machine with one these are skipped, the addresses being made up.
    if (std::getenv("DILOCO_HOST_CHECK_LAUNCH_PATHS")) {
        const diloco_launch shapes[] = {{0, 0, -1, 0}, {64, 1, 2, 0}, {256, 0, 0, 0}, {512, 1, 1, 1}, {128, 1, 3, 2}, {64, 0, 32, 0}};
        for (const diloco_launch& sh : shapes)
            for (int M : {1, 2, 8, 9, 26, 27, 40, 41, 100, 65535})
                for (int64_t n : {(int64_t)1, (int64_t)4099, (int64_t)1 << 33}) {
                    const int64_t stride = n + (M % 2);
                    for (int var : {(int)DILOCO_EAGER, (int)DILOCO_DELAYED, DILOCO_EAGER | DILOCO_STATE_NO_MEAN}) {
                        if ((int64_t)M * stride > ((int64_t)1 << 44)) continue;   // keep the made-up ranges apart
                        int rc = diloco_outer_eager_shaped(P(0), DILOCO_F32, M, n, stride, F(2), F(4), F(6), stride, F(7),
                                                           0.7, 0.9, 1, var, 1, nullptr, &sh);
                        if (rc != DILOCO_ERR_LAUNCH && rc != DILOCO_ERR_ALIAS && rc != DILOCO_ERR_SHAPE) EXPECT(rc, DILOCO_ERR_LAUNCH);
                    }
                    if ((int64_t)M * stride <= ((int64_t)1 << 25)) {
                        int rc = diloco_outer_sync_shaped(P(0), DILOCO_BF16, M, n, stride, F(2), F(3), nullptr, 0.7, 0.9, 0, 0, nullptr, &sh);
                        if (rc != DILOCO_ERR_LAUNCH) EXPECT(rc, DILOCO_ERR_LAUNCH);
                        rc = diloco_inner_adamw_shaped(P(0), P(1), P(2), P(3), M, n, stride, DILOCO_BF16, DILOCO_F32, 4e-4, 0.9, 0.95, 1e-8, 0.1, 31, nullptr, &sh);
                        if (rc != DILOCO_ERR_LAUNCH) EXPECT(rc, DILOCO_ERR_LAUNCH);
                    }
                }
    }

    if (failures) {
        std::printf("%d host checks FAILED\n", failures);
        return 1;
    }
    std::printf("host checks passed\n");
    return 0;
}

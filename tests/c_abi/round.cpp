// The C ABI used from a plain HIP host program (no Python, no torch): one compress +
// aggregate round of a small tensor list through include/sparseloco.h, compared bit
// for bit with the CPU oracle (test infrastructure, linked here as a checker only).
// Built by __graft_entry__.build(); run by tests/test_gpu_c_abi.py.  Exit code 0 = equal.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "sparseloco.h"

extern "C" {
typedef struct {
    int64_t rows, cols, offset;
    int32_t layout, reserved;
} slo_tensor;
int64_t slo_payload_bytes(const slo_tensor *t, int nt, int tile, int k);
int slo_compress(const slo_tensor *t, int nt, int tile, int k, float *e, const float *delta, float beta,
                 int ef_frozen, uint8_t *payload, uint16_t *sel_idx, float *sel_val, uint8_t *sel_code,
                 float *lut_out);
int slo_decompress_avg_apply(const slo_tensor *t, int nt, int tile, int k, float *theta,
                             const uint8_t *const *payloads, int R, float lr);
}

#define HIP_OK(x)                                                                     \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                                 \
        }                                                                             \
    } while (0)
#define SL_OK_OR_FAIL(x)                                                          \
    do {                                                                          \
        int s_ = (x);                                                             \
        if (s_ != SL_OK) {                                                        \
            std::printf("%s failed: %s (%s)\n", #x, sl_strerror(s_), sl_last_hip_error()); \
            return 3;                                                             \
        }                                                                         \
    } while (0)

static uint32_t lcg(uint32_t &s) { return s = s * 1664525u + 1013904223u; }
static float small_value(uint32_t &s)     // roughly uniform in (-2e-3, 2e-3), sum of two draws
{
    const float a = (float)(lcg(s) >> 8) * (1.0f / 16777216.0f), b = (float)(lcg(s) >> 8) * (1.0f / 16777216.0f);
    return (a + b - 1.0f) * 2e-3f;
}

int main()
{
    const int k = 64, R = 3;
    const float beta = 0.95f, lr = 0.7f;
    const sl_tensor tensors[3] = {{150, 210, 0, SL_LAYOUT_TILE64, 0},
                                  {1, 9000, 31552, SL_LAYOUT_FLAT, 0},
                                  {128, 192, 40576, SL_LAYOUT_TILE64, 0}};
    const int64_t n = 40576 + 128 * 192;
    slo_tensor ot[3];
    for (int i = 0; i < 3; ++i) ot[i] = {tensors[i].rows, tensors[i].cols, tensors[i].offset, tensors[i].layout, 0};

    sl_plan *plan = nullptr;
    SL_OK_OR_FAIL(sl_plan_create(tensors, 3, k, &plan));
    const size_t pay_bytes = sl_payload_bytes(plan);
    if ((int64_t)pay_bytes != slo_payload_bytes(ot, 3, 64, k)) {
        std::printf("payload size differs\n");
        return 1;
    }
    float *d_e, *d_delta, *d_theta;
    void *d_ws, *d_pay[R];
    HIP_OK(hipMalloc((void **)&d_e, n * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_delta, n * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_theta, n * sizeof(float)));
    HIP_OK(hipMalloc(&d_ws, sl_workspace_bytes(plan)));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    uint32_t seed = 12345u;
    std::vector<float> theta(n), theta_ref;
    for (auto &v : theta) v = 10.0f * small_value(seed);
    theta_ref = theta;
    HIP_OK(hipMemcpy(d_theta, theta.data(), n * sizeof(float), hipMemcpyHostToDevice));

    std::vector<std::vector<uint8_t>> ref_pay(R, std::vector<uint8_t>(pay_bytes));
    int bad = 0;
    for (int r = 0; r < R; ++r) {
        std::vector<float> e(n), delta(n);
        for (auto &v : e) v = small_value(seed);
        for (auto &v : delta) v = small_value(seed);
        HIP_OK(hipMalloc(&d_pay[r], pay_bytes));
        HIP_OK(hipMemcpy(d_e, e.data(), n * sizeof(float), hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(d_delta, delta.data(), n * sizeof(float), hipMemcpyHostToDevice));
        SL_OK_OR_FAIL(sl_compress(plan, d_e, d_delta, beta, SL_COMPRESS_DEFAULT, nullptr, d_pay[r], d_ws, stream));
        HIP_OK(hipStreamSynchronize(stream));
        std::vector<uint8_t> pay(pay_bytes);
        std::vector<float> e_gpu(n);
        HIP_OK(hipMemcpy(pay.data(), d_pay[r], pay_bytes, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(e_gpu.data(), d_e, n * sizeof(float), hipMemcpyDeviceToHost));
        if (slo_compress(ot, 3, 64, k, e.data(), delta.data(), beta, 0, ref_pay[r].data(), nullptr, nullptr,
                         nullptr, nullptr)) {
            std::printf("oracle failed\n");
            return 1;
        }
        if (std::memcmp(pay.data(), ref_pay[r].data(), pay_bytes)) bad |= 1, std::printf("worker %d: payload differs\n", r);
        if (std::memcmp(e_gpu.data(), e.data(), n * sizeof(float))) bad |= 2, std::printf("worker %d: e differs\n", r);
        SL_OK_OR_FAIL(sl_payload_validate(plan, d_pay[r], d_ws, stream));
    }
    const void *pays[R];
    const uint8_t *ref_ptrs[R];
    for (int r = 0; r < R; ++r) pays[r] = d_pay[r], ref_ptrs[r] = ref_pay[r].data();
    SL_OK_OR_FAIL(sl_decompress_avg_apply(plan, d_theta, pays, R, lr, stream));
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(theta.data(), d_theta, n * sizeof(float), hipMemcpyDeviceToHost));
    slo_decompress_avg_apply(ot, 3, 64, k, theta_ref.data(), ref_ptrs, R, lr);
    if (std::memcmp(theta.data(), theta_ref.data(), n * sizeof(float))) bad |= 4, std::printf("theta differs\n");

    // argument errors come back as status codes, nothing is launched
    if (sl_compress(plan, d_e, d_e, beta, 0, nullptr, d_pay[0], d_ws, stream) != SL_ERR_INVALID_ARG) bad |= 8;
    if (sl_decompress_avg_apply(plan, d_theta, pays, 0, lr, stream) != SL_ERR_INVALID_ARG) bad |= 8;

    for (int r = 0; r < R; ++r) (void)hipFree(d_pay[r]);
    (void)hipFree(d_e), (void)hipFree(d_delta), (void)hipFree(d_theta), (void)hipFree(d_ws);
    (void)hipStreamDestroy(stream);
    SL_OK_OR_FAIL(sl_plan_destroy(plan));
    if (bad) {
        std::printf("c-abi round FAILED (mask %d)\n", bad);
        return 1;
    }
    std::printf("c-abi round ok: payloads, e and theta bit-identical to the oracle (k=%d, R=%d, %lld elements)\n", k, R,
                (long long)n);
    return 0;
}

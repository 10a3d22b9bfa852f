// A caller of libpipeoptim that uses nothing but the C ABI and the HIP runtime: no Python, no PyTorch.
// It builds a small ragged stage in device memory, runs the fused step + prediction (paper Table 1, Eq. 1,
// Eq. 5) and the prediction-only call on a stream of its own, and checks every element against the CPU
// oracle (linked as a C library; test infrastructure).  With the argument "arena" the buffers come from the
// library's near-memory arena instead of hipMalloc and the plan is localized over it.
// Run by tests/test_gpu_c_caller.py on a GPU machine.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pipeoptim.h"

extern "C" int po_oracle_step_predict(int opt, double lr, double beta1, double beta2, double eps, double weight_decay,
                                      int decay_in_prediction, long long t, int s, long long n, const float* W,
                                      const float* g, const float* m, const float* v, float* W_out, float* m_out,
                                      float* v_out, float* What_f32, uint16_t* What_bf16, int nthreads);
extern "C" uint16_t po_oracle_bf16_from_f32(float x);
extern "C" int po_oracle_predict(int opt, double lr, double beta1, double beta2, double eps, double weight_decay,
                                 int decay_in_prediction, long long t, int s, long long n, const float* W,
                                 const float* m, const float* v, float* What_f32, uint16_t* What_bf16, int nthreads);

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define PO_CHECK(x) do { int rc_ = (x); if (rc_ != PO_OK) { std::printf("libpipeoptim error %d at line %d: %s\n", rc_, __LINE__, pipeoptim_last_error()); return 1; } } while (0)

namespace {

// splitmix64 -> approximately normal values (sum of 4 uniforms), scaled
struct Rng {
    uint64_t s;
    uint64_t next() { uint64_t z = (s += 0x9E3779B97F4A7C15ull); z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull; z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; return z ^ (z >> 31); }
    float normalish(float sigma) { double a = 0; for (int i = 0; i < 4; ++i) a += (double)(next() >> 11) / 9007199254740992.0 - 0.5; return (float)(a * 1.7320508 * sigma); }
};

int bf16_order(uint16_t b) { return (b & 0x8000) ? -(int)(b & 0x7FFF) : (int)(b & 0x7FFF); }

// The library rounds ITS fp32 prediction to bf16, so its code may be the rounding of any value inside the
// fp32 tolerance band around the reference: normally that is the reference's code or a neighbour; where W
// and s*lr*dW nearly cancel the band can span a few of the (then tiny) bf16 steps.
bool bf16_within_band(uint16_t got, float ref, double tol)
{
    const int lo = bf16_order(po_oracle_bf16_from_f32((float)((double)ref - tol)));
    const int hi = bf16_order(po_oracle_bf16_from_f32((float)((double)ref + tol)));
    const int c = bf16_order(got);
    return c >= (lo < hi ? lo : hi) && c <= (lo < hi ? hi : lo);
}

}  // namespace

int main(int argc, char** argv)
{
    const bool use_arena = argc > 1 && std::strcmp(argv[1], "arena") == 0;
    const std::vector<int64_t> numel = {1, 255, 0, 4097, 70001, 12};
    const int n_tensors = (int)numel.size();
    po_hyper h{};
    h.opt = PO_ADAMW; h.decay_in_prediction = 1; h.lr = 1e-3; h.beta1 = 0.9; h.beta2 = 0.999; h.eps = 1e-8; h.weight_decay = 0.01;
    const int64_t t = 1000;
    int32_t s = -1;
    PO_CHECK(pipeoptim_version_difference(4, 0, &s));        // first stage of a 4-stage pipeline: s = 3

    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    std::vector<std::vector<float>> hW(n_tensors), hg(n_tensors), hm(n_tensors), hv(n_tensors);
    std::vector<float*> dW(n_tensors, nullptr), dm(n_tensors, nullptr), dv(n_tensors, nullptr);
    std::vector<const float*> dg(n_tensors, nullptr);
    std::vector<void*> dH(n_tensors, nullptr);
    Rng rng{20231200839ull};
    po_arena* arena = nullptr;
    if (use_arena) PO_CHECK(pipeoptim_arena_create(&arena, (int64_t)64 << 20));
    for (int i = 0; i < n_tensors; ++i) {
        const size_t n = (size_t)numel[i];
        hW[i].resize(n); hg[i].resize(n); hm[i].resize(n); hv[i].resize(n);
        for (size_t k = 0; k < n; ++k) {
            hW[i][k] = rng.normalish(0.02f); hg[i][k] = rng.normalish(1e-4f); hm[i][k] = rng.normalish(1e-5f);
            const float r = rng.normalish(1e-4f); hv[i][k] = r * r;
        }
        if (n == 0) continue;
        float* g_dev = nullptr;
        if (use_arena) {       // the five streams of a tensor in one call: one block-to-die layout
            const int64_t bytes[5] = {(int64_t)n * 4, (int64_t)n * 4, (int64_t)n * 4, (int64_t)n * 4, (int64_t)n * 2};
            void* p[5];
            PO_CHECK(pipeoptim_arena_alloc(arena, 5, bytes, p));
            dW[i] = (float*)p[0]; g_dev = (float*)p[1]; dm[i] = (float*)p[2]; dv[i] = (float*)p[3]; dH[i] = p[4];
        } else {
            HIP_OK(hipMalloc((void**)&dW[i], n * 4)); HIP_OK(hipMalloc((void**)&g_dev, n * 4));
            HIP_OK(hipMalloc((void**)&dm[i], n * 4)); HIP_OK(hipMalloc((void**)&dv[i], n * 4));
            HIP_OK(hipMalloc(&dH[i], n * 2));
        }
        dg[i] = g_dev;
        HIP_OK(hipMemcpy(dW[i], hW[i].data(), n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(g_dev, hg[i].data(), n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(dm[i], hm[i].data(), n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(dv[i], hv[i].data(), n * 4, hipMemcpyHostToDevice));
    }

    po_plan* plan = nullptr;
    PO_CHECK(pipeoptim_plan_create(&plan, n_tensors, numel.data(), dW.data(), dg.data(), dm.data(), dv.data(), dH.data(),
                                   PO_WHAT_BF16, stream));
    int64_t n_params = 0, n_chunks = 0, n_unaligned = 0;
    PO_CHECK(pipeoptim_plan_info(plan, &n_params, &n_chunks, &n_unaligned));
    std::printf("plan: %lld parameters in %d tensors, %lld chunks\n", (long long)n_params, n_tensors, (long long)n_chunks);
    if (use_arena) {
        int64_t n_local = -1;
        PO_CHECK(pipeoptim_plan_localize(plan, arena, stream, &n_local));
        std::printf("near-memory tile order for %lld parameters\n", (long long)n_local);
        if (n_local != n_params) { std::printf("every tensor's streams came from one arena call, all should be marked\n"); return 1; }
    }
    PO_CHECK(pipeoptim_step_predict(plan, &h, t, s, stream));
    HIP_OK(hipStreamSynchronize(stream));

    const double bc1 = 1.0 - std::pow(h.beta1, (double)t), bc2 = 1.0 - std::pow(h.beta2, (double)t);
    double worst = 0.0;
    int worst_ulp = 0, outside = 0;
    std::vector<std::vector<float>> W1(n_tensors), m1(n_tensors), v1(n_tensors);      // state after the fused call
    for (int i = 0; i < n_tensors; ++i) {
        const size_t n = (size_t)numel[i];
        if (n == 0) continue;
        std::vector<float> rW(n), rm(n), rv(n), rH(n);
        std::vector<uint16_t> rH16(n), gH16(n);
        W1[i].resize(n); m1[i].resize(n); v1[i].resize(n);
        if (po_oracle_step_predict(2, h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, 1, t, s, (long long)n, hW[i].data(),
                                   hg[i].data(), hm[i].data(), hv[i].data(), rW.data(), rm.data(), rv.data(), rH.data(),
                                   rH16.data(), 1) != 0) { std::printf("oracle rejected its arguments\n"); return 1; }
        HIP_OK(hipMemcpy(W1[i].data(), dW[i], n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(m1[i].data(), dm[i], n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(v1[i].data(), dv[i], n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(gH16.data(), dH[i], n * 2, hipMemcpyDeviceToHost));
        for (size_t k = 0; k < n; ++k) {
            // tolerance: 1e-6 of the magnitudes of the terms that make up each result
            const double aW = std::fabs(hW[i][k]), ag = std::fabs(hg[i][k]), am = std::fabs(hm[i][k]);
            const double m_abs = h.beta1 * am + (1 - h.beta1) * ag;
            const double d_abs = m_abs / bc1 / (std::sqrt((double)rv[k] / bc2) + h.eps) + h.weight_decay * aW;
            const double eW = std::fabs((double)W1[i][k] - rW[k]) / (aW + h.lr * d_abs + 1e-45);
            const double em = std::fabs((double)m1[i][k] - rm[k]) / (m_abs + 1e-45);
            const double ev = std::fabs((double)v1[i][k] - rv[k]) / ((double)rv[k] + 1e-45);
            worst = std::fmax(worst, std::fmax(eW, std::fmax(em, ev)));
            const int ulp = std::abs(bf16_order(gH16[k]) - bf16_order(rH16[k]));
            worst_ulp = ulp > worst_ulp ? ulp : worst_ulp;
            if (!bf16_within_band(gH16[k], rH[k], 1e-6 * (aW + s * h.lr * d_abs) + 1e-45)) ++outside;
        }
    }
    std::printf("fused call: worst fp32 error %.3e of scale (limit 1e-6); bf16 What at most %d ulp from the reference code, "
                "%d outside the rounding of the fp32 band\n", worst, worst_ulp, outside);
    if (!(worst <= 1e-6) || outside != 0) { std::printf("FAILED\n"); return 1; }

    // prediction alone from the state the fused call left, for the next stage's version difference
    PO_CHECK(pipeoptim_version_difference(4, 1, &s));        // s = 2
    PO_CHECK(pipeoptim_predict(plan, &h, t, s, stream));
    HIP_OK(hipStreamSynchronize(stream));
    worst_ulp = 0;
    outside = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const size_t n = (size_t)numel[i];
        if (n == 0) continue;
        std::vector<float> rH(n);
        std::vector<uint16_t> rH16(n), gH16(n);
        if (po_oracle_predict(2, h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, 1, t, s, (long long)n, W1[i].data(),
                              m1[i].data(), v1[i].data(), rH.data(), rH16.data(), 1) != 0) { std::printf("oracle rejected its arguments\n"); return 1; }
        HIP_OK(hipMemcpy(gH16.data(), dH[i], n * 2, hipMemcpyDeviceToHost));
        for (size_t k = 0; k < n; ++k) {
            const int ulp = std::abs(bf16_order(gH16[k]) - bf16_order(rH16[k]));
            worst_ulp = ulp > worst_ulp ? ulp : worst_ulp;
            const double aW = std::fabs(W1[i][k]);
            const double d_abs = std::fabs(m1[i][k]) / bc1 / (std::sqrt((double)v1[i][k] / bc2) + h.eps) + h.weight_decay * aW;
            if (!bf16_within_band(gH16[k], rH[k], 1e-6 * (aW + s * h.lr * d_abs) + 1e-45)) ++outside;
        }
    }
    std::printf("prediction-only call: bf16 What at most %d ulp from the reference code, %d outside the rounding of the fp32 band\n",
                worst_ulp, outside);
    if (outside != 0) { std::printf("FAILED\n"); return 1; }

    // error paths reachable from C: bad step index, optimizer without its state buffer
    if (pipeoptim_step_predict(plan, &h, 0, s, stream) != PO_EINVAL) { std::printf("t = 0 was accepted\n"); return 1; }
    PO_CHECK(pipeoptim_plan_destroy(plan));
    if (use_arena) PO_CHECK(pipeoptim_arena_destroy(arena));
    for (int i = 0; i < n_tensors && !use_arena; ++i) {
        if (!dW[i]) continue;
        HIP_OK(hipFree(dW[i])); HIP_OK(hipFree(const_cast<float*>(dg[i]))); HIP_OK(hipFree(dm[i])); HIP_OK(hipFree(dv[i])); HIP_OK(hipFree(dH[i]));
    }
    HIP_OK(hipStreamDestroy(stream));
    std::printf("c caller ok\n");
    return 0;
}

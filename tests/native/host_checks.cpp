// Host-only exercise of libpipeoptim's entry points that never touch the device, built with
// AddressSanitizer + UndefinedBehaviorSanitizer on the host side and run by tests/test_host_sanitizers.py.
// It checks return codes only; the value checks live in the Python tests.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pipeoptim.h"

#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, pipeoptim_last_error()); return 1; } } while (0)

int main()
{
    // Eq. 4
    int32_t s = -1;
    EXPECT(pipeoptim_version_difference(4, 0, &s) == PO_OK && s == 3);
    EXPECT(pipeoptim_version_difference(4, 4, &s) == PO_EINVAL);
    EXPECT(pipeoptim_version_difference(4, 0, nullptr) == PO_EINVAL);

    // coefficients
    po_hyper h{};
    h.opt = PO_ADAMW; h.decay_in_prediction = 1; h.lr = 1e-3; h.beta1 = 0.9; h.beta2 = 0.999; h.eps = 1e-8; h.weight_decay = 0.01;
    po_coeffs c{};
    EXPECT(pipeoptim_coefficients(&h, 1, 0, &c) == PO_OK && c.s_is_zero == 1);
    EXPECT(pipeoptim_coefficients(&h, INT64_MAX, INT32_MAX, &c) == PO_OK);
    EXPECT(pipeoptim_coefficients(&h, 0, 0, &c) == PO_EINVAL);
    EXPECT(pipeoptim_coefficients(nullptr, 1, 0, &c) == PO_EINVAL);
    EXPECT(std::strlen(pipeoptim_last_error()) > 0);

    // chunk table: exact-size buffers, count-only calls, a list with huge and empty tensors
    std::vector<int64_t> numel = {0, 1, 255, 256, 257, 65535, 65536, 65537, 0, 131072000, (int64_t(1) << 32) + 5};
    for (int64_t chunk : {int64_t(256), int64_t(4096), int64_t(65536), int64_t(1) << 30}) {
        int64_t n = -1;
        EXPECT(pipeoptim_chunk_table_build((int64_t)numel.size(), numel.data(), chunk, nullptr, 0, &n) == PO_OK && n > 0);
        std::vector<po_chunk> table((size_t)n);
        int64_t n2 = -1;
        EXPECT(pipeoptim_chunk_table_build((int64_t)numel.size(), numel.data(), chunk, table.data(), n, &n2) == PO_OK && n2 == n);
        std::vector<int64_t> covered(numel.size(), 0);
        for (const po_chunk& e : table) {
            EXPECT(e.tensor < numel.size());
            EXPECT(covered[e.tensor] == (int64_t)e.chunk * chunk);
            const int64_t end = (int64_t)(e.chunk + 1) * chunk;
            covered[e.tensor] = end < numel[e.tensor] ? end : numel[e.tensor];
        }
        for (size_t i = 0; i < numel.size(); ++i) EXPECT(covered[i] == numel[i]);
        if (n > 3) {   // a buffer that is too small is filled up to its capacity and no further
            std::vector<po_chunk> small(3);
            EXPECT(pipeoptim_chunk_table_build((int64_t)numel.size(), numel.data(), chunk, small.data(), 3, &n2) == PO_OK && n2 == n);
        }
    }

    // plan creation: every validation failure happens before the first device call
    po_plan* plan = nullptr;
    int64_t one[1] = {1024};
    float* W[1] = {reinterpret_cast<float*>(uintptr_t(1) << 20)};
    float* m[1] = {reinterpret_cast<float*>((uintptr_t(1) << 20) + 65536)};
    float* v[1] = {reinterpret_cast<float*>((uintptr_t(1) << 20) + 2 * 65536)};
    const float* g[1] = {reinterpret_cast<const float*>((uintptr_t(1) << 20) + 3 * 65536)};
    void* Wh[1] = {reinterpret_cast<void*>((uintptr_t(1) << 20) + 4 * 65536)};
    void* overlapping[1] = {reinterpret_cast<void*>((uintptr_t(1) << 20) + 4092)};
    void* odd[1] = {reinterpret_cast<void*>((uintptr_t(1) << 20) + 4 * 65536 + 1)};
    EXPECT(pipeoptim_plan_create(&plan, 1, one, W, g, m, v, overlapping, PO_WHAT_F32, nullptr) == PO_EINVAL && !plan);
    EXPECT(pipeoptim_plan_create(&plan, 1, one, W, g, m, v, odd, PO_WHAT_BF16, nullptr) == PO_EALIGN && !plan);
    EXPECT(pipeoptim_plan_create(&plan, 1, one, W, g, m, v, Wh, 9, nullptr) == PO_EINVAL && !plan);
    EXPECT(pipeoptim_plan_create(nullptr, 1, one, W, g, m, v, Wh, PO_WHAT_F32, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_plan_create_mixed(&plan, 1, one, W, reinterpret_cast<const void* const*>(g), 5, m, v, Wh, PO_WHAT_F32, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_plan_destroy(nullptr) == PO_OK);
    EXPECT(pipeoptim_step_predict(nullptr, &h, 1, 1, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_predict(nullptr, &h, 1, 1, nullptr) == PO_EINVAL);
    // near-memory arena and tile order: argument checks, and the order itself over every aligned run of 16
    po_arena* arena = nullptr;
    EXPECT(pipeoptim_arena_create(nullptr, 1 << 20) == PO_EINVAL);
    EXPECT(pipeoptim_arena_create(&arena, 0) == PO_EINVAL && !arena);
    EXPECT(pipeoptim_arena_create(&arena, (int64_t(1) << 40) + 1) == PO_EINVAL && !arena);
    EXPECT(pipeoptim_arena_destroy(nullptr) == PO_OK);
    void* ptr1[1] = {nullptr};
    EXPECT(pipeoptim_arena_alloc(nullptr, 1, one, ptr1) == PO_EINVAL);
    EXPECT(pipeoptim_arena_set_skew(nullptr, 0) == PO_EINVAL);
    int32_t half = 7;
    EXPECT(pipeoptim_arena_near_half(nullptr, nullptr, &half) == PO_EINVAL);
    EXPECT(pipeoptim_arena_info(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == PO_EINVAL);
    int64_t n_timed = 0, n_disagree = 0;
    EXPECT(pipeoptim_arena_check(nullptr, &n_timed, &n_disagree) == PO_EINVAL);
    EXPECT(pipeoptim_probe_copy_near(nullptr, nullptr, nullptr, 16384, 0, nullptr) == PO_EINVAL);
    uint32_t slot = 0;
    EXPECT(pipeoptim_local_slot(3, 7, 16, &slot) == PO_OK && slot == 10);
    EXPECT(pipeoptim_local_slot(12, 7, 16, &slot) == PO_OK && slot == 3);
    EXPECT(pipeoptim_local_slot(0, 8, 16, &slot) == PO_EINVAL);
    int32_t phase = 0;
    EXPECT(pipeoptim_plan_launch_phase(nullptr, &phase) == PO_EINVAL);
    int64_t n_local = -1;
    EXPECT(pipeoptim_plan_localize(nullptr, nullptr, nullptr, &n_local) == PO_EINVAL);
    EXPECT(pipeoptim_plan_local_params(nullptr, &n_local) == PO_EINVAL);
    EXPECT(pipeoptim_plan_learn_layout(nullptr, nullptr, &n_local) == PO_EINVAL);
    EXPECT(pipeoptim_plan_chunk_marks(nullptr, nullptr, 0, &n_local) == PO_EINVAL);
    double share = 0.0;
    EXPECT(pipeoptim_plan_near_share(nullptr, &share) == PO_EINVAL);
    {   // one stream of 4096 elements on a block boundary of a piece whose even blocks are near to half 1, weight 8
        const uint64_t stream = uint64_t(64) << 21, piece = uint64_t(64) << 21;
        const int32_t weight = 8;
        const int8_t half = 1;
        double near[2] = {-1.0, -1.0};
        EXPECT(pipeoptim_chunk_vote(1, &stream, &weight, 4096, 1, &piece, &half, near) == PO_OK && near[0] == 0.0 && near[1] == 8.0 * 4096);
        EXPECT(pipeoptim_chunk_vote(1, &stream, &weight, 4096, 1, &piece, &half, nullptr) == PO_EINVAL);
        EXPECT(pipeoptim_chunk_vote(6, &stream, &weight, 4096, 1, &piece, &half, near) == PO_EINVAL);
        const uint64_t lo[2] = {piece + 4, piece - 100}, hi[2] = {piece + (uint64_t(3) << 21) + 8, piece + 4};
        uint64_t run_lo[2] = {0, 0}, run_hi[2] = {0, 0};
        int64_t n_runs = -1;
        EXPECT(pipeoptim_whole_pieces(2, lo, hi, run_lo, run_hi, 2, &n_runs) == PO_OK && n_runs == 1 &&
               run_lo[0] == piece && run_hi[0] == piece + (uint64_t(3) << 21));
        EXPECT(pipeoptim_whole_pieces(2, lo, hi, run_lo, run_hi, 2, nullptr) == PO_EINVAL);
    }
    po_launch eff{};
    EXPECT(pipeoptim_plan_effective_launch(nullptr, PO_KERNEL_KIND_FUSED, PO_ADAM, &eff) == PO_EINVAL);
    for (int32_t first_half = 0; first_half < 2; ++first_half)
        for (uint32_t base = 0; base < 4096; base += 16) {
            uint32_t seen = 0;
            for (uint32_t k = 0; k < 16; ++k) {
                uint32_t tile = 0;
                EXPECT(pipeoptim_local_tile(base + k, first_half, &tile) == PO_OK);
                EXPECT(tile >= base && tile < base + 16);
                seen |= 1u << (tile - base);
            }
            EXPECT(seen == 0xFFFFu);
        }
    uint32_t tile = 0;
    EXPECT(pipeoptim_local_tile(0, 2, &tile) == PO_EINVAL);
    EXPECT(pipeoptim_local_tile(0, 0, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_probe_copy(nullptr, nullptr, 8, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_plan_set_pointers(nullptr, 1, Wh, nullptr) == PO_EINVAL);
    int64_t syncs = -1;
    EXPECT(pipeoptim_device_sync_count(&syncs) == PO_OK && syncs == 0);
    EXPECT(pipeoptim_device_sync_count(nullptr) == PO_EINVAL);

    // the allocation-free entry point: every limit and argument check comes before the first device call
    EXPECT(pipeoptim_step_predict_static(1, one, W, g, m, v, overlapping, PO_WHAT_F32, &h, 1, 1, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_step_predict_static(1, one, W, g, m, v, odd, PO_WHAT_BF16, &h, 1, 1, nullptr) == PO_EALIGN);
    EXPECT(pipeoptim_step_predict_static(1, one, W, g, m, nullptr, Wh, PO_WHAT_F32, &h, 1, 1, nullptr) == PO_EINVAL);   // AdamW needs v
    EXPECT(pipeoptim_step_predict_static(1, one, W, g, m, v, Wh, PO_WHAT_F32, &h, 0, 1, nullptr) == PO_EINVAL);         // t < 1
    EXPECT(pipeoptim_step_predict_static(1, one, W, g, m, v, Wh, PO_WHAT_F32, nullptr, 1, 1, nullptr) == PO_EINVAL);
    EXPECT(pipeoptim_step_predict_static(0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, PO_WHAT_F32, &h, 1, 1, nullptr) == PO_OK);
    {
        const int64_t too_many = PO_STATIC_MAX_TENSORS + 1;
        std::vector<int64_t> zeros((size_t)too_many, 0);
        std::vector<float*> nul((size_t)too_many, nullptr);
        std::vector<void*> nulv((size_t)too_many, nullptr);
        EXPECT(pipeoptim_step_predict_static(too_many, zeros.data(), nul.data(), const_cast<const float* const*>(nul.data()), nul.data(),
                                             nul.data(), nulv.data(), PO_WHAT_F32, &h, 1, 1, nullptr) == PO_EINVAL);
        EXPECT(std::strstr(pipeoptim_last_error(), "at most") != nullptr);
        // one tensor that needs more chunk-table entries than the static table holds (addresses far apart, never touched)
        int64_t huge[1] = {(int64_t)PO_STATIC_MAX_CHUNKS * 65536 + 1};
        float* bW[1] = {reinterpret_cast<float*>(uintptr_t(1) << 40)};
        const float* bg[1] = {reinterpret_cast<const float*>(uintptr_t(2) << 40)};
        float* bm[1] = {reinterpret_cast<float*>(uintptr_t(3) << 40)};
        float* bv[1] = {reinterpret_cast<float*>(uintptr_t(4) << 40)};
        void* bh[1] = {reinterpret_cast<void*>(uintptr_t(5) << 40)};
        EXPECT(pipeoptim_step_predict_static(1, huge, bW, bg, bm, bv, bh, PO_WHAT_BF16, &h, 1, 1, nullptr) == PO_EINVAL);
        EXPECT(std::strstr(pipeoptim_last_error(), "chunk-table entries") != nullptr);
    }

    std::printf("host checks passed\n");
    return 0;
}

// Internal declarations shared by the host side (pipeoptim.hip) and the kernels
// (step_predict_kernels.hip) of libpipeoptim.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pipeoptim.h"

// Per-tensor descriptor, resident in device memory for the life of a plan.
// 64 bytes so that a workgroup fetches one with a single scalar cache line.
struct alignas(64) po_tensor_desc {
    float* W;
    const void* g;     // fp32 or bf16, by the plan's grad_dtype
    float* m;
    float* v;          // nullptr in an SGDM-only plan
    void* What;
    int64_t numel;
    uint32_t flags;    // PO_DESC_VECTOR_OK: every base pointer is 16-byte aligned
    uint32_t pad;
};
static_assert(sizeof(po_tensor_desc) == 64, "descriptor layout");

enum : uint32_t { PO_DESC_VECTOR_OK = 1u };

// Launches the fused kernel for the given launch shape.  All shape limits were
// validated by the caller; returns the HIP status of the launch.
hipError_t po_launch_step_predict(int opt, int what_dtype, int grad_dtype, const po_launch& L,
                                  const po_tensor_desc* d_descs, const po_chunk* d_chunks,
                                  uint32_t n_chunks, const po_coeffs& c, hipStream_t stream);

// Same for the prediction-only kernel (reads W, m, v; writes What).
hipError_t po_launch_predict(int opt, int what_dtype, const po_launch& L, const po_tensor_desc* d_descs,
                             const po_chunk* d_chunks, uint32_t n_chunks, const po_coeffs& c, hipStream_t stream);

hipError_t po_launch_probe_copy(void* dst, const void* src, int64_t nbytes, hipStream_t stream);

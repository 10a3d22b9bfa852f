// pipeoptim_step_predict_static: the fused step + prediction for callers that cannot allocate.
//
// The plan-based call keeps its tensor descriptors and chunk table in device memory that pipeoptim_plan_create
// allocates.  Here the same two tables live in a fixed device array that is part of the library's image
// (`scratch` below): the descriptors travel to it inside kernel arguments (no copy from host memory, so no
// staging buffer either), the chunk table is built from them on the device, and the fused kernel then runs
// over the tables exactly as it does for a plan.  Nothing is allocated on the device and no allocating HIP routine is
// called (the argument checks use ordinary host heap memory).
#include <cstddef>
#include <cstring>
#include <mutex>
#include <vector>

#include "po_internal.h"

namespace {

constexpr size_t kDescBytes = (size_t)PO_STATIC_MAX_TENSORS * sizeof(po_tensor_desc);      // 64 KiB
constexpr size_t kChunkBytes = (size_t)PO_STATIC_MAX_CHUNKS * sizeof(po_chunk);            // 512 KiB
constexpr size_t kScratchBytes = kDescBytes + kChunkBytes;

}  // namespace

// Descriptors at offset 0, chunk table behind them.  One copy per GPU, kept until the process ends; every call on
// a GPU shares it.  In host code this name only stands for the symbol: the device address comes from
// hipGetSymbolAddress (scratch_of_current_device) and is what every kernel below is handed.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// The device address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(unsigned char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return po_fail(PO_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return po_fail(PO_EINVAL, "device %d: only devices 0..%d are supported here", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return po_fail(PO_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
    return PO_OK;
}

// Up to kBatch descriptors per launch ride in the kernel arguments (3 KiB of the 4 KiB a launch may carry).
constexpr uint32_t kBatch = 48;
struct alignas(64) WriteArgs {
    po_tensor_desc* dst;
    uint32_t count;
    uint32_t pad[13];
    po_tensor_desc d[kBatch];
};
static_assert(offsetof(WriteArgs, d) == 64 && sizeof(WriteArgs) == 64 + kBatch * 64, "argument block layout");
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define PO_CONSTANT __attribute__((address_space(4)))

// dst[0 .. count) = d[0 .. count), 16 bytes per lane and step.  count <= kBatch; dst has room for them.  The
// descriptors are read straight out of the kernel-argument segment (indexing the by-value argument with a lane's
// index would make the compiler copy it to per-lane memory first).
__global__ __launch_bounds__(256) void static_write_descs_kernel(WriteArgs a)
{
    const PO_CONSTANT char* args = (const PO_CONSTANT char*)__builtin_amdgcn_kernarg_segment_ptr();
    const PO_CONSTANT u32x4* src = (const PO_CONSTANT u32x4*)(args + offsetof(WriteArgs, d));
    u32x4* out = reinterpret_cast<u32x4*>(a.dst);
    const uint32_t pieces = (a.count < kBatch ? a.count : kBatch) * (uint32_t)(sizeof(po_tensor_desc) / 16);
    for (uint32_t i = threadIdx.x; i < pieces; i += blockDim.x) out[i] = src[i];
}

// The chunk table of the descriptors' ragged list, as the host builds it for a plan: tensors in list order, the
// chunks of a tensor in ascending order, empty tensors contribute none.  One workgroup of 1024 threads: thread i
// counts the chunks of tensor i, a scan over LDS turns the counts into first-entry positions, and the threads
// then share out the entries (the tensor of an entry by binary search in the positions).
// n_tensors <= 1024; n_chunks (what the host computed for the same list) <= the room behind `chunks`.
__global__ __launch_bounds__(1024) void static_build_chunks_kernel(const po_tensor_desc* descs, uint32_t n_tensors,
                                                                  int64_t chunk_elems, po_chunk* chunks, uint32_t n_chunks)
{
    __shared__ uint32_t scan[2][1024];
    __shared__ uint32_t first[1025];        // first[i] = position of tensor i's first entry; first[n_tensors] = total
    const uint32_t tid = threadIdx.x;
    uint32_t k = 0;
    if (tid < n_tensors) {
        const int64_t n = descs[tid].numel;
        k = n > 0 ? (uint32_t)((n + chunk_elems - 1) / chunk_elems) : 0u;
    }
    scan[0][tid] = k;
    __syncthreads();
    int cur = 0;
    for (uint32_t off = 1; off < 1024u; off <<= 1) {
        const uint32_t x = scan[cur][tid] + (tid >= off ? scan[cur][tid - off] : 0u);
        scan[cur ^ 1][tid] = x;
        __syncthreads();
        cur ^= 1;
    }
    first[tid + 1] = scan[cur][tid];          // inclusive sums
    if (tid == 0) first[0] = 0;
    __syncthreads();
    const uint32_t total = first[n_tensors] < n_chunks ? first[n_tensors] : n_chunks;
    for (uint32_t slot = tid; slot < total; slot += 1024u) {
        uint32_t lo = 0, hi = n_tensors;      // the tensor i with first[i] <= slot < first[i + 1]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (first[mid] <= slot) lo = mid; else hi = mid;
        }
        chunks[slot] = po_chunk{lo, slot - first[lo]};
    }
}

}  // namespace

extern "C" int pipeoptim_step_predict_static(int64_t n_tensors, const int64_t* numel, float* const* W,
                                             const float* const* g, float* const* m, float* const* v,
                                             void* const* What, int32_t what_dtype, const po_hyper* hyper,
                                             int64_t t, int32_t s, void* hip_stream)
try {
    po_coeffs c;
    int rc = pipeoptim_coefficients(hyper, t, s, &c);
    if (rc != PO_OK) return rc;
    if (n_tensors > PO_STATIC_MAX_TENSORS)
        return po_fail(PO_EINVAL, "pipeoptim_step_predict_static takes at most %d tensors (got %lld); use a plan",
                       PO_STATIC_MAX_TENSORS, (long long)n_tensors);
    const bool needs_m = hyper->opt != PO_RMSPROP && hyper->opt != PO_ADAGRAD;
    const bool needs_v = hyper->opt != PO_SGDM && hyper->opt != PO_NESTEROV;
    if (n_tensors > 0 && ((needs_m && !m) || (needs_v && !v)))
        return po_fail(PO_EINVAL, "optimizer %d needs the %s buffers", hyper->opt, needs_m && !m ? "m" : "v");
    std::vector<po_tensor_desc> descs;
    int64_t n_params = 0;
    rc = po_describe_list(n_tensors, numel, W, reinterpret_cast<const void* const*>(g), PO_GRAD_F32, m, v, What,
                          what_dtype, descs, &n_params, nullptr);
    if (rc != PO_OK) return rc;
    po_launch L = po_default_launch();
    int64_t n_chunks = 0;
    rc = pipeoptim_chunk_table_build(n_tensors, numel, L.chunk_elems, nullptr, 0, &n_chunks);
    if (rc != PO_OK) return rc;
    if (n_chunks > PO_STATIC_MAX_CHUNKS)
        return po_fail(PO_EINVAL, "pipeoptim_step_predict_static: the list needs %lld chunk-table entries of %lld elements, "
                       "the static table holds %d; use a plan", (long long)n_chunks, (long long)L.chunk_elems, PO_STATIC_MAX_CHUNKS);
    if (n_chunks == 0) return PO_OK;
    L.lds_bytes = po_auto_lds_bytes(PO_KERNEL_KIND_FUSED, hyper->opt, n_params, PO_LAYOUT_PLAIN);

    unsigned char* base = nullptr;
    rc = scratch_of_current_device(&base);
    if (rc != PO_OK) return rc;
    po_tensor_desc* d_descs = reinterpret_cast<po_tensor_desc*>(base);
    po_chunk* d_chunks = reinterpret_cast<po_chunk*>(base + kDescBytes);
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // every kernel below is enqueued on `stream`, so each sees what the one before it wrote
    for (int64_t at = 0; at < n_tensors; at += kBatch) {
        WriteArgs args;
        std::memset(&args, 0, sizeof args);
        args.dst = d_descs + at;
        args.count = (uint32_t)(n_tensors - at < (int64_t)kBatch ? n_tensors - at : (int64_t)kBatch);
        std::memcpy(args.d, descs.data() + at, (size_t)args.count * sizeof(po_tensor_desc));
        hipLaunchKernelGGL(static_write_descs_kernel, dim3(1), dim3(256), 0, stream, args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return po_fail(PO_EHIP, "launch of the descriptor kernel: %s", hipGetErrorString(e));
    }
    hipLaunchKernelGGL(static_build_chunks_kernel, dim3(1), dim3(1024), 0, stream, d_descs, (uint32_t)n_tensors,
                       L.chunk_elems, d_chunks, (uint32_t)n_chunks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return po_fail(PO_EHIP, "launch of the chunk-table kernel: %s", hipGetErrorString(e));
    e = po_launch_step_predict(hyper->opt, what_dtype, PO_GRAD_F32, L, d_descs, d_chunks, (uint32_t)n_chunks, c, stream,
                               0u, nullptr, false);
    if (e != hipSuccess) return po_fail(PO_EHIP, "launch of the fused step+predict kernel: %s", hipGetErrorString(e));
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_step_predict_static: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_step_predict_static: unexpected exception"); }

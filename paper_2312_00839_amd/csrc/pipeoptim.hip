// Host side of libpipeoptim: the C ABI declared in include/pipeoptim.h.
//
// Holds the plan (tensor descriptors + chunk table, mirrored on the device and
// uploaded on the caller's stream from pinned staging memory), the
// derivation of the fp32 kernel coefficients from the double hyper-parameters
// (bias corrections of paper Table 1 in fp64), the version-difference rule of
// paper Eq. 4, and argument validation.  The kernels live in
// step_predict_kernels.hip.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <utility>
#include <vector>

#include "po_internal.h"

namespace {
thread_local char g_err[512] = "";
}

int po_fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

namespace {

int fail_hip(hipError_t e, const char* what)
{
    return po_fail(PO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr int64_t kMaxChunkElems = int64_t(1) << 30;

int check_launch(const po_launch& L)
{
    if (L.block != 64 && L.block != 128 && L.block != 256) return po_fail(PO_EINVAL, "launch.block must be 64, 128 or 256");
    if (L.lds_bytes < PO_LDS_AUTO || L.lds_bytes > 65536) return po_fail(PO_EINVAL, "launch.lds_bytes must be 0..65536, or -1 (chosen per call)");
    const int64_t tile = (int64_t)L.block * 4;
    const int64_t ratio = L.chunk_elems > 0 ? L.chunk_elems / tile : 0;
    if (L.chunk_elems <= 0 || L.chunk_elems > kMaxChunkElems || L.chunk_elems % tile != 0 || (ratio & (ratio - 1)) != 0)
        return po_fail(PO_EINVAL, "launch.chunk_elems must be block*4 (%lld) times a power of two, at most 2^30",
                    (long long)tile);
    return PO_OK;
}

// one workgroup per tile: the grid must fit HIP's limit
int check_grid(const po_launch& L, int64_t n_chunks)
{
    const int64_t tiles = L.chunk_elems / ((int64_t)L.block * 4);
    if (n_chunks > 0 && tiles > (int64_t(0x7FFFFFF8) / n_chunks))
        return po_fail(PO_EINVAL, "grid of %lld chunks x %lld tiles exceeds 2^31 workgroups; raise block or lower chunk_elems",
                    (long long)n_chunks, (long long)tiles);
    return PO_OK;
}

int build_chunks(int64_t n_tensors, const int64_t* numel, int64_t chunk_elems, po_chunk* out, int64_t capacity,
                 int64_t* n_chunks)
{
    if (n_tensors < 0) return po_fail(PO_EINVAL, "n_tensors < 0");
    if (n_tensors > 0 && !numel) return po_fail(PO_EINVAL, "numel is NULL");
    if (chunk_elems <= 0 || chunk_elems > kMaxChunkElems) return po_fail(PO_EINVAL, "chunk_elems out of range");
    if (n_tensors > (int64_t)UINT32_MAX) return po_fail(PO_EINVAL, "too many tensors");
    if (capacity < 0 || (capacity > 0 && !out)) return po_fail(PO_EINVAL, "bad output buffer");
    if (!n_chunks) return po_fail(PO_EINVAL, "n_chunks is NULL");
    int64_t total = 0;
    for (int64_t i = 0; i < n_tensors; ++i) {
        if (numel[i] < 0) return po_fail(PO_EINVAL, "numel[%lld] < 0", (long long)i);
        const int64_t k = (numel[i] + chunk_elems - 1) / chunk_elems;
        if (k > (int64_t)UINT32_MAX) return po_fail(PO_EINVAL, "tensor %lld needs too many chunks", (long long)i);
        for (int64_t j = 0; j < k; ++j, ++total)
            if (total < capacity) out[total] = po_chunk{(uint32_t)i, (uint32_t)j};
    }
    if (total > (int64_t)UINT32_MAX) return po_fail(PO_EINVAL, "chunk table too long; raise chunk_elems");
    *n_chunks = total;
    return PO_OK;
}

bool finite_d(double x) { return std::isfinite(x); }

}  // namespace

// The library waits for the whole device in very few places (arena set-up, and as a fallback when a stream a
// plan remembers no longer exists); every such wait goes through here so that it can be counted.
static std::atomic<int64_t> g_device_syncs{0};

hipError_t po_device_sync()
{
    g_device_syncs.fetch_add(1, std::memory_order_relaxed);
    return hipDeviceSynchronize();
}

struct po_plan {
    int64_t n_tensors = 0;
    int64_t n_params = 0;
    int64_t n_unaligned = 0;
    int64_t n_local_params = 0;   // parameters of tensors that run in the near-memory tile order
    double near_bytes = 0.0;      // of the fused call's bytes per launch, those known to be near beyond the plain order's half
    int32_t what_dtype = PO_WHAT_F32;
    int32_t grad_dtype = PO_GRAD_F32;
    bool has_v = false;
    bool has_m = false;
    int device = 0;
    po_launch launch{};           // fused kernel
    po_launch predict_launch{};   // prediction-only kernel; chunk_elems always equals launch.chunk_elems
    std::vector<int64_t> numel;
    std::vector<po_tensor_desc> descs;    // host mirror
    std::vector<po_chunk> chunks;         // host mirror (tensor indices without marks)
    // Near-memory order decided chunk by chunk from the learnt die layout of caller-placed buffers
    // (pipeoptim_plan_learn_layout): -1 plain order, 0 / 1 the XCC half near to the chunk's first 8 KiB blocks.
    // Valid (and uploaded in the chunk table's top bits) only while chunk_marks_valid.
    std::vector<int8_t> chunk_mark;
    bool chunk_marks_valid = false;
    po_tensor_desc* d_descs = nullptr;
    po_chunk* d_chunks = nullptr;
    int64_t d_chunks_capacity = 0;
    // Pinned staging memory for the asynchronous table uploads.  Descriptors: two buffers used in turn, each
    // guarded by the event recorded behind its last copy, so that pipeoptim_plan_set_pointers may be called again
    // while the previous upload is still queued.  Chunk table: one buffer (it is rewritten only by
    // pipeoptim_plan_set_launch, which waits for the plan's streams first).
    po_tensor_desc* h_descs[2] = {nullptr, nullptr};
    hipEvent_t ev_descs[2] = {nullptr, nullptr};
    bool ev_recorded[2] = {false, false};
    int next_staging = 0;
    po_chunk* h_chunks = nullptr;
    int64_t h_chunks_capacity = 0;
    // The latest upload: its stream, and the event behind it.  A launch on any other stream first makes that
    // stream wait for the event; `ordered_stream` is the stream known to be ordered behind the upload already.
    hipEvent_t ev_upload = nullptr;            // one of ev_descs, or ev_chunks
    hipEvent_t ev_chunks = nullptr;
    hipStream_t upload_stream = nullptr;
    bool uploaded = false;                     // an upload was ever enqueued (upload_stream is meaningful)
    mutable hipStream_t ordered_stream = nullptr;
    mutable hipStream_t last_launch_stream = nullptr;
    mutable bool launched = false;
    // Pinned host word (64 bytes allocated) that workgroup 0 of every launch in the near-memory tile order writes
    // its XCC id to: the XCC on which the stream's hardware queue starts its launches.  The next call passes the
    // value it finds there to its kernel.  Allocated by pipeoptim_plan_localize, nullptr before.
    uint32_t* h_phase = nullptr;
};

namespace {

// All buffers of a stage must be pairwise disjoint: W, m, v are rewritten in place while other
// workgroups still read their own parts, and What is written from values read earlier.
int check_disjoint(const std::vector<po_tensor_desc>& descs, int grad_dtype, int what_dtype)
{
    struct Range { uintptr_t lo, hi; int64_t tensor; char kind; };
    std::vector<Range> r;
    r.reserve(descs.size() * 5);
    const size_t gsz = grad_dtype == PO_GRAD_BF16 ? 2 : 4, hsz = what_dtype == PO_WHAT_BF16 ? 2 : 4;
    for (size_t i = 0; i < descs.size(); ++i) {
        const po_tensor_desc& d = descs[i];
        const size_t n = (size_t)d.numel;
        if (n == 0) continue;
        r.push_back({(uintptr_t)d.W, (uintptr_t)d.W + n * 4, (int64_t)i, 'W'});
        r.push_back({(uintptr_t)d.g, (uintptr_t)d.g + n * gsz, (int64_t)i, 'g'});
        if (d.m) r.push_back({(uintptr_t)d.m, (uintptr_t)d.m + n * 4, (int64_t)i, 'm'});
        if (d.v) r.push_back({(uintptr_t)d.v, (uintptr_t)d.v + n * 4, (int64_t)i, 'v'});
        r.push_back({(uintptr_t)d.What, (uintptr_t)d.What + n * hsz, (int64_t)i, 'h'});
    }
    std::sort(r.begin(), r.end(), [](const Range& a, const Range& b) { return a.lo < b.lo; });
    for (size_t k = 1; k < r.size(); ++k)
        if (r[k].lo < r[k - 1].hi)
            return po_fail(PO_EINVAL, "buffers overlap: %c of tensor %lld and %c of tensor %lld (h = What)", r[k - 1].kind,
                        (long long)r[k - 1].tensor, r[k].kind, (long long)r[k].tensor);
    return PO_OK;
}

// Recomputes every descriptor's flags from its pointers (this drops near-memory marks: they hold for the
// addresses pipeoptim_plan_localize looked at, not for new ones).  Returns the tensors on the scalar path.
int64_t refresh_flags(std::vector<po_tensor_desc>& descs)
{
    int64_t n_unaligned = 0;
    for (auto& d : descs) {
        uintptr_t bits = (uintptr_t)d.W | (uintptr_t)d.g | (uintptr_t)d.m | (uintptr_t)d.v | (uintptr_t)d.What;
        d.flags = (bits & 15u) == 0 ? PO_DESC_VECTOR_OK : 0u;
        if (!d.flags && d.numel > 0) ++n_unaligned;
    }
    return n_unaligned;
}

}  // namespace

// Validates a ragged list as the plan and the allocation-free entry point take it, and turns it into
// descriptors (flags set).  Nothing here touches the device.
int po_describe_list(int64_t n_tensors, const int64_t* numel, float* const* W, const void* const* g, int32_t grad_dtype,
                     float* const* m, float* const* v, void* const* What, int32_t what_dtype,
                     std::vector<po_tensor_desc>& descs, int64_t* n_params, int64_t* n_unaligned)
{
    if (n_tensors < 0) return po_fail(PO_EINVAL, "n_tensors < 0");
    if (n_tensors > (int64_t)PO_CHUNK_TENSOR_MASK) return po_fail(PO_EINVAL, "too many tensors (at most 2^30 - 1)");
    if (n_tensors > 0 && (!numel || !W || !g || !What)) return po_fail(PO_EINVAL, "a required pointer array is NULL");
    if (n_tensors > 0 && !m && !v) return po_fail(PO_EINVAL, "a stage needs at least one of m and v");
    if (what_dtype != PO_WHAT_F32 && what_dtype != PO_WHAT_BF16) return po_fail(PO_EINVAL, "unknown what_dtype %d", what_dtype);
    if (grad_dtype != PO_GRAD_F32 && grad_dtype != PO_GRAD_BF16) return po_fail(PO_EINVAL, "unknown grad_dtype %d", grad_dtype);
    const uintptr_t what_mask = what_dtype == PO_WHAT_BF16 ? 1u : 3u;
    const uintptr_t grad_mask = grad_dtype == PO_GRAD_BF16 ? 1u : 3u;
    int64_t total = 0;
    for (int64_t i = 0; i < n_tensors; ++i) {
        if (numel[i] < 0) return po_fail(PO_EINVAL, "numel[%lld] < 0", (long long)i);
        if (numel[i] == 0) continue;
        if (!W[i] || !g[i] || !What[i] || (m && !m[i]) || (v && !v[i]))
            return po_fail(PO_EINVAL, "tensor %lld has a NULL buffer", (long long)i);
        if (((uintptr_t)W[i] | (m ? (uintptr_t)m[i] : 0) | (v ? (uintptr_t)v[i] : 0)) & 3u)
            return po_fail(PO_EALIGN, "tensor %lld: fp32 buffer not 4-byte aligned", (long long)i);
        if ((uintptr_t)g[i] & grad_mask) return po_fail(PO_EALIGN, "tensor %lld: g not aligned to its element", (long long)i);
        if ((uintptr_t)What[i] & what_mask) return po_fail(PO_EALIGN, "tensor %lld: What not aligned to its element", (long long)i);
        total += numel[i];
    }
    descs.resize((size_t)n_tensors);
    for (int64_t i = 0; i < n_tensors; ++i) {
        po_tensor_desc& d = descs[(size_t)i];
        d.W = W[i]; d.g = g[i]; d.m = m ? m[i] : nullptr; d.v = v ? v[i] : nullptr; d.What = What[i];
        d.numel = numel[i]; d.flags = 0; d.pad = 0;
    }
    const int rc = check_disjoint(descs, grad_dtype, what_dtype);
    if (rc != PO_OK) return rc;
    const int64_t un = refresh_flags(descs);
    if (n_params) *n_params = total;
    if (n_unaligned) *n_unaligned = un;
    return PO_OK;
}

// Occupancy cap (unused LDS per single-wave workgroup; a CU has 160 KiB) by kernel, number of state streams and
// stage size, as measured on MI355X.  The streaming pattern runs fastest with roughly 72-75 KB of loads and
// stores in flight per CU: fewer and the latency is not hidden, more and the DRAM pages of the 4-8 concurrent
// streams evict each other.  A fused Adam/AdamW tile moves 7.5 KB (10 workgroups per CU), a one-state
// optimizer's 5.5-6 KB (13), a prediction tile 3.5 KB (20) or 2.5 KB (26).  Smaller stages, whose launch is
// dominated by ramp-up and ramp-down, like a few more.
int32_t po_auto_lds_bytes(int kernel, int opt, int64_t n_params, int layout)
{
    const bool two_state = opt == PO_ADAM || opt == PO_ADAMW;
    const bool large = n_params >= (int64_t(1) << 27), mid = n_params >= (int64_t(1) << 25);
    // a learnt layout (caller-placed buffers, about two thirds of the traffic near) likes the arena's cap for the fused
    // two-state kernel from mid-sized stages up (config 3's shapes: 6.62 -> 6.71 TB/s) and the plain caps otherwise
    if (layout == PO_LAYOUT_LEARNT) layout = (kernel == PO_KERNEL_KIND_FUSED && two_state && mid) ? PO_LAYOUT_ARENA : PO_LAYOUT_PLAIN;
    const bool local = layout == PO_LAYOUT_ARENA;
    if (local) {
        // every XCC on its own die's memory: shorter latency, no shared link; the sweeps put the optimum at 10
        // workgroups per CU for the fused two-state kernel at every size from 64 M parameters up, at 12-13 for the
        // one-state kernels, and at 16 (20 on mid-sized stages) for the prediction kernel
        if (kernel == PO_KERNEL_KIND_PREDICT) return two_state ? (large ? 10240 : 8192) : (large ? 7168 : 6144);
        if (two_state) return mid ? 16384 : 12288;
        return 12288;
    }
    if (kernel == PO_KERNEL_KIND_PREDICT) return two_state ? 8192 : 6144;
    if (two_state) return large ? 16384 : mid ? 14336 : 10240;
    return mid ? 12288 : 10240;
}

// Default launch shape, as measured on MI355X: single-wave workgroups, one 256-element tile each, and an
// occupancy cap chosen per call (see above).  Bigger workgroups measured slower at every stage size.
po_launch po_default_launch()
{
    po_launch L{};
    L.block = 64;
    L.lds_bytes = PO_LDS_AUTO;
    L.chunk_elems = 65536;
    return L;
}

namespace {

// The plan's tables and the caller's buffers live on the device that was current at plan creation.
int check_device(const po_plan* p)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev != p->device)
        return po_fail(PO_EINVAL, "plan belongs to device %d but device %d is current", p->device, dev);
    return PO_OK;
}

// Does the plan hold the state buffers this optimizer updates?
int check_state(const po_plan* p, int opt)
{
    const bool needs_m = opt != PO_RMSPROP && opt != PO_ADAGRAD;
    const bool needs_v = opt != PO_SGDM && opt != PO_NESTEROV;
    if (needs_m && !p->has_m) return po_fail(PO_EINVAL, "optimizer %d needs a plan created with m", opt);
    if (needs_v && !p->has_v) return po_fail(PO_EINVAL, "optimizer %d needs a plan created with v", opt);
    return PO_OK;
}

// The launch shape a call runs with: lds_bytes == PO_LDS_AUTO resolved for the optimizer in use.
po_launch resolve_launch(const po_plan* p, const po_launch& L, int kernel, int opt)
{
    po_launch R = L;
    const bool local = p->n_local_params * 2 >= p->n_params && p->n_local_params > 0;
    const int layout = !local ? PO_LAYOUT_PLAIN : p->chunk_marks_valid ? PO_LAYOUT_LEARNT : PO_LAYOUT_ARENA;
    if (R.lds_bytes == PO_LDS_AUTO) {
        R.lds_bytes = po_auto_lds_bytes(kernel, opt, p->n_params, layout);
        // an fp32 What makes the fused two-state tile 8 KB instead of 7.5: in the near-memory orders 8 workgroups per
        // CU are then ahead of 10 (config 5's shapes, arena 6.95 -> 6.98 TB/s, learnt 6.85 -> 6.93; config 4's likewise)
        if (layout != PO_LAYOUT_PLAIN && kernel == PO_KERNEL_KIND_FUSED && p->what_dtype == PO_WHAT_F32 && R.lds_bytes == 16384)
            R.lds_bytes = 18432;
    }
    return R;
}

// Waits for the two streams the plan used last: a launch there may still read the tables.  If one of them no
// longer exists (the caller destroyed it), waits for the device instead.
int wait_for_plan_streams(const po_plan* p)
{
    hipError_t e = hipSuccess;
    if (p->launched) e = hipStreamSynchronize(p->last_launch_stream);
    if (e == hipSuccess && p->uploaded && (!p->launched || p->upload_stream != p->last_launch_stream)) e = hipStreamSynchronize(p->upload_stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        e = po_device_sync();
    }
    if (e != hipSuccess) return fail_hip(e, "waiting for the plan's streams");
    return PO_OK;
}

// Uploads form one chain: an upload on another stream than the previous one first makes its stream wait for the
// previous upload, so that the copies land in call order and the latest event stands for all of them.
hipError_t chain_behind_previous_upload(const po_plan* p, hipStream_t stream)
{
    if (p->ev_upload && stream != p->upload_stream) return hipStreamWaitEvent(stream, p->ev_upload, 0);
    return hipSuccess;
}

// Copies the host descriptors into the staging buffer whose turn it is and enqueues its upload on `stream`.
int upload_descs(po_plan* p, hipStream_t stream)
{
    if (p->n_tensors == 0) return PO_OK;
    const int k = p->next_staging;
    hipError_t e = hipSuccess;
    if (p->ev_recorded[k]) e = hipEventSynchronize(p->ev_descs[k]);      // the copy out of this buffer two uploads ago
    if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize(staging buffer)");
    e = chain_behind_previous_upload(p, stream);
    if (e != hipSuccess) return fail_hip(e, "hipStreamWaitEvent(previous upload)");
    const size_t bytes = (size_t)p->n_tensors * sizeof(po_tensor_desc);
    std::memcpy(p->h_descs[k], p->descs.data(), bytes);
    e = hipMemcpyAsync(p->d_descs, p->h_descs[k], bytes, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync(tensor descriptors)");      // nothing was enqueued
    // From here on the device table WILL change, so the call must not fail any more: if the event cannot be
    // recorded, wait for the copy instead (then neither the staging buffer nor another stream needs the event).
    e = hipEventRecord(p->ev_descs[k], stream);
    p->ev_recorded[k] = (e == hipSuccess);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        (void)hipStreamSynchronize(stream);
    }
    p->next_staging = k ^ 1;
    p->ev_upload = p->ev_recorded[k] ? p->ev_descs[k] : nullptr;
    p->uploaded = true;
    p->upload_stream = stream;
    p->ordered_stream = stream;
    return PO_OK;
}

// Rebuilds the chunk table for the plan's chunk_elems and enqueues its upload on `stream`.  The caller has made
// sure that no launch still reads the old table and that the previous upload out of h_chunks is done.
int upload_chunks(po_plan* p, hipStream_t stream)
{
    int64_t n = 0;
    int rc = build_chunks(p->n_tensors, p->numel.data(), p->launch.chunk_elems, nullptr, 0, &n);
    if (rc != PO_OK) return rc;
    p->chunks.resize((size_t)n);
    rc = build_chunks(p->n_tensors, p->numel.data(), p->launch.chunk_elems, p->chunks.data(), n, &n);
    if (rc != PO_OK) return rc;
    if (n > p->d_chunks_capacity) {
        if (p->d_chunks) (void)hipFree(p->d_chunks);
        p->d_chunks = nullptr;
        p->d_chunks_capacity = 0;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&p->d_chunks), (size_t)n * sizeof(po_chunk));
        if (e != hipSuccess) return po_fail(PO_ENOMEM, "hipMalloc(chunk table, %lld entries): %s", (long long)n,
                                         hipGetErrorString(e));
        p->d_chunks_capacity = n;
    }
    if (n > p->h_chunks_capacity) {
        if (p->h_chunks) (void)hipHostFree(p->h_chunks);
        p->h_chunks = nullptr;
        p->h_chunks_capacity = 0;
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&p->h_chunks), (size_t)n * sizeof(po_chunk), hipHostMallocDefault);
        if (e != hipSuccess) return po_fail(PO_ENOMEM, "hipHostMalloc(chunk table staging): %s", hipGetErrorString(e));
        p->h_chunks_capacity = n;
    }
    if (p->chunk_marks_valid && (int64_t)p->chunk_mark.size() != n) p->chunk_marks_valid = false;
    if (n > 0) {
        std::memcpy(p->h_chunks, p->chunks.data(), (size_t)n * sizeof(po_chunk));
        if (p->chunk_marks_valid)
            for (int64_t k = 0; k < n; ++k)
                if (p->chunk_mark[(size_t)k] >= 0)
                    p->h_chunks[k].tensor |= PO_CHUNK_LOCAL | (p->chunk_mark[(size_t)k] ? PO_CHUNK_HALF1 : 0u);
        hipError_t e = chain_behind_previous_upload(p, stream);
        if (e != hipSuccess) return fail_hip(e, "hipStreamWaitEvent(previous upload)");
        e = hipMemcpyAsync(p->d_chunks, p->h_chunks, (size_t)n * sizeof(po_chunk), hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync(chunk table)");
        e = hipEventRecord(p->ev_chunks, stream);
        if (e != hipSuccess) {                       // as for the descriptors: wait for the copy instead
            (void)hipGetLastError();
            (void)hipStreamSynchronize(stream);
        }
        p->ev_upload = (e == hipSuccess) ? p->ev_chunks : nullptr;
        p->uploaded = true;
        p->upload_stream = stream;
        p->ordered_stream = stream;
    }
    return PO_OK;
}

// Before a launch on `stream`: if the latest table upload went to another stream, make `stream` wait for it.
hipError_t order_behind_upload(const po_plan* p, hipStream_t stream)
{
    if (p->ev_upload && stream != p->ordered_stream) {
        hipError_t e = hipStreamWaitEvent(stream, p->ev_upload, 0);
        if (e != hipSuccess) return e;
        p->ordered_stream = stream;
    }
    p->last_launch_stream = stream;
    p->launched = true;
    return hipSuccess;
}

}  // namespace

namespace {

constexpr uintptr_t kPiece = uintptr_t(2) << 20;       // what the driver backs large allocations with; see near_arena.hip

// The fp32 streams of a tensor and what each weighs in the fused call's traffic, in bytes moved per element.
struct VotingStream { uintptr_t base; int weight; };
int voting_streams(const po_plan* p, const po_tensor_desc& d, VotingStream out[5])
{
    int k = 0;
    out[k++] = {(uintptr_t)d.W, 8};
    if (p->grad_dtype == PO_GRAD_F32) out[k++] = {(uintptr_t)d.g, 4};
    if (d.m) out[k++] = {(uintptr_t)d.m, 8};
    if (d.v) out[k++] = {(uintptr_t)d.v, 8};
    if (p->what_dtype == PO_WHAT_F32) out[k++] = {(uintptr_t)d.What, 4};
    return k;
}

// What timing found out about the memory under a plan's buffers: for the 2 MiB pieces of some address ranges, the XCC
// half that is near to the piece's 8 KiB blocks with address bit 13 clear (-1: could not be told).
struct PieceLayout {
    std::vector<std::pair<uintptr_t, uintptr_t>> ranges;      // sorted, disjoint, piece-aligned [lo, hi)
    std::vector<std::vector<int8_t>> answer;                  // per range, per piece
    int at(uintptr_t addr) const                              // -1: not timed or not decided
    {
        auto it = std::upper_bound(ranges.begin(), ranges.end(), std::make_pair(addr, ~uintptr_t(0)));
        if (it == ranges.begin()) return -1;
        --it;
        if (addr < it->first || addr >= it->second) return -1;
        return answer[(size_t)(it - ranges.begin())][(size_t)((addr - it->first) / kPiece)];
    }
};

// The runs of whole, 2 MiB-aligned pieces every byte of which lies in at least one of the byte ranges [lo, hi)
// (sorted, disjoint).  Ranges that touch or overlap count as one; a gap of a single byte ends a run.
std::vector<std::pair<uintptr_t, uintptr_t>> whole_pieces_inside(std::vector<std::pair<uintptr_t, uintptr_t>> bytes)
{
    std::sort(bytes.begin(), bytes.end());
    std::vector<std::pair<uintptr_t, uintptr_t>> merged, pieces;
    for (const auto& r : bytes) {
        if (r.first >= r.second) continue;
        if (!merged.empty() && r.first <= merged.back().second) merged.back().second = std::max(merged.back().second, r.second);
        else merged.push_back(r);
    }
    for (const auto& r : merged) {
        const uintptr_t lo = (r.first + kPiece - 1) / kPiece * kPiece, hi = r.second / kPiece * kPiece;
        if (lo < hi) pieces.push_back({lo, hi});
    }
    return pieces;
}

// Times every whole 2 MiB piece inside the union of the plan's fp32 streams.  Every byte of every stream is readable
// device memory, so such a piece may be read wherever it lies (buffers that a caching allocator placed back to
// back merge into one range).  Waits for the device, several times.
int time_pieces_under(const po_plan* p, PieceLayout& out)
{
    std::vector<std::pair<uintptr_t, uintptr_t>> bytes;       // exact byte ranges of the streams
    for (const po_tensor_desc& d : p->descs) {
        if (d.numel == 0) continue;
        VotingStream st[5];
        const int ns = voting_streams(p, d, st);
        for (int k = 0; k < ns; ++k) bytes.push_back({st[k].base, st[k].base + (uintptr_t)d.numel * 4});
    }
    out.ranges = whole_pieces_inside(bytes);
    out.answer.resize(out.ranges.size());
    for (size_t k = 0; k < out.ranges.size(); ++k) {
        const size_t n = (size_t)((out.ranges[k].second - out.ranges[k].first) / kPiece);
        out.answer[k].assign(n, (int8_t)-1);
        const int rc = po_probe_layout(reinterpret_cast<const void*>(out.ranges[k].first), n, out.answer[k].data());
        if (rc != PO_OK) return rc;
    }
    return PO_OK;
}

// One chunk-table entry's vote.  Under mark h the XCCs of half h take the first 8 KiB of every 16 KiB of the chunk's
// elements.  With a stream's part of the chunk starting o bytes into an 8 KiB block whose near half is x, 8192 - o
// of those bytes lie in that block and o in the next one (near to the other half), and the second 8 KiB likewise:
// the stream's bytes vote (8192 - o) : o for x.  o = 0 for buffers on a block boundary (any large allocation); a
// stream 4 KiB off has no say, being half near and half far under either order.  A chunk that straddles two pieces
// votes with each part's own layout.  near[h] = bytes of the call's traffic that mark h would make near; `begin` =
// byte offset of the chunk inside each of the `ns` streams.
void chunk_vote(const VotingStream* st, int ns, uintptr_t begin, int64_t elems, const PieceLayout& pieces, double near[2])
{
    near[0] = near[1] = 0.0;
    for (int j = 0; j < ns; ++j) {
        const uintptr_t a0 = st[j].base + begin, a1 = a0 + (uintptr_t)elems * 4;
        const double o = (double)(a0 % 8192u) / 8192.0;
        const int first_block_odd = (int)((a0 >> 13) & 1u);
        for (uintptr_t at = a0; at < a1;) {
            const uintptr_t stop = std::min(a1, (at / kPiece + 1) * kPiece);
            const int even_blocks_near = pieces.at(at);
            if (even_blocks_near >= 0) {
                const int x = first_block_odd ^ even_blocks_near;
                const double traffic = (double)(stop - at) * (st[j].weight / 4.0);
                near[x] += traffic * (1.0 - o);
                near[1 - x] += traffic * o;
            }
            at = stop;
        }
    }
}

}  // namespace

extern "C" {

const char* pipeoptim_last_error(void) { return g_err; }

int pipeoptim_device_sync_count(int64_t* count)
{
    if (!count) return po_fail(PO_EINVAL, "count is NULL");
    *count = g_device_syncs.load(std::memory_order_relaxed);
    return PO_OK;
}

int pipeoptim_version_difference(int32_t D, int32_t rank, int32_t* s_out)
{
    if (!s_out) return po_fail(PO_EINVAL, "s_out is NULL");
    if (D < 1 || rank < 0 || rank >= D) return po_fail(PO_EINVAL, "need 0 <= rank < D (D=%d, rank=%d)", D, rank);
    *s_out = D - rank - 1;   // paper Eq. 4
    return PO_OK;
}

int pipeoptim_coefficients(const po_hyper* h, int64_t t, int32_t s, po_coeffs* out)
{
    if (!h || !out) return po_fail(PO_EINVAL, "hyper or out is NULL");
    if (h->opt < PO_SGDM || h->opt > PO_ADAGRAD) return po_fail(PO_EINVAL, "unknown optimizer %d", h->opt);
    if (t < 1) return po_fail(PO_EINVAL, "t must be >= 1 (got %lld): steps are 1-based", (long long)t);
    if (s < 0) return po_fail(PO_EINVAL, "s must be >= 0 (got %d)", s);
    if (!finite_d(h->lr) || !finite_d(h->eps) || !finite_d(h->weight_decay) || !finite_d(h->beta1) || !finite_d(h->beta2))
        return po_fail(PO_EINVAL, "non-finite hyper-parameter");
    if (h->eps < 0) return po_fail(PO_EINVAL, "eps must be >= 0");
    po_coeffs c{};
    if (h->opt == PO_SGDM) {
        if (h->beta1 < 0 || h->beta1 >= 1) return po_fail(PO_EINVAL, "momentum must be in [0,1)");
        if (h->beta2 < 0 || h->beta2 > 1) return po_fail(PO_EINVAL, "dampening must be in [0,1]");
        c.beta1 = (float)h->beta1;
        c.grad_scale = (float)(1.0 - h->beta2);
        c.beta2 = 0.f;
        c.one_m_beta2 = 0.f;
        c.inv_bc1 = 1.f;
        c.inv_sqrt_bc2 = 1.f;
        c.eps = 0.f;
        c.wd_coupled = (float)h->weight_decay;
    } else if (h->opt == PO_NESTEROV) {
        if (h->beta1 < 0 || h->beta1 >= 1) return po_fail(PO_EINVAL, "momentum must be in [0,1)");
        c.beta1 = (float)h->beta1;
        c.grad_scale = 1.f;
        c.inv_bc1 = 1.f;
        c.inv_sqrt_bc2 = 1.f;
        c.wd_coupled = (float)h->weight_decay;
    } else if (h->opt == PO_RMSPROP || h->opt == PO_ADAGRAD) {
        // one kernel serves both: v' = beta2*v + one_m_beta2*g~^2, Adagrad being the case (1, 1)
        if (h->opt == PO_RMSPROP && (h->beta2 < 0 || h->beta2 >= 1)) return po_fail(PO_EINVAL, "alpha must be in [0,1)");
        c.beta2 = h->opt == PO_RMSPROP ? (float)h->beta2 : 1.f;
        c.one_m_beta2 = h->opt == PO_RMSPROP ? (float)(1.0 - h->beta2) : 1.f;
        c.inv_bc1 = 1.f;
        c.inv_sqrt_bc2 = 1.f;
        c.eps = (float)h->eps;
        c.wd_coupled = (float)h->weight_decay;
    } else {
        if (h->beta1 < 0 || h->beta1 >= 1 || h->beta2 < 0 || h->beta2 >= 1) return po_fail(PO_EINVAL, "betas must be in [0,1)");
        // bias corrections of Table 1, in fp64; t >= 1 and beta < 1 keep both strictly positive
        const double bc1 = 1.0 - std::pow(h->beta1, (double)t);
        const double bc2 = 1.0 - std::pow(h->beta2, (double)t);
        c.beta1 = (float)h->beta1;
        c.grad_scale = (float)(1.0 - h->beta1);
        c.beta2 = (float)h->beta2;
        c.one_m_beta2 = (float)(1.0 - h->beta2);
        c.inv_bc1 = (float)(1.0 / bc1);
        c.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
        c.eps = (float)h->eps;
        if (h->opt == PO_ADAM) {
            c.wd_coupled = (float)h->weight_decay;
        } else {
            c.wd_step = (float)h->weight_decay;
            c.wd_pred = h->decay_in_prediction ? (float)h->weight_decay : 0.f;
        }
    }
    c.lr = (float)h->lr;
    c.s_lr = (float)((double)s * h->lr);
    c.s_is_zero = (s == 0);
    *out = c;
    return PO_OK;
}

int pipeoptim_auto_lds_bytes(int32_t kernel, int32_t opt, int64_t n_params, int32_t* out)
{
    if (!out) return po_fail(PO_EINVAL, "out is NULL");
    if (kernel != PO_KERNEL_KIND_FUSED && kernel != PO_KERNEL_KIND_PREDICT) return po_fail(PO_EINVAL, "kernel must be 0 (fused) or 1 (prediction)");
    if (opt < PO_SGDM || opt > PO_ADAGRAD) return po_fail(PO_EINVAL, "unknown optimizer %d", opt);
    if (n_params < 0) return po_fail(PO_EINVAL, "n_params < 0");
    *out = po_auto_lds_bytes(kernel, opt, n_params, PO_LAYOUT_PLAIN);
    return PO_OK;
}

int pipeoptim_chunk_table_build(int64_t n_tensors, const int64_t* numel, int64_t chunk_elems, po_chunk* out,
                                int64_t capacity, int64_t* n_chunks)
try {
    return build_chunks(n_tensors, numel, chunk_elems, out, capacity, n_chunks);
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_chunk_table_build: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_chunk_table_build: unexpected exception"); }

int pipeoptim_plan_create_mixed(po_plan** out, int64_t n_tensors, const int64_t* numel, float* const* W,
                                const void* const* g, int32_t grad_dtype, float* const* m, float* const* v,
                                void* const* What, int32_t what_dtype, void* hip_stream)
try {
    if (!out) return po_fail(PO_EINVAL, "out is NULL");
    *out = nullptr;
    // the holder frees the host side if anything below throws or fails before device memory exists
    std::unique_ptr<po_plan> holder(new (std::nothrow) po_plan);
    po_plan* p = holder.get();
    if (!p) return po_fail(PO_ENOMEM, "out of host memory");
    int rc = po_describe_list(n_tensors, numel, W, g, grad_dtype, m, v, What, what_dtype, p->descs, &p->n_params,
                              &p->n_unaligned);
    if (rc != PO_OK) return rc;
    p->n_tensors = n_tensors;
    p->what_dtype = what_dtype;
    p->grad_dtype = grad_dtype;
    p->has_v = (v != nullptr);
    p->has_m = (m != nullptr);
    p->numel.assign(numel, numel + n_tensors);
    p->launch = po_default_launch();
    p->predict_launch = p->launch;

    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipGetDevice(&p->device);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    rc = PO_OK;
    if (n_tensors > 0) {
        const size_t bytes = (size_t)n_tensors * sizeof(po_tensor_desc);
        e = hipMalloc(reinterpret_cast<void**>(&p->d_descs), bytes);
        if (e != hipSuccess) rc = po_fail(PO_ENOMEM, "hipMalloc(descriptors): %s", hipGetErrorString(e));
        for (int k = 0; k < 2 && rc == PO_OK; ++k) {
            e = hipHostMalloc(reinterpret_cast<void**>(&p->h_descs[k]), bytes, hipHostMallocDefault);
            if (e != hipSuccess) { p->h_descs[k] = nullptr; rc = po_fail(PO_ENOMEM, "hipHostMalloc(descriptor staging): %s", hipGetErrorString(e)); break; }
            e = hipEventCreateWithFlags(&p->ev_descs[k], hipEventDisableTiming);
            if (e != hipSuccess) { p->ev_descs[k] = nullptr; rc = fail_hip(e, "hipEventCreateWithFlags"); }
        }
        if (rc == PO_OK) {
            e = hipEventCreateWithFlags(&p->ev_chunks, hipEventDisableTiming);
            if (e != hipSuccess) { p->ev_chunks = nullptr; rc = fail_hip(e, "hipEventCreateWithFlags"); }
        }
    }
    if (rc == PO_OK) rc = upload_descs(p, stream);
    if (rc == PO_OK) rc = upload_chunks(p, stream);
    if (rc == PO_OK) rc = check_grid(p->launch, (int64_t)p->chunks.size());
    if (rc != PO_OK) {
        char keep[sizeof g_err];
        std::memcpy(keep, g_err, sizeof keep);       // destroy may overwrite the message of the real failure
        pipeoptim_plan_destroy(holder.release());
        std::memcpy(g_err, keep, sizeof keep);
        return rc;
    }
    *out = holder.release();
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_plan_create_mixed: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_plan_create_mixed: unexpected exception"); }

int pipeoptim_plan_create(po_plan** out, int64_t n_tensors, const int64_t* numel, float* const* W,
                          const float* const* g, float* const* m, float* const* v, void* const* What,
                          int32_t what_dtype, void* hip_stream)
{
    return pipeoptim_plan_create_mixed(out, n_tensors, numel, W, reinterpret_cast<const void* const*>(g), PO_GRAD_F32,
                                       m, v, What, what_dtype, hip_stream);
}

int pipeoptim_plan_destroy(po_plan* p)
{
    if (!p) return PO_OK;
    int rc = PO_OK;
    if (p->d_descs || p->d_chunks || p->h_phase) rc = wait_for_plan_streams(p);
    if (p->d_descs) (void)hipFree(p->d_descs);
    if (p->d_chunks) (void)hipFree(p->d_chunks);
    for (int k = 0; k < 2; ++k) {
        if (p->h_descs[k]) (void)hipHostFree(p->h_descs[k]);
        if (p->ev_descs[k]) (void)hipEventDestroy(p->ev_descs[k]);
    }
    if (p->h_chunks) (void)hipHostFree(p->h_chunks);
    if (p->ev_chunks) (void)hipEventDestroy(p->ev_chunks);
    if (p->h_phase) (void)hipHostFree(p->h_phase);
    delete p;
    return rc;
}

int pipeoptim_plan_set_pointers(po_plan* p, int32_t which, void* const* ptrs, void* hip_stream)
try {
    if (!p) return po_fail(PO_EINVAL, "plan is NULL");
    if (which < 0 || which > 4) return po_fail(PO_EINVAL, "which must be 0..4");
    if (which == 3 && !p->has_v) return po_fail(PO_EINVAL, "plan has no v column");
    if (which == 2 && !p->has_m) return po_fail(PO_EINVAL, "plan has no m column");
    if (p->n_tensors > 0 && !ptrs) return po_fail(PO_EINVAL, "ptrs is NULL");
    const uintptr_t mask = ((which == 4 && p->what_dtype == PO_WHAT_BF16) || (which == 1 && p->grad_dtype == PO_GRAD_BF16)) ? 1u : 3u;
    for (int64_t i = 0; i < p->n_tensors; ++i) {
        if (p->numel[(size_t)i] == 0) continue;
        if (!ptrs[i]) return po_fail(PO_EINVAL, "tensor %lld: NULL pointer", (long long)i);
        if ((uintptr_t)ptrs[i] & mask) return po_fail(PO_EALIGN, "tensor %lld: pointer not aligned to its element", (long long)i);
    }
    int rc = check_device(p);
    if (rc != PO_OK) return rc;
    // everything the call changes, so that any failure below leaves the plan exactly as it was
    const std::vector<po_tensor_desc> saved = p->descs;
    const int64_t saved_unaligned = p->n_unaligned, saved_local = p->n_local_params;
    const double saved_near = p->near_bytes;
    const bool saved_marks = p->chunk_marks_valid;
    for (int64_t i = 0; i < p->n_tensors; ++i) {
        po_tensor_desc& d = p->descs[(size_t)i];
        switch (which) {
        case 0: d.W = static_cast<float*>(ptrs[i]); break;
        case 1: d.g = ptrs[i]; break;
        case 2: d.m = static_cast<float*>(ptrs[i]); break;
        case 3: d.v = static_cast<float*>(ptrs[i]); break;
        case 4: d.What = ptrs[i]; break;
        }
    }
    rc = check_disjoint(p->descs, p->grad_dtype, p->what_dtype);
    if (rc == PO_OK) {
        p->n_unaligned = refresh_flags(p->descs);
        // A learnt order was decided mostly by W, m and v (8 bytes of traffic per element each): it stays in force
        // when only g or What move (any order is correct; this one is still the better one for three streams of
        // four).  When W, m or v move, the marks in the device table are ignored from the next launch on.
        const bool keep_learnt = saved_marks && (which == 1 || which == 4);
        if (!keep_learnt) {
            p->n_local_params = 0;
            p->near_bytes = 0.0;
            p->chunk_marks_valid = false;
        }
        rc = upload_descs(p, static_cast<hipStream_t>(hip_stream));
    }
    if (rc != PO_OK) {      // the device table was not touched: upload_descs fails before or at the enqueue of its copy
        p->descs = saved;
        p->n_unaligned = saved_unaligned;
        p->n_local_params = saved_local;
        p->near_bytes = saved_near;
        p->chunk_marks_valid = saved_marks;
    }
    return rc;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_plan_set_pointers: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_plan_set_pointers: unexpected exception"); }

int pipeoptim_plan_get_launch(const po_plan* p, po_launch* out)
{
    if (!p || !out) return po_fail(PO_EINVAL, "plan or out is NULL");
    *out = p->launch;
    return PO_OK;
}

int pipeoptim_plan_set_launch(po_plan* p, const po_launch* L)
try {
    if (!p || !L) return po_fail(PO_EINVAL, "plan or launch is NULL");
    int rc = check_launch(*L);
    if (rc != PO_OK) return rc;
    int64_t n_new = 0;
    rc = build_chunks(p->n_tensors, p->numel.data(), L->chunk_elems, nullptr, 0, &n_new);
    if (rc == PO_OK) rc = check_grid(*L, n_new);
    if (rc != PO_OK) return rc;
    const bool rechunk = L->chunk_elems != p->launch.chunk_elems;
    const po_launch old = p->launch, old_predict = p->predict_launch;
    p->launch = *L;
    p->predict_launch.chunk_elems = L->chunk_elems;
    {   // the two kernels share the chunk table: keep the prediction kernel's tile a power-of-two divisor of it
        const int64_t ptile = (int64_t)p->predict_launch.block * 4;
        const int64_t ratio = L->chunk_elems / ptile;
        if (L->chunk_elems % ptile != 0 || (ratio & (ratio - 1)) != 0) p->predict_launch.block = L->block;
    }
    if (rechunk && p->n_tensors > 0) {
        rc = check_device(p);
        if (rc == PO_OK) rc = wait_for_plan_streams(p);   // a launch may still read the old table; the old upload is done
        if (rc != PO_OK) { p->launch = old; p->predict_launch = old_predict; return rc; }
        if (p->chunk_marks_valid) { p->chunk_marks_valid = false; p->n_local_params = 0; p->near_bytes = 0.0; }   // marks belong to the old table
        rc = upload_chunks(p, p->upload_stream);
        if (rc != PO_OK) { p->launch = old; p->predict_launch = old_predict; (void)upload_chunks(p, p->upload_stream); return rc; }
    }
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_plan_set_launch: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_plan_set_launch: unexpected exception"); }

int pipeoptim_plan_get_predict_launch(const po_plan* p, po_launch* out)
{
    if (!p || !out) return po_fail(PO_EINVAL, "plan or out is NULL");
    *out = p->predict_launch;
    return PO_OK;
}

int pipeoptim_plan_set_predict_launch(po_plan* p, const po_launch* L_in)
{
    if (!p || !L_in) return po_fail(PO_EINVAL, "plan or launch is NULL");
    po_launch L = *L_in;
    if (L.chunk_elems == 0) L.chunk_elems = p->launch.chunk_elems;
    int rc = check_launch(L);
    if (rc != PO_OK) return rc;
    if (L.chunk_elems != p->launch.chunk_elems)
        return po_fail(PO_EINVAL, "the prediction kernel shares the plan's chunk table: chunk_elems must be %lld",
                    (long long)p->launch.chunk_elems);
    rc = check_grid(L, (int64_t)p->chunks.size());
    if (rc != PO_OK) return rc;
    p->predict_launch = L;
    return PO_OK;
}

int pipeoptim_plan_localize(po_plan* p, const po_arena* arena, void* hip_stream, int64_t* n_local_params)
try {
    if (!p) return po_fail(PO_EINVAL, "plan is NULL");
    int rc_dev = check_device(p);
    if (rc_dev != PO_OK) return rc_dev;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (arena && !p->h_phase) {
        hipError_t eh = hipHostMalloc(reinterpret_cast<void**>(&p->h_phase), 64, hipHostMallocDefault);
        if (eh != hipSuccess) { p->h_phase = nullptr; return po_fail(PO_ENOMEM, "hipHostMalloc(phase word): %s", hipGetErrorString(eh)); }
        *p->h_phase = 0;
    }
    const std::vector<po_tensor_desc> saved = p->descs;
    int64_t n_local = 0;
    double near_gain = 0.0;
    for (int64_t i = 0; i < p->n_tensors; ++i) {
        po_tensor_desc& d = p->descs[(size_t)i];
        d.flags &= ~(PO_DESC_LOCAL | PO_DESC_HALF1);
        if (!arena || d.numel == 0) continue;
        // every fp32 stream of the tensor: inside the arena, one class, 16 KiB aligned.  Then the 8 KiB block that
        // holds elements [2048 j, 2048 j + 2048) of any of them is near to XCC half (j & 1) ^ class.
        const size_t n = (size_t)d.numel * 4;
        const void* streams[5] = {d.W, p->grad_dtype == PO_GRAD_F32 ? d.g : nullptr, d.m, d.v,
                                  p->what_dtype == PO_WHAT_F32 ? d.What : nullptr};
        int cls = -2;                                   // -2: no stream seen yet; -1: not eligible
        for (const void* q : streams) {
            if (!q) continue;
            const int c = ((uintptr_t)q & 16383u) ? -1 : po_arena_class_of(arena, q, n);
            cls = (cls == -2 || cls == c) ? c : -1;
            if (cls == -1) break;
        }
        if (cls < 0) continue;
        d.flags |= PO_DESC_LOCAL | (cls ? PO_DESC_HALF1 : 0u);
        n_local += d.numel;
        int fp32_bytes = 0;                             // moved per element through the tensor's fp32 streams: all near now
        for (int k = 0; k < 5; ++k) if (streams[k]) fp32_bytes += (k == 1 || k == 4) ? 4 : 8;
        near_gain += 0.5 * fp32_bytes * (double)d.numel;
    }
    hipError_t e = hipSuccess;
    if (arena && n_local > 0) {
        // where this stream's launches start: a tiny kernel reports it, and the answer is needed before the next launch
        e = po_launch_phase_probe(p->h_phase, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
    }
    if (e != hipSuccess) { p->descs = saved; return fail_hip(e, "phase probe"); }
    const int rc = upload_descs(p, stream);
    if (rc != PO_OK) { p->descs = saved; return rc; }
    p->n_local_params = n_local;
    p->near_bytes = near_gain;
    p->chunk_marks_valid = false;           // the two ways of marking do not mix: the last call wins
    if (n_local_params) *n_local_params = n_local;
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_plan_localize: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_plan_localize: unexpected exception"); }

int pipeoptim_plan_learn_layout(po_plan* p, void* hip_stream, int64_t* n_local_params)
try {
    if (!p) return po_fail(PO_EINVAL, "plan is NULL");
    int rc = check_device(p);
    if (rc != PO_OK) return rc;
    const uintptr_t chunk_bytes = (uintptr_t)p->launch.chunk_elems * 4;
    if (chunk_bytes < 16384 || chunk_bytes > kPiece)
        return po_fail(PO_EINVAL, "learning the layout needs chunk_elems between 4096 and 524288 (it is %lld)", (long long)p->launch.chunk_elems);
    if ((int64_t)p->launch.block * 4 != PO_LOCAL_TILE_ELEMS)
        return po_fail(PO_EINVAL, "the near-memory tile order is defined for 256-element tiles (block 64); the plan's block is %d", p->launch.block);
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // nothing of the plan may be in flight while its tables change under a launch's feet (the timing waits for the
    // whole device anyway)
    rc = wait_for_plan_streams(p);
    if (rc != PO_OK) return rc;
    PieceLayout pieces;
    rc = time_pieces_under(p, pieces);
    if (rc != PO_OK) return rc;

    // chunk by chunk: the half that brings more bytes near wins; a chunk none of whose streams is known stays plain
    std::vector<int8_t> mark(p->chunks.size(), (int8_t)-1);
    int64_t n_local = 0;
    double near_gain = 0.0;
    for (size_t k = 0; k < p->chunks.size(); ++k) {
        const po_chunk& ch = p->chunks[k];
        const int64_t begin = (int64_t)ch.chunk * p->launch.chunk_elems;
        const int64_t elems = std::min<int64_t>(p->launch.chunk_elems, p->descs[ch.tensor].numel - begin);
        VotingStream st[5];
        const int ns = voting_streams(p, p->descs[ch.tensor], st);
        double near[2];
        chunk_vote(st, ns, (uintptr_t)begin * 4, elems, pieces, near);
        if (near[0] + near[1] == 0.0) continue;
        mark[k] = (int8_t)(near[1] > near[0] ? 1 : 0);
        n_local += elems;
        // of the voting bytes the winner's are near and the loser's far; the plain order had half of each near
        near_gain += 0.5 * std::fabs(near[1] - near[0]);
    }
    if (!p->h_phase && n_local > 0) {
        hipError_t eh = hipHostMalloc(reinterpret_cast<void**>(&p->h_phase), 64, hipHostMallocDefault);
        if (eh != hipSuccess) { p->h_phase = nullptr; return po_fail(PO_ENOMEM, "hipHostMalloc(phase word): %s", hipGetErrorString(eh)); }
        *p->h_phase = 0;
    }
    if (n_local > 0) {
        // where this stream's launches start: a tiny kernel reports it, and the answer is needed before the next launch
        hipError_t e = po_launch_phase_probe(p->h_phase, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail_hip(e, "phase probe");
    }
    // arena marks and learnt marks do not mix: drop the former (descriptors), install the latter (chunk table)
    const std::vector<po_tensor_desc> saved = p->descs;
    bool had_arena_marks = false;
    for (auto& d : p->descs) { had_arena_marks = had_arena_marks || (d.flags & PO_DESC_LOCAL); d.flags &= ~(PO_DESC_LOCAL | PO_DESC_HALF1); }
    if (had_arena_marks) {
        rc = upload_descs(p, stream);
        if (rc != PO_OK) { p->descs = saved; return rc; }
        p->n_local_params = 0;
        p->near_bytes = 0.0;
    }
    const std::vector<int8_t> old_mark = p->chunk_mark;
    const bool old_valid = p->chunk_marks_valid;
    p->chunk_mark = mark;
    p->chunk_marks_valid = true;
    rc = upload_chunks(p, stream);
    if (rc != PO_OK) { p->chunk_mark = old_mark; p->chunk_marks_valid = old_valid; return rc; }
    p->n_local_params = n_local;
    p->near_bytes = near_gain;
    if (n_local_params) *n_local_params = n_local;
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_plan_learn_layout: out of host memory"); }
catch (...) { return po_fail(PO_EINVAL, "pipeoptim_plan_learn_layout: unexpected exception"); }

int pipeoptim_whole_pieces(int64_t n_ranges, const uint64_t* lo, const uint64_t* hi, uint64_t* piece_lo, uint64_t* piece_hi,
                           int64_t capacity, int64_t* n_runs)
try {
    if (n_ranges < 0 || capacity < 0 || !n_runs) return po_fail(PO_EINVAL, "bad argument");
    if ((n_ranges > 0 && (!lo || !hi)) || (capacity > 0 && (!piece_lo || !piece_hi))) return po_fail(PO_EINVAL, "a required array is NULL");
    std::vector<std::pair<uintptr_t, uintptr_t>> bytes;
    for (int64_t k = 0; k < n_ranges; ++k) {
        if (lo[k] > hi[k]) return po_fail(PO_EINVAL, "range %lld ends before it starts", (long long)k);
        bytes.push_back({(uintptr_t)lo[k], (uintptr_t)hi[k]});
    }
    const auto runs = whole_pieces_inside(bytes);
    for (size_t k = 0; k < runs.size() && (int64_t)k < capacity; ++k) { piece_lo[k] = runs[k].first; piece_hi[k] = runs[k].second; }
    *n_runs = (int64_t)runs.size();
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_whole_pieces: out of host memory"); }

int pipeoptim_chunk_vote(int32_t n_streams, const uint64_t* first_byte, const int32_t* weight, int64_t elems,
                         int64_t n_pieces, const uint64_t* piece_addr, const int8_t* even_blocks_near, double* near)
try {
    if (n_streams < 0 || n_streams > 5 || elems < 0 || n_pieces < 0 || !near) return po_fail(PO_EINVAL, "bad argument");
    if ((n_streams > 0 && (!first_byte || !weight)) || (n_pieces > 0 && (!piece_addr || !even_blocks_near)))
        return po_fail(PO_EINVAL, "a required array is NULL");
    PieceLayout pieces;
    for (int64_t k = 0; k < n_pieces; ++k) {
        if (piece_addr[k] % kPiece != 0 || (k > 0 && piece_addr[k] <= piece_addr[k - 1]))
            return po_fail(PO_EINVAL, "piece addresses must be 2 MiB aligned and ascending");
        if (even_blocks_near[k] < -1 || even_blocks_near[k] > 1) return po_fail(PO_EINVAL, "a piece's layout must be -1, 0 or 1");
        pieces.ranges.push_back({(uintptr_t)piece_addr[k], (uintptr_t)piece_addr[k] + kPiece});
        pieces.answer.push_back(std::vector<int8_t>(1, even_blocks_near[k]));
    }
    VotingStream st[5];
    for (int32_t j = 0; j < n_streams; ++j) {
        if ((first_byte[j] & 3u) || weight[j] < 0) return po_fail(PO_EINVAL, "stream %d: address not 4-byte aligned or negative weight", j);
        st[j] = {(uintptr_t)first_byte[j], weight[j]};
    }
    chunk_vote(st, n_streams, 0, elems, pieces, near);
    return PO_OK;
}
catch (const std::bad_alloc&) { return po_fail(PO_ENOMEM, "pipeoptim_chunk_vote: out of host memory"); }

int pipeoptim_plan_chunk_marks(const po_plan* p, int8_t* out, int64_t capacity, int64_t* n_chunks)
{
    if (!p || !n_chunks) return po_fail(PO_EINVAL, "plan or n_chunks is NULL");
    if (capacity < 0 || (capacity > 0 && !out)) return po_fail(PO_EINVAL, "bad output buffer");
    const int64_t n = (int64_t)p->chunks.size();
    for (int64_t k = 0; k < n && k < capacity; ++k)
        out[k] = (p->chunk_marks_valid && (size_t)k < p->chunk_mark.size()) ? p->chunk_mark[(size_t)k] : (int8_t)-1;
    *n_chunks = n;
    return PO_OK;
}

int pipeoptim_plan_near_share(const po_plan* p, double* share)
{
    if (!p || !share) return po_fail(PO_EINVAL, "plan or share is NULL");
    const int per_param = 8 + (p->grad_dtype == PO_GRAD_F32 ? 4 : 2) + (p->has_m ? 8 : 0) + (p->has_v ? 8 : 0) +
                          (p->what_dtype == PO_WHAT_F32 ? 4 : 2);
    *share = p->n_params > 0 ? 0.5 + p->near_bytes / ((double)per_param * (double)p->n_params) : 0.5;
    return PO_OK;
}

int pipeoptim_plan_local_params(const po_plan* p, int64_t* n_local_params)
{
    if (!p || !n_local_params) return po_fail(PO_EINVAL, "plan or n_local_params is NULL");
    *n_local_params = p->n_local_params;
    return PO_OK;
}

int pipeoptim_plan_launch_phase(const po_plan* p, int32_t* phase)
{
    if (!p || !phase) return po_fail(PO_EINVAL, "plan or phase is NULL");
    *phase = p->h_phase ? (int32_t)(*static_cast<volatile uint32_t*>(p->h_phase) & 7u) : -1;
    return PO_OK;
}

int pipeoptim_plan_effective_launch(const po_plan* p, int32_t kernel, int32_t opt, po_launch* out)
{
    if (!p || !out) return po_fail(PO_EINVAL, "plan or out is NULL");
    if (kernel != PO_KERNEL_KIND_FUSED && kernel != PO_KERNEL_KIND_PREDICT) return po_fail(PO_EINVAL, "kernel must be 0 (fused) or 1 (prediction)");
    if (opt < PO_SGDM || opt > PO_ADAGRAD) return po_fail(PO_EINVAL, "unknown optimizer %d", opt);
    *out = resolve_launch(p, kernel == PO_KERNEL_KIND_FUSED ? p->launch : p->predict_launch, kernel, opt);
    return PO_OK;
}

int pipeoptim_local_tile(uint32_t tile_in_chunk, int32_t first_block_half, uint32_t* out)
{
    if (!out) return po_fail(PO_EINVAL, "out is NULL");
    if (first_block_half != 0 && first_block_half != 1) return po_fail(PO_EINVAL, "first_block_half must be 0 or 1");
    *out = po_local_tile(tile_in_chunk, (uint32_t)first_block_half);
    return PO_OK;
}

int pipeoptim_local_slot(uint32_t workgroup, uint32_t phase, uint32_t n_slots, uint32_t* out)
{
    if (!out) return po_fail(PO_EINVAL, "out is NULL");
    if (phase > 7u) return po_fail(PO_EINVAL, "phase must be 0..7");
    if (n_slots == 0 || (n_slots & 7u) != 0 || workgroup >= n_slots) return po_fail(PO_EINVAL, "n_slots must be a positive multiple of 8 and workgroup below it");
    *out = po_local_slot(workgroup, phase, n_slots);
    return PO_OK;
}

int pipeoptim_plan_info(const po_plan* p, int64_t* n_params, int64_t* n_chunks, int64_t* n_unaligned)
{
    if (!p) return po_fail(PO_EINVAL, "plan is NULL");
    if (n_params) *n_params = p->n_params;
    if (n_chunks) *n_chunks = (int64_t)p->chunks.size();
    if (n_unaligned) *n_unaligned = p->n_unaligned;
    return PO_OK;
}

int pipeoptim_step_predict(const po_plan* p, const po_hyper* h, int64_t t, int32_t s, void* hip_stream)
{
    if (!p) return po_fail(PO_EINVAL, "plan is NULL");
    po_coeffs c;
    int rc = pipeoptim_coefficients(h, t, s, &c);
    if (rc != PO_OK) return rc;
    rc = check_state(p, h->opt);
    if (rc != PO_OK) return rc;
    if (p->chunks.empty()) return PO_OK;
    rc = check_device(p);
    if (rc != PO_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const po_launch L = resolve_launch(p, p->launch, PO_KERNEL_KIND_FUSED, h->opt);
    const bool local = p->n_local_params > 0 && p->h_phase;
    const uint32_t phase = local ? (*static_cast<volatile uint32_t*>(p->h_phase) & 7u) : 0u;
    hipError_t e = order_behind_upload(p, stream);
    if (e == hipSuccess)
        e = po_launch_step_predict(h->opt, p->what_dtype, p->grad_dtype, L, p->d_descs, p->d_chunks,
                                   (uint32_t)p->chunks.size(), c, stream, phase, local ? p->h_phase : nullptr,
                                   p->chunk_marks_valid);
    if (e != hipSuccess) return fail_hip(e, "launch of the fused step+predict kernel");
    return PO_OK;
}

int pipeoptim_predict(const po_plan* p, const po_hyper* h, int64_t t, int32_t s, void* hip_stream)
{
    if (!p) return po_fail(PO_EINVAL, "plan is NULL");
    po_coeffs c;
    int rc = pipeoptim_coefficients(h, t, s, &c);
    if (rc != PO_OK) return rc;
    if (h->opt > PO_ADAMW)
        return po_fail(PO_EINVAL, "optimizer %d: the direction needs the gradient, there is no prediction from the state alone", h->opt);
    rc = check_state(p, h->opt);
    if (rc != PO_OK) return rc;
    if (p->chunks.empty()) return PO_OK;
    rc = check_device(p);
    if (rc != PO_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const po_launch L = resolve_launch(p, p->predict_launch, PO_KERNEL_KIND_PREDICT, h->opt);
    const bool local = p->n_local_params > 0 && p->h_phase;
    const uint32_t phase = local ? (*static_cast<volatile uint32_t*>(p->h_phase) & 7u) : 0u;
    hipError_t e = order_behind_upload(p, stream);
    if (e == hipSuccess)
        e = po_launch_predict(h->opt, p->what_dtype, L, p->d_descs, p->d_chunks, (uint32_t)p->chunks.size(), c,
                              stream, phase, local ? p->h_phase : nullptr, p->chunk_marks_valid);
    if (e != hipSuccess) return fail_hip(e, "launch of the prediction kernel");
    return PO_OK;
}

int pipeoptim_probe_copy(void* dst, const void* src, int64_t nbytes, void* hip_stream)
{
    if (nbytes < 0 || (nbytes & 15)) return po_fail(PO_EINVAL, "nbytes must be a non-negative multiple of 16");
    if (nbytes == 0) return PO_OK;
    if (!dst || !src) return po_fail(PO_EINVAL, "dst or src is NULL");
    if (((uintptr_t)dst | (uintptr_t)src) & 15u) return po_fail(PO_EALIGN, "dst and src must be 16-byte aligned");
    hipError_t e = po_launch_probe_copy(dst, src, nbytes, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "launch of the copy kernel");
    return PO_OK;
}

}  // extern "C"

// Fused optimizer step + weight prediction kernels for gfx950 (MI355X).
//
// The path is elementwise and HBM-bound (about 0.4 flop per byte), so there is
// no MFMA and no LDS traffic here: the whole design is about moving 24-32 bytes
// per parameter exactly once, as full-width coalesced dwordx4 accesses, in an
// order the memory system likes.
//
//   per element (paper Table 1, Eq. 1, Eq. 5), fp32 arithmetic:
//     g~ = g + wd_c*W
//     m' = b1*m + gs*g~                    (SGDM: b1 = u, gs = 1 - tau)
//     v' = b2*v + (1-b2)*g~*g~             (Adam, AdamW)
//     r  = (m'*inv_bc1) / (sqrt(v')*inv_sqrt_bc2 + eps)      (SGDM: r = m')
//     W'   = W - lr  *(r + wd_step*W)
//     What = W - s_lr*(r + wd_pred*W)      (s == 0: What = W)
//   and by the same recipe, beyond Table 1: Nesterov (m' = u*m + g~, r = g~ + u*m'), RMSprop and Adagrad
//   (v' = b2*v + c2*g~*g~ with (b2, c2) = (alpha, 1-alpha) or (1, 1), r = g~ / (sqrt(v') + eps)).
//
// Work decomposition.  The host's chunk table lists (tensor, chunk) pairs at a
// coarse granularity (chunk_elems); the grid has one small workgroup per TILE
// of block*4 elements, workgroup -> (chunk, tile in chunk) by shift and
// mask, and workgroups whose tile starts past the end of the tensor exit at
// once.  A workgroup reads the chunk entry and the tensor descriptor through
// the scalar path, builds one buffer resource per stream that covers exactly
// its tile (so the hardware drops any access outside it), issues all its loads,
// does the arithmetic and stores.  Measured on MI355X, this streaming pattern
// runs fastest with single-wave workgroups, one tile each, streaming cache
// hints on every access (loads nt; stores nt + sc1, which sends them on instead
// of letting them age in L2) and an occupancy capped to roughly 10 waves per
// CU (16 for the read-dominated prediction-only kernel): a tighter window of addresses in flight per stream keeps more DRAM pages
// open across the 7-8 concurrent streams.  The cap is applied by giving each
// workgroup an unused dynamic LDS allocation (lds_bytes).
//
// Only the last tile of a tensor can be ragged; it, and any tensor whose base
// pointers are not 16-byte aligned, takes an element-wise path (dword / short
// accesses, still coalesced across the wave).
#include "po_internal.h"

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Cache policy bits of gfx940-family memory instructions as the buffer builtins take them.
constexpr int CP_NT = 2, CP_SC1 = 16;

constexpr int PO_KERNEL_FUSED = PO_KERNEL_KIND_FUSED, PO_KERNEL_PREDICT = PO_KERNEL_KIND_PREDICT;

// Kernel-side optimizer families: the three rows of Table 1, Nesterov, and one for RMSprop and Adagrad
// (which differ only in two coefficients).  Which state streams a family reads and rewrites:
enum { K_SGDM = PO_SGDM, K_ADAM = PO_ADAM, K_ADAMW = PO_ADAMW, K_NESTEROV = PO_NESTEROV, K_RMS = PO_RMSPROP };
template <int OPT> struct Streams {
    static constexpr bool M = OPT != K_RMS;
    static constexpr bool V = OPT == K_ADAM || OPT == K_ADAMW || OPT == K_RMS;
};

// Cache policy of every access (measured on MI355X against plain accesses and every mix of the two, per stream
// group): loads streaming (nt), whether the line is read once (g) or rewritten right after (W, m, v); stores
// streaming and written through (nt + sc1), i.e. sent on instead of left to age in L2.
constexpr int LD_POLICY = CP_NT, ST_POLICY = CP_NT | CP_SC1;

// Raw buffer resource (stride 0) over [p, p + bytes): accesses past `bytes` are dropped by the hardware.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ float as_f(uint32_t x) { return __builtin_bit_cast(float, x); }
__device__ __forceinline__ uint32_t as_u(float x) { return __builtin_bit_cast(uint32_t, x); }

// fp32 -> bf16, round to nearest even (hardware conversion on gfx950); two values packed low/high.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 in = {lo, hi};
    bf16x2 out = __builtin_convertvector(in, bf16x2);
    return __builtin_bit_cast(uint32_t, out);
}

__device__ __forceinline__ uint16_t to_bf16(float x)
{
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(x));
}

// One element of the update.  m and v are updated in place; returns W' and What.
template <int OPT>
__device__ __forceinline__ void update_element(const po_coeffs& c, float W, float g, float& m, float& v,
                                               float& W_new, float& W_hat)
{
    float r;
    if constexpr (OPT == K_SGDM) {
        float gt = fmaf(c.wd_coupled, W, g);
        m = fmaf(c.beta1, m, c.grad_scale * gt);
        r = m;
        W_new = fmaf(-c.lr, r, W);
        W_hat = fmaf(-c.s_lr, r, W);
    } else if constexpr (OPT == K_NESTEROV) {
        float gt = fmaf(c.wd_coupled, W, g);
        m = fmaf(c.beta1, m, gt);
        r = fmaf(c.beta1, m, gt);
        W_new = fmaf(-c.lr, r, W);
        W_hat = fmaf(-c.s_lr, r, W);
    } else if constexpr (OPT == K_RMS) {
        float gt = fmaf(c.wd_coupled, W, g);
        v = fmaf(c.beta2, v, c.one_m_beta2 * (gt * gt));
        r = gt / (sqrtf(v) + c.eps);
        W_new = fmaf(-c.lr, r, W);
        W_hat = fmaf(-c.s_lr, r, W);
    } else {
        float gt = (OPT == K_ADAM) ? fmaf(c.wd_coupled, W, g) : g;
        m = fmaf(c.beta1, m, c.grad_scale * gt);
        v = fmaf(c.beta2, v, c.one_m_beta2 * (gt * gt));
        float denom = fmaf(sqrtf(v), c.inv_sqrt_bc2, c.eps);
        r = (m * c.inv_bc1) / denom;
        if constexpr (OPT == K_ADAMW) {
            W_new = fmaf(-c.lr, fmaf(c.wd_step, W, r), W);
            W_hat = fmaf(-c.s_lr, fmaf(c.wd_pred, W, r), W);
        } else {
            W_new = fmaf(-c.lr, r, W);
            W_hat = fmaf(-c.s_lr, r, W);
        }
    }
    if (c.s_is_zero) W_hat = W;
}

// Prediction alone from the cached state (no gradient, no state update): dW from the stored m, v.
template <int OPT>
__device__ __forceinline__ float predict_element(const po_coeffs& c, float W, float m, float v)
{
    float r;
    if constexpr (OPT == PO_SGDM) {
        r = m;
    } else {
        r = (m * c.inv_bc1) / fmaf(sqrtf(v), c.inv_sqrt_bc2, c.eps);
        if constexpr (OPT == PO_ADAMW) r = fmaf(c.wd_pred, W, r);
    }
    return c.s_is_zero ? W : fmaf(-c.s_lr, r, W);
}

// Everything a kernel needs besides the tables, as ONE by-value kernel argument of 128 bytes.  Each
// workgroup lives for one tile only, so the scalar round trips in front of its first vector load are a
// fixed cost per tile: the kernel fetches this block with two wide scalar loads at its very top instead of
// letting the compiler fetch the fields one wait at a time (about 1 % on the prediction-only kernel).
struct alignas(32) KArgs {
    const po_tensor_desc* descs;
    const po_chunk* chunks;
    int64_t chunk_elems;
    uint32_t n_slots;        // chunks * tiles per chunk
    uint32_t tiles_log2;     // log2(tiles per chunk)
    uint32_t reserved;
    uint32_t tile;           // block * 4
    po_coeffs c;             // 52 bytes
    uint32_t local_ok;       // bit 0: this launch shape supports the near-memory tile order (1 KiB tiles, whole groups
                             //    of 16 tiles per chunk); bit 1: the chunk table's own marks are valid as well
    uint32_t* phase_out;     // host-visible word that workgroup 0 writes its XCC id to (or nullptr)
    uint32_t phase;          // XCC on which this queue's launches start, as last observed: workgroup id b runs
                             // on XCC (b + phase) mod 8
    uint32_t pad[5];
};
static_assert(sizeof(KArgs) == 128, "KArgs is loaded as 64 + 64 bytes");

typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
#define PO_CONSTANT __attribute__((address_space(4)))

__device__ __forceinline__ KArgs load_kargs()
{
    const PO_CONSTANT char* base = (const PO_CONSTANT char*)__builtin_amdgcn_kernarg_segment_ptr();
    union { struct { u32x16 a; u32x16 b; } raw; KArgs k; } u;
    u.raw.a = *(const PO_CONSTANT u32x16*)base;
    u.raw.b = *(const PO_CONSTANT u32x16*)(base + 64);
    return u.k;
}

// Which tile does this workgroup own?  slot = chunk_index * tiles_per_chunk + tile_in_chunk.  Returns false
// for tiles that start past the end of the tensor's last chunk.  The 64-byte descriptor comes in one scalar load.
struct Tile {
    po_tensor_desc d;
    int64_t off;        // first element of the tile within the tensor
    uint32_t len;       // elements of the tile that exist (== tile size except at the tensor's end)
    bool full;          // len == tile size and all base pointers are 16-byte aligned
};

__device__ __forceinline__ bool locate_tile(const KArgs& a, Tile& t)
{
    uint32_t slot = blockIdx.x;
    if (a.local_ok) {
        // rotate the ids (n_slots is a multiple of 16 here) so that slot p runs on XCC p mod 8 whatever XCC the
        // queue starts its launches on; the rotation is the same for every workgroup of the launch, so each
        // slot is still taken exactly once even if `phase` is out of date (then only the locality suffers)
        slot = po_local_slot(slot, a.phase, a.n_slots);
    }
    if (slot >= a.n_slots) return false;
    // the tables are not written while a kernel runs: read them through the constant address space so that
    // the (workgroup-uniform) loads go down the scalar path and their results stay in SGPRs
    const u32x2 entry = *(const PO_CONSTANT u32x2*)(uintptr_t)(a.chunks + (slot >> a.tiles_log2));
    const po_chunk ch{entry[0] & PO_CHUNK_TENSOR_MASK, entry[1]};
    union { u32x16 raw; po_tensor_desc d; } u;
    u.raw = *(const PO_CONSTANT u32x16*)(uintptr_t)(a.descs + ch.tensor);
    t.d = u.d;
    uint32_t tile_in_chunk = slot & ((1u << a.tiles_log2) - 1u);
    // near-memory order: the workgroups on XCCs 0-3 take the tiles whose blocks are near to their die.  Either the
    // whole tensor sits in an arena (descriptor flags), or the plan learnt the layout of this chunk (chunk marks)
    if (a.local_ok) {
        if (t.d.flags & PO_DESC_LOCAL) tile_in_chunk = po_local_tile(tile_in_chunk, (t.d.flags & PO_DESC_HALF1) ? 1u : 0u);
        else if ((a.local_ok & 2u) && (entry[0] & PO_CHUNK_LOCAL)) tile_in_chunk = po_local_tile(tile_in_chunk, (entry[0] & PO_CHUNK_HALF1) ? 1u : 0u);
    }
    t.off = (int64_t)ch.chunk * a.chunk_elems + (int64_t)tile_in_chunk * a.tile;
    if (t.off >= t.d.numel) return false;
    t.len = (t.d.numel - t.off < (int64_t)a.tile) ? (uint32_t)(t.d.numel - t.off) : a.tile;
    t.full = t.len == a.tile && (t.d.flags & PO_DESC_VECTOR_OK);
    return true;
}

// Workgroup 0 tells the host which XCC this queue started the launch on, for the next launch's `phase`.
__device__ __forceinline__ void report_phase(const KArgs& a)
{
    if (a.phase_out && blockIdx.x == 0 && threadIdx.x == 0) *a.phase_out = po_xcc_id();
}

// bf16 -> fp32 is exact: the bf16 pattern is the upper half of the fp32 pattern.
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return as_f(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return as_f(pair & 0xFFFF0000u); }

// GB16: gradients are bf16 (8 bytes per lane instead of 16).
template <int OPT, bool BF16, bool GB16>
__global__ __launch_bounds__(256) void step_predict_kernel(KArgs)
{
    constexpr bool HAS_M = Streams<OPT>::M, HAS_V = Streams<OPT>::V;

    const KArgs a = load_kargs();
    const po_coeffs& c = a.c;
    report_phase(a);
    Tile t;
    if (!locate_tile(a, t)) return;
    const po_tensor_desc* d = &t.d;
    const int64_t off = t.off;
    const uint32_t len = t.len;

    const __amdgpu_buffer_rsrc_t rW = make_rsrc(d->W + off, len * 4u);
    const __amdgpu_buffer_rsrc_t rg = GB16 ? make_rsrc(static_cast<const uint16_t*>(d->g) + off, len * 2u)
                                           : make_rsrc(static_cast<const float*>(d->g) + off, len * 4u);
    // a family without a stream never touches its resource (W stands in so that the descriptor is valid)
    const __amdgpu_buffer_rsrc_t rm = make_rsrc((HAS_M ? d->m : d->W) + off, len * 4u);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc((HAS_V ? d->v : d->W) + off, len * 4u);
    const __amdgpu_buffer_rsrc_t rh = BF16 ? make_rsrc(static_cast<uint16_t*>(d->What) + off, len * 2u)
                                           : make_rsrc(static_cast<float*>(d->What) + off, len * 4u);
    const uint32_t tid = threadIdx.x, nthr = a.tile / 4u;

    if (t.full) {
        // full tile, aligned: every lane moves 4 consecutive elements per stream; all loads go out before any use
        const uint32_t b = tid * 16u;
        u32x4 W, g, m, v;
        W = __builtin_amdgcn_raw_buffer_load_b128(rW, b, 0, LD_POLICY);
        if constexpr (GB16) {
            const u32x2 p = __builtin_amdgcn_raw_buffer_load_b64(rg, b >> 1, 0, LD_POLICY);
            g = u32x4{as_u(bf16_lo(p[0])), as_u(bf16_hi(p[0])), as_u(bf16_lo(p[1])), as_u(bf16_hi(p[1]))};
        } else {
            g = __builtin_amdgcn_raw_buffer_load_b128(rg, b, 0, LD_POLICY);
        }
        if constexpr (HAS_M) m = __builtin_amdgcn_raw_buffer_load_b128(rm, b, 0, LD_POLICY);
        if constexpr (HAS_V) v = __builtin_amdgcn_raw_buffer_load_b128(rv, b, 0, LD_POLICY);
        u32x4 Wn, Wh;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float mm = HAS_M ? as_f(m[e]) : 0.f, vv = HAS_V ? as_f(v[e]) : 0.f, wn, wh;
            update_element<OPT>(c, as_f(W[e]), as_f(g[e]), mm, vv, wn, wh);
            if constexpr (HAS_M) m[e] = as_u(mm);
            if constexpr (HAS_V) v[e] = as_u(vv);
            Wn[e] = as_u(wn);
            Wh[e] = as_u(wh);
        }
        __builtin_amdgcn_raw_buffer_store_b128(Wn, rW, b, 0, ST_POLICY);
        if constexpr (HAS_M) __builtin_amdgcn_raw_buffer_store_b128(m, rm, b, 0, ST_POLICY);
        if constexpr (HAS_V) __builtin_amdgcn_raw_buffer_store_b128(v, rv, b, 0, ST_POLICY);
        if constexpr (BF16) {
            u32x2 p = {pack_bf16x2(as_f(Wh[0]), as_f(Wh[1])), pack_bf16x2(as_f(Wh[2]), as_f(Wh[3]))};
            __builtin_amdgcn_raw_buffer_store_b64(p, rh, b >> 1, 0, ST_POLICY);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(Wh, rh, b, 0, ST_POLICY);
        }
    } else {
        // ragged last tile of a tensor, or a tensor without 16-byte alignment: one element per lane per step
        for (uint32_t i = tid; i < len; i += nthr) {
            const uint32_t b = i * 4u;
            float W = as_f(__builtin_amdgcn_raw_buffer_load_b32(rW, b, 0, LD_POLICY));
            float g = GB16 ? as_f((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rg, i * 2u, 0, LD_POLICY) << 16)
                           : as_f(__builtin_amdgcn_raw_buffer_load_b32(rg, b, 0, LD_POLICY));
            float mm = HAS_M ? as_f(__builtin_amdgcn_raw_buffer_load_b32(rm, b, 0, LD_POLICY)) : 0.f;
            float vv = HAS_V ? as_f(__builtin_amdgcn_raw_buffer_load_b32(rv, b, 0, LD_POLICY)) : 0.f;
            float wn, wh;
            update_element<OPT>(c, W, g, mm, vv, wn, wh);
            __builtin_amdgcn_raw_buffer_store_b32(as_u(wn), rW, b, 0, ST_POLICY);
            if constexpr (HAS_M) __builtin_amdgcn_raw_buffer_store_b32(as_u(mm), rm, b, 0, ST_POLICY);
            if constexpr (HAS_V) __builtin_amdgcn_raw_buffer_store_b32(as_u(vv), rv, b, 0, ST_POLICY);
            if constexpr (BF16) __builtin_amdgcn_raw_buffer_store_b16(to_bf16(wh), rh, i * 2u, 0, ST_POLICY);
            else __builtin_amdgcn_raw_buffer_store_b32(as_u(wh), rh, b, 0, ST_POLICY);
        }
    }
}

// What = W - s_lr*dW from the cached m, v: reads W, m (, v) once, writes What.  Same decomposition as above.
template <int OPT, bool BF16>
__global__ __launch_bounds__(256) void predict_kernel(KArgs)
{
    constexpr bool ADAM = OPT != PO_SGDM;

    const KArgs a = load_kargs();
    const po_coeffs& c = a.c;
    report_phase(a);
    Tile t;
    if (!locate_tile(a, t)) return;
    const po_tensor_desc* d = &t.d;
    const int64_t off = t.off;
    const uint32_t len = t.len;
    const __amdgpu_buffer_rsrc_t rW = make_rsrc(d->W + off, len * 4u);
    const __amdgpu_buffer_rsrc_t rm = make_rsrc(d->m + off, len * 4u);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(ADAM ? d->v + off : d->m + off, len * 4u);
    const __amdgpu_buffer_rsrc_t rh = BF16 ? make_rsrc(static_cast<uint16_t*>(d->What) + off, len * 2u)
                                           : make_rsrc(static_cast<float*>(d->What) + off, len * 4u);
    const uint32_t tid = threadIdx.x, nthr = a.tile / 4u;

    if (t.full) {
        const uint32_t b = tid * 16u;
        u32x4 W, m, v;
        W = __builtin_amdgcn_raw_buffer_load_b128(rW, b, 0, LD_POLICY);
        m = __builtin_amdgcn_raw_buffer_load_b128(rm, b, 0, LD_POLICY);
        if constexpr (ADAM) v = __builtin_amdgcn_raw_buffer_load_b128(rv, b, 0, LD_POLICY);
        float wh[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            wh[e] = predict_element<OPT>(c, as_f(W[e]), as_f(m[e]), ADAM ? as_f(v[e]) : 0.f);
        if constexpr (BF16) {
            u32x2 p = {pack_bf16x2(wh[0], wh[1]), pack_bf16x2(wh[2], wh[3])};
            __builtin_amdgcn_raw_buffer_store_b64(p, rh, b >> 1, 0, ST_POLICY);
        } else {
            u32x4 p = {as_u(wh[0]), as_u(wh[1]), as_u(wh[2]), as_u(wh[3])};
            __builtin_amdgcn_raw_buffer_store_b128(p, rh, b, 0, ST_POLICY);
        }
    } else {
        for (uint32_t i = tid; i < len; i += nthr) {
            const uint32_t b = i * 4u;
            float W = as_f(__builtin_amdgcn_raw_buffer_load_b32(rW, b, 0, LD_POLICY));
            float mm = as_f(__builtin_amdgcn_raw_buffer_load_b32(rm, b, 0, LD_POLICY));
            float vv = ADAM ? as_f(__builtin_amdgcn_raw_buffer_load_b32(rv, b, 0, LD_POLICY)) : 0.f;
            float wh = predict_element<OPT>(c, W, mm, vv);
            if constexpr (BF16) __builtin_amdgcn_raw_buffer_store_b16(to_bf16(wh), rh, i * 2u, 0, ST_POLICY);
            else __builtin_amdgcn_raw_buffer_store_b32(as_u(wh), rh, b, 0, ST_POLICY);
        }
    }
}

// Where a launch starts its round over the XCCs: last observed value, and where workgroup 0 reports the next.
struct Phase { uint32_t value; uint32_t* report; bool chunk_marks; };

template <int KIND, int OPT, bool BF16, bool GB16>
hipError_t launch_one(const po_launch& L, const po_tensor_desc* descs, const po_chunk* chunks, uint32_t n_chunks,
                      const po_coeffs& c, hipStream_t stream, Phase ph)
{
    const uint32_t tile = (uint32_t)L.block * 4u;
    const uint32_t tiles_per_chunk = (uint32_t)(L.chunk_elems / tile);      // a power of two (validated by the host)
    uint32_t tiles_log2 = 0;
    while ((1u << tiles_log2) < tiles_per_chunk) ++tiles_log2;
    const uint64_t grid = (uint64_t)n_chunks << tiles_log2;
    if (grid > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    if (L.lds_bytes < 0) return hipErrorInvalidValue;      // the host resolves PO_LDS_AUTO before it gets here
    KArgs a{};
    a.descs = descs;
    a.chunks = chunks;
    a.chunk_elems = L.chunk_elems;
    a.n_slots = (uint32_t)grid;
    a.tiles_log2 = tiles_log2;
    a.tile = tile;
    a.c = c;
    a.local_ok = (tile == PO_LOCAL_TILE_ELEMS && tiles_per_chunk >= PO_LOCAL_GROUP_TILES) ? (ph.chunk_marks ? 3u : 1u) : 0u;
    a.phase = a.local_ok ? (ph.value & 7u) : 0u;
    a.phase_out = a.local_ok ? ph.report : nullptr;
    if constexpr (KIND == PO_KERNEL_PREDICT)
        hipLaunchKernelGGL((predict_kernel<OPT, BF16>), dim3((uint32_t)grid), dim3(L.block), (size_t)L.lds_bytes, stream, a);
    else
        hipLaunchKernelGGL((step_predict_kernel<OPT, BF16, GB16>), dim3((uint32_t)grid), dim3(L.block),
                           (size_t)L.lds_bytes, stream, a);
    return hipGetLastError();
}

template <int KIND, int OPT>
hipError_t dispatch_dtype(int what_dtype, int grad_dtype, const po_launch& L, const po_tensor_desc* d,
                          const po_chunk* ch, uint32_t n, const po_coeffs& c, hipStream_t s, Phase ph)
{
    const bool h16 = what_dtype == PO_WHAT_BF16;
    if constexpr (KIND == PO_KERNEL_FUSED) {
        if (grad_dtype == PO_GRAD_BF16)
            return h16 ? launch_one<KIND, OPT, true, true>(L, d, ch, n, c, s, ph)
                       : launch_one<KIND, OPT, false, true>(L, d, ch, n, c, s, ph);
    }
    return h16 ? launch_one<KIND, OPT, true, false>(L, d, ch, n, c, s, ph)
               : launch_one<KIND, OPT, false, false>(L, d, ch, n, c, s, ph);
}

// One workgroup per XCC; workgroup 0 writes the id of the XCC it runs on.
__global__ __launch_bounds__(64) void phase_probe_kernel(uint32_t* out)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *out = po_xcc_id();
}

// Plain copy: the yardstick for what one read stream plus one write stream reach on this chip.
// One single-wave workgroup per 1 KiB, streaming loads, streaming write-through stores (the fastest plain
// copy measured on MI355X).
__global__ __launch_bounds__(64) void probe_copy_kernel(char* __restrict__ dst, const char* __restrict__ src,
                                                        int64_t nbytes)
{
    const int64_t base = (int64_t)blockIdx.x * 1024;
    const int64_t left = nbytes - base;
    const uint32_t len = left < 1024 ? (uint32_t)left : 1024u;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(src + base, len), rd = make_rsrc(dst + base, len);
    const uint32_t b = threadIdx.x * 16u;
    u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, b, 0, CP_NT);
    __builtin_amdgcn_raw_buffer_store_b128(x, rd, b, 0, CP_NT | CP_SC1);
}

// The same copy in the near-memory tile order, for buffers from one class range of an arena: the yardstick for
// what one read stream plus one write stream reach when every XCC stays on its own die's memory.
__global__ __launch_bounds__(64) void probe_copy_near_kernel(char* __restrict__ dst, const char* __restrict__ src,
                                                             uint32_t n_tiles, uint32_t first_block_half, uint32_t phase,
                                                             uint32_t* phase_out)
{
    if (phase_out && blockIdx.x == 0 && threadIdx.x == 0) *phase_out = po_xcc_id();
    const uint32_t tile = po_local_tile(po_local_slot(blockIdx.x, phase, n_tiles), first_block_half);
    const int64_t base = (int64_t)tile * 1024;
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(src + base, 1024u), rd = make_rsrc(dst + base, 1024u);
    const uint32_t b = threadIdx.x * 16u;
    u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, b, 0, CP_NT);
    __builtin_amdgcn_raw_buffer_store_b128(x, rd, b, 0, CP_NT | CP_SC1);
}

}  // namespace

hipError_t po_launch_probe_copy_near(void* dst, const void* src, int64_t nbytes, uint32_t first_block_half, uint32_t phase,
                                     uint32_t* phase_report, int32_t lds_bytes, hipStream_t stream)
{
    if (nbytes <= 0) return hipSuccess;
    const int64_t n_tiles = nbytes / 1024;                 // the caller checked: a multiple of 16 tiles, below 2^31
    if (nbytes % 16384 != 0 || n_tiles > 0x7FFFFFF0ll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(probe_copy_near_kernel, dim3((uint32_t)n_tiles), dim3(64), (size_t)lds_bytes, stream,
                       static_cast<char*>(dst), static_cast<const char*>(src), (uint32_t)n_tiles, first_block_half & 1u,
                       phase & 7u, phase_report);
    return hipGetLastError();
}

hipError_t po_launch_phase_probe(uint32_t* host_visible_word, hipStream_t stream)
{
    hipLaunchKernelGGL(phase_probe_kernel, dim3(8), dim3(64), 0, stream, host_visible_word);
    return hipGetLastError();
}

hipError_t po_launch_step_predict(int opt, int what_dtype, int grad_dtype, const po_launch& L,
                                  const po_tensor_desc* d_descs, const po_chunk* d_chunks, uint32_t n_chunks,
                                  const po_coeffs& c, hipStream_t stream, uint32_t phase, uint32_t* phase_report, bool chunk_marks)
{
    if (n_chunks == 0) return hipSuccess;
    switch (opt) {
    case PO_SGDM: return dispatch_dtype<PO_KERNEL_FUSED, PO_SGDM>(what_dtype, grad_dtype, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    case PO_ADAM: return dispatch_dtype<PO_KERNEL_FUSED, PO_ADAM>(what_dtype, grad_dtype, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    case PO_ADAMW: return dispatch_dtype<PO_KERNEL_FUSED, PO_ADAMW>(what_dtype, grad_dtype, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    case PO_NESTEROV: return dispatch_dtype<PO_KERNEL_FUSED, K_NESTEROV>(what_dtype, grad_dtype, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    case PO_RMSPROP:
    case PO_ADAGRAD: return dispatch_dtype<PO_KERNEL_FUSED, K_RMS>(what_dtype, grad_dtype, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    }
    return hipErrorInvalidValue;
}

hipError_t po_launch_predict(int opt, int what_dtype, const po_launch& L, const po_tensor_desc* d_descs,
                             const po_chunk* d_chunks, uint32_t n_chunks, const po_coeffs& c, hipStream_t stream,
                             uint32_t phase, uint32_t* phase_report, bool chunk_marks)
{
    if (n_chunks == 0) return hipSuccess;
    switch (opt) {
    case PO_SGDM: return dispatch_dtype<PO_KERNEL_PREDICT, PO_SGDM>(what_dtype, PO_GRAD_F32, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    case PO_ADAM: return dispatch_dtype<PO_KERNEL_PREDICT, PO_ADAM>(what_dtype, PO_GRAD_F32, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    case PO_ADAMW: return dispatch_dtype<PO_KERNEL_PREDICT, PO_ADAMW>(what_dtype, PO_GRAD_F32, L, d_descs, d_chunks, n_chunks, c, stream, Phase{phase, phase_report, chunk_marks});
    }
    return hipErrorInvalidValue;
}

hipError_t po_launch_probe_copy(void* dst, const void* src, int64_t nbytes, hipStream_t stream)
{
    if (nbytes <= 0) return hipSuccess;
    const int64_t grid = (nbytes + 1023) / 1024;
    if (grid > 0x7FFFFFFFll) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((uint32_t)grid), dim3(64), 0, stream, static_cast<char*>(dst),
                       static_cast<const char*>(src), nbytes);
    return hipGetLastError();
}

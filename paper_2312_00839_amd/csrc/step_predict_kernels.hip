// Fused optimizer step + weight prediction kernels for gfx950 (MI355X).
//
// The path is elementwise and HBM-bound (about 0.4 flop per byte), so there is
// no MFMA and no LDS here: the whole design is about moving 24-32 bytes per
// parameter exactly once with full-width, coalesced dwordx4 accesses and enough
// of them in flight per wave.
//
//   per element (paper Table 1, Eq. 1, Eq. 5), fp32 arithmetic:
//     g~ = g + wd_c*W
//     m' = b1*m + gs*g~                    (SGDM: b1 = u, gs = 1 - tau)
//     v' = b2*v + (1-b2)*g~*g~             (Adam, AdamW)
//     r  = (m'*inv_bc1) / (sqrt(v')*inv_sqrt_bc2 + eps)      (SGDM: r = m')
//     W'   = W - lr  *(r + wd_step*W)
//     What = W - s_lr*(r + wd_pred*W)      (s == 0: What = W)
//
// Work decomposition: the host's chunk table lists (tensor, chunk) pairs; a
// workgroup takes one entry (or strides over the table when the grid is
// capped), reads the tensor's descriptor through the scalar path and walks the
// chunk in tiles of block*VEC*UNROLL elements.  In a full tile every lane first
// issues all of its loads (UNROLL groups x 3-4 streams x VEC/4 dwordx4), then
// does the arithmetic, then stores.  Only the last chunk of a tensor has a
// ragged tail, handled by the same lanes with per-group bounds checks and a
// scalar remainder; a tensor whose base pointers are not 16-byte aligned takes
// a scalar loop.
#include "po_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tensor pointers come out of a descriptor in memory, so the compiler cannot tell which address
// space they are in and would emit flat accesses; they are device-global by contract.
#define PO_GLOBAL __attribute__((address_space(1)))
typedef PO_GLOBAL float gfloat;
typedef PO_GLOBAL const float gcfloat;
typedef PO_GLOBAL void gvoid;
typedef PO_GLOBAL uint16_t gu16;

constexpr int NT_LOAD = 1, NT_STORE = 2;

template <int NT>
__device__ __forceinline__ f32x4 load4(gcfloat* p)
{
    if constexpr (NT & NT_LOAD) return __builtin_nontemporal_load((PO_GLOBAL const f32x4*)p);
    else return *(PO_GLOBAL const f32x4*)p;
}

template <int NT, typename V>
__device__ __forceinline__ void storev(gvoid* p, V x)
{
    if constexpr (NT & NT_STORE) __builtin_nontemporal_store(x, (PO_GLOBAL V*)p);
    else *(PO_GLOBAL V*)p = x;
}

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
    if constexpr (OPT == PO_SGDM) {
        float gt = fmaf(c.wd_coupled, W, g);
        m = fmaf(c.beta1, m, c.grad_scale * gt);
        r = m;
        W_new = fmaf(-c.lr, r, W);
        W_hat = fmaf(-c.s_lr, r, W);
    } else {
        float gt = (OPT == PO_ADAM) ? fmaf(c.wd_coupled, W, g) : g;
        m = fmaf(c.beta1, m, c.grad_scale * gt);
        v = fmaf(c.beta2, v, c.one_m_beta2 * (gt * gt));
        float denom = fmaf(sqrtf(v), c.inv_sqrt_bc2, c.eps);
        r = (m * c.inv_bc1) / denom;
        if constexpr (OPT == PO_ADAMW) {
            W_new = fmaf(-c.lr, fmaf(c.wd_step, W, r), W);
            W_hat = fmaf(-c.s_lr, fmaf(c.wd_pred, W, r), W);
        } else {
            W_new = fmaf(-c.lr, r, W);
            W_hat = fmaf(-c.s_lr, r, W);
        }
    }
    if (c.s_is_zero) W_hat = W;
}

// VEC consecutive elements held by one lane.
template <int VEC>
struct Group {
    f32x4 W[VEC / 4], g[VEC / 4], m[VEC / 4], v[VEC / 4];
};

template <int OPT, int VEC, int NT>
__device__ __forceinline__ void load_group(Group<VEC>& G, gcfloat* W, gcfloat* g, gcfloat* m,
                                           gcfloat* v, int64_t i)
{
#pragma unroll
    for (int k = 0; k < VEC / 4; ++k) {
        G.W[k] = load4<NT>(W + i + 4 * k);
        G.g[k] = load4<NT>(g + i + 4 * k);
        G.m[k] = load4<NT>(m + i + 4 * k);
        if constexpr (OPT != PO_SGDM) G.v[k] = load4<NT>(v + i + 4 * k);
    }
}

template <int OPT, bool BF16, int VEC, int NT>
__device__ __forceinline__ void compute_store_group(const po_coeffs& c, Group<VEC>& G, gfloat* W, gfloat* m,
                                                    gfloat* v, gvoid* What, int64_t i)
{
    f32x4 Wn[VEC / 4], Wh[VEC / 4];
#pragma unroll
    for (int k = 0; k < VEC / 4; ++k) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float mm = G.m[k][e], vv = (OPT != PO_SGDM) ? G.v[k][e] : 0.f, wn, wh;
            update_element<OPT>(c, G.W[k][e], G.g[k][e], mm, vv, wn, wh);
            G.m[k][e] = mm;
            if constexpr (OPT != PO_SGDM) G.v[k][e] = vv;
            Wn[k][e] = wn;
            Wh[k][e] = wh;
        }
    }
#pragma unroll
    for (int k = 0; k < VEC / 4; ++k) {
        storev<NT>(W + i + 4 * k, Wn[k]);
        storev<NT>(m + i + 4 * k, G.m[k]);
        if constexpr (OPT != PO_SGDM) storev<NT>(v + i + 4 * k, G.v[k]);
    }
    if constexpr (BF16) {
        gu16* out = (gu16*)What + i;
        if constexpr (VEC == 8) {
            u32x4 p = {pack_bf16x2(Wh[0][0], Wh[0][1]), pack_bf16x2(Wh[0][2], Wh[0][3]),
                       pack_bf16x2(Wh[1][0], Wh[1][1]), pack_bf16x2(Wh[1][2], Wh[1][3])};
            storev<NT>(out, p);
        } else {
            u32x2 p = {pack_bf16x2(Wh[0][0], Wh[0][1]), pack_bf16x2(Wh[0][2], Wh[0][3])};
            storev<NT>(out, p);
        }
    } else {
        gfloat* out = (gfloat*)What + i;
#pragma unroll
        for (int k = 0; k < VEC / 4; ++k) storev<NT>(out + 4 * k, Wh[k]);
    }
}

template <int OPT, bool BF16>
__device__ __forceinline__ void scalar_range(const po_coeffs& c, gfloat* W, gcfloat* g, gfloat* m, gfloat* v,
                                             gvoid* What, int64_t begin, int64_t end, int tid, int nthreads)
{
    for (int64_t i = begin + tid; i < end; i += nthreads) {
        float mm = m[i], vv = (OPT != PO_SGDM) ? v[i] : 0.f, wn, wh;
        update_element<OPT>(c, W[i], g[i], mm, vv, wn, wh);
        W[i] = wn;
        m[i] = mm;
        if constexpr (OPT != PO_SGDM) v[i] = vv;
        if constexpr (BF16) ((gu16*)What)[i] = to_bf16(wh);
        else ((gfloat*)What)[i] = wh;
    }
}

template <int OPT, bool BF16, int VEC, int UNROLL, int NT>
__global__ __launch_bounds__(256) void step_predict_kernel(const po_tensor_desc* __restrict__ descs,
                                                           const po_chunk* __restrict__ chunks,
                                                           uint32_t n_chunks, int64_t chunk_elems,
                                                           int xcd_remap, po_coeffs c)
{
    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int64_t tile = (int64_t)nthr * VEC * UNROLL;

    // With xcd_remap the slot space is 8 equal ranges (one per XCD; workgroup ids go round-robin
    // over the XCDs), padded to 8*ceil(n/8) slots; padding slots do nothing.
    const uint32_t per_xcd = (n_chunks + 7u) / 8u;
    const uint32_t n_slots = xcd_remap ? per_xcd * 8u : n_chunks;
    for (uint32_t slot = blockIdx.x; slot < n_slots; slot += gridDim.x) {
        uint32_t ci = slot;
        if (xcd_remap) {
            ci = (slot & 7u) * per_xcd + (slot >> 3);
            if (ci >= n_chunks) continue;
        }
        const po_chunk ch = chunks[ci];
        const po_tensor_desc* d = descs + ch.tensor;
        const int64_t off = (int64_t)ch.chunk * chunk_elems;
        const int64_t numel = d->numel;
        const int64_t len = (numel - off < chunk_elems) ? (numel - off) : chunk_elems;
        gfloat* W = (gfloat*)d->W + off;
        gcfloat* g = (gcfloat*)d->g + off;
        gfloat* m = (gfloat*)d->m + off;
        gfloat* v = (OPT != PO_SGDM) ? (gfloat*)d->v + off : nullptr;
        gvoid* What = BF16 ? (gvoid*)((gu16*)d->What + off) : (gvoid*)((gfloat*)d->What + off);

        if (!(d->flags & PO_DESC_VECTOR_OK)) {
            scalar_range<OPT, BF16>(c, W, g, m, v, What, 0, len, tid, nthr);
            continue;
        }

        int64_t base = 0;
        for (; base + tile <= len; base += tile) {
            Group<VEC> G[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                load_group<OPT, VEC, NT>(G[u], W, g, m, v, base + ((int64_t)u * nthr + tid) * VEC);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                compute_store_group<OPT, BF16, VEC, NT>(c, G[u], W, m, v, What,
                                                        base + ((int64_t)u * nthr + tid) * VEC);
        }
        if (base < len) {
            // ragged tail of the tensor's last chunk: whole groups while they fit, then single elements
            const int64_t vec_end = base + ((len - base) / VEC) * VEC;
            for (int64_t i = base + (int64_t)tid * VEC; i < vec_end; i += (int64_t)nthr * VEC) {
                Group<VEC> G;
                load_group<OPT, VEC, NT>(G, W, g, m, v, i);
                compute_store_group<OPT, BF16, VEC, NT>(c, G, W, m, v, What, i);
            }
            scalar_range<OPT, BF16>(c, W, g, m, v, What, vec_end, len, tid, nthr);
        }
    }
}

template <int OPT, bool BF16, int VEC, int UNROLL, int NT>
hipError_t launch_one(const po_launch& L, const po_tensor_desc* descs, const po_chunk* chunks, uint32_t n_chunks,
                      const po_coeffs& c, hipStream_t stream)
{
    // one workgroup per slot (xcd_remap pads the slot space to a multiple of 8), capped by max_grid;
    // any grid size covers every slot exactly once through the kernel's stride loop
    uint32_t grid = L.xcd_remap ? ((n_chunks + 7u) / 8u) * 8u : n_chunks;
    if (L.max_grid > 0 && grid > (uint32_t)L.max_grid) {
        grid = (uint32_t)L.max_grid;
        if (L.xcd_remap && grid >= 8u) grid &= ~7u;   // keeps a workgroup on one XCD's range
    }
    if (grid > (1u << 24)) grid = 1u << 24;           // stay far below the grid-size limits
    hipLaunchKernelGGL((step_predict_kernel<OPT, BF16, VEC, UNROLL, NT>), dim3(grid), dim3(L.block), 0, stream,
                       descs, chunks, n_chunks, L.chunk_elems, L.xcd_remap, c);
    return hipGetLastError();
}

template <int OPT, bool BF16, int VEC, int UNROLL>
hipError_t dispatch_nt(const po_launch& L, const po_tensor_desc* d, const po_chunk* ch, uint32_t n,
                       const po_coeffs& c, hipStream_t s)
{
    switch (L.nontemporal) {
    case 0: return launch_one<OPT, BF16, VEC, UNROLL, 0>(L, d, ch, n, c, s);
    case 1: return launch_one<OPT, BF16, VEC, UNROLL, 1>(L, d, ch, n, c, s);
    case 2: return launch_one<OPT, BF16, VEC, UNROLL, 2>(L, d, ch, n, c, s);
    case 3: return launch_one<OPT, BF16, VEC, UNROLL, 3>(L, d, ch, n, c, s);
    }
    return hipErrorInvalidValue;
}

template <int OPT, bool BF16>
hipError_t dispatch_shape(const po_launch& L, const po_tensor_desc* d, const po_chunk* ch, uint32_t n,
                          const po_coeffs& c, hipStream_t s)
{
    if (L.vec == 4 && L.unroll == 1) return dispatch_nt<OPT, BF16, 4, 1>(L, d, ch, n, c, s);
    if (L.vec == 4 && L.unroll == 2) return dispatch_nt<OPT, BF16, 4, 2>(L, d, ch, n, c, s);
    if (L.vec == 4 && L.unroll == 4) return dispatch_nt<OPT, BF16, 4, 4>(L, d, ch, n, c, s);
    if (L.vec == 8 && L.unroll == 1) return dispatch_nt<OPT, BF16, 8, 1>(L, d, ch, n, c, s);
    if (L.vec == 8 && L.unroll == 2) return dispatch_nt<OPT, BF16, 8, 2>(L, d, ch, n, c, s);
    return hipErrorInvalidValue;
}

template <int OPT>
hipError_t dispatch_dtype(int what_dtype, const po_launch& L, const po_tensor_desc* d, const po_chunk* ch,
                          uint32_t n, const po_coeffs& c, hipStream_t s)
{
    return what_dtype == PO_WHAT_BF16 ? dispatch_shape<OPT, true>(L, d, ch, n, c, s)
                                      : dispatch_shape<OPT, false>(L, d, ch, n, c, s);
}

// Plain copy: the yardstick for what a read+write stream reaches on this chip.
__global__ __launch_bounds__(256) void probe_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                         int64_t n_vec)
{
    const int64_t tile = (int64_t)blockDim.x * 4;
    for (int64_t base = (int64_t)blockIdx.x * tile; base < n_vec; base += (int64_t)gridDim.x * tile) {
        u32x4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int64_t i = base + (int64_t)u * blockDim.x + threadIdx.x;
            if (i < n_vec) x[u] = src[i];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int64_t i = base + (int64_t)u * blockDim.x + threadIdx.x;
            if (i < n_vec) dst[i] = x[u];
        }
    }
}

}  // namespace

hipError_t po_launch_step_predict(int opt, int what_dtype, const po_launch& L, const po_tensor_desc* d_descs,
                                  const po_chunk* d_chunks, uint32_t n_chunks, const po_coeffs& c,
                                  hipStream_t stream)
{
    if (n_chunks == 0) return hipSuccess;
    switch (opt) {
    case PO_SGDM: return dispatch_dtype<PO_SGDM>(what_dtype, L, d_descs, d_chunks, n_chunks, c, stream);
    case PO_ADAM: return dispatch_dtype<PO_ADAM>(what_dtype, L, d_descs, d_chunks, n_chunks, c, stream);
    case PO_ADAMW: return dispatch_dtype<PO_ADAMW>(what_dtype, L, d_descs, d_chunks, n_chunks, c, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t po_launch_probe_copy(void* dst, const void* src, int64_t nbytes, hipStream_t stream)
{
    const int64_t n_vec = nbytes / 16;
    if (n_vec == 0) return hipSuccess;
    const int64_t tile = 256 * 4;
    int64_t grid = (n_vec + tile - 1) / tile;
    if (grid > (1 << 20)) grid = 1 << 20;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((uint32_t)grid), dim3(256), 0, stream, static_cast<u32x4*>(dst),
                       static_cast<const u32x4*>(src), n_vec);
    return hipGetLastError();
}

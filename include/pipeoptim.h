/*
 * pipeoptim.h -- C ABI of libpipeoptim: PipeOptim's optimizer-dependent weight
 * prediction fused with the optimizer step, for one pipeline stage's ragged
 * list of fp32 parameter tensors, on one AMD MI355X (gfx950).
 *
 * One call of pipeoptim_step_predict() makes one coalesced pass over the stage:
 * it reads W_t, g_t and the cached optimizer state once, and writes the updated
 * state, the stepped weights W_{t+1} (paper Eq. 1, first line) and the predicted
 * weights What_{t+s} = W_t - lr*s*dW_t (paper Eq. 3 / Eq. 5) that the next
 * forward pass uses, with dW_t from the optimizer's update rule (paper Table 1).
 *
 * Typical sequence:  pipeoptim_plan_create(stage's W, g, m, v, What pointers)  ->  every iteration
 * pipeoptim_step_predict(plan, hyper, t, s, stream)  ->  pipeoptim_plan_destroy.  A caller that lets the library
 * place the stage's memory gets the pointers from pipeoptim_arena_create / pipeoptim_arena_alloc (one call per
 * tensor for its W, g, m, v, What buffers) and calls pipeoptim_plan_localize once after pipeoptim_plan_create: the
 * kernels then keep every XCC of the chip on its own I/O die's HBM (about 4 % faster on a large stage).  A caller
 * that places the memory itself calls pipeoptim_plan_learn_layout once instead (about 3 % faster).
 *
 * Conventions for every function
 *   - extern "C"; returns PO_OK (0) or a negative po_status; never throws.
 *   - Tensor pointers are DEVICE pointers.  Who owns the memory behind them:
 *       * Buffers the caller allocated (e.g. through PyTorch) stay the caller's: the plan_* and step/predict
 *         calls never allocate, free, move or keep tensor memory; a plan owns only its own small tables
 *         (tensor descriptors + chunk table on the device, their pinned staging copies on the host).
 *       * Buffers handed out by pipeoptim_arena_alloc are device memory that the LIBRARY allocates (HIP virtual
 *         memory management) and owns: they live until pipeoptim_arena_destroy, the caller only uses them.
 *         A caller opts into that by creating an arena; nothing else in the library allocates tensor memory.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Work is enqueued and not waited for, except where a function says it
 *     waits.  No call that a training loop makes per step (pipeoptim_step_predict, pipeoptim_predict,
 *     pipeoptim_plan_set_pointers) waits for the device or for a stream; the set-up calls that do say so.
 *   - On failure nothing is launched and pipeoptim_last_error() describes it.
 *   - Calls on one plan (or one arena) must not overlap in time: give each host thread its own plan, or serialise.
 */
#ifndef PIPEOPTIM_H
#define PIPEOPTIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PO_OK = 0,
    PO_EINVAL = -1,  /* bad argument: NULL where a pointer is required, t < 1, s < 0, negative size,
                        beta outside [0,1), non-finite hyper-parameter, an optimizer whose state buffer the plan lacks,
                        launch shape outside the documented limits */
    PO_EALIGN = -2,  /* a tensor base pointer is not aligned to its element size */
    PO_EHIP   = -3,  /* a HIP call failed; the HIP error string is in pipeoptim_last_error() */
    PO_ENOMEM = -4   /* host or device allocation of the plan's tables failed */
} po_status;

/* 0-2: the rows of paper Table 1.  3-5: further optimizers by the table's own recipe (paper Sec. III-A.3: dW_t
 * follows from the update rule of the optimizer in use; by Eq. 1 it is the optimizer's increment over lr). */
typedef enum {
    PO_SGDM = 0, PO_ADAM = 1, PO_ADAMW = 2,
    PO_NESTEROV = 3,   /* momentum SGD with Nesterov look-ahead: state m                 */
    PO_RMSPROP  = 4,   /* RMSprop, no momentum, not centred: state v                     */
    PO_ADAGRAD  = 5    /* Adagrad, no learning-rate decay: state v (the running sum)     */
} po_optimizer;
typedef enum { PO_WHAT_F32 = 0, PO_WHAT_BF16 = 1 } po_what_dtype;       /* element type of What */
typedef enum { PO_GRAD_F32 = 0, PO_GRAD_BF16 = 1 } po_grad_dtype;       /* element type of g */

/*
 * Hyper-parameters, in double; the library derives the fp32 kernel coefficients
 * (including the bias corrections 1-beta1^t and 1-beta2^t of Table 1) itself.
 */
typedef struct po_hyper {
    int32_t opt;                  /* po_optimizer */
    int32_t decay_in_prediction;  /* AdamW only.  1: dW_t = r + wd*W, the whole per-step increment over lr,
                                     so that Eq. 1 holds and s = 1 predicts the optimizer's own step.
                                     0: the prediction uses Table 1's AdamW row alone (r); the step still decays. */
    double lr;
    double beta1;                 /* Adam/AdamW beta1;  SGDM, Nesterov: momentum factor u; RMSprop, Adagrad: ignored */
    double beta2;                 /* Adam/AdamW beta2;  SGDM: dampening tau;  RMSprop: smoothing constant alpha;
                                     Nesterov, Adagrad: ignored */
    double eps;                   /* epsilon, added after the root (Adam, AdamW, RMSprop, Adagrad); else ignored */
    double weight_decay;          /* AdamW: decoupled, W shrinks by lr*wd*W.  All others: coupled L2,
                                     g + wd*W enters the state update.                    */
} po_hyper;

/* fp32 coefficients one launch runs with (what the host derives from po_hyper, t and s). */
typedef struct po_coeffs {
    float beta1;          /* u or beta1                                   */
    float grad_scale;     /* 1 - tau or 1 - beta1                         */
    float beta2;          /* beta2 (0 for SGDM)                           */
    float one_m_beta2;    /* 1 - beta2 (0 for SGDM)                       */
    float inv_bc1;        /* 1 / (1 - beta1^t)          (1 for SGDM)      */
    float inv_sqrt_bc2;   /* 1 / sqrt(1 - beta2^t)      (1 for SGDM)      */
    float eps;
    float lr;             /* step:       W' = W - lr   * dW               */
    float s_lr;           /* prediction: What = W - s_lr * dW,  s_lr = s*lr */
    float wd_coupled;     /* wd for SGDM/Adam, else 0                     */
    float wd_step;        /* wd for AdamW, else 0 (decay inside the step's dW) */
    float wd_pred;        /* wd for AdamW with decay_in_prediction, else 0 */
    int32_t s_is_zero;    /* 1: What is a copy of W (last pipeline stage, paper Algorithm 1 else-branch) */
} po_coeffs;

/* One entry of the chunk table: elements [chunk * chunk_elems, min(numel, (chunk+1) * chunk_elems)) of `tensor`. */
typedef struct po_chunk {
    uint32_t tensor;
    uint32_t chunk;
} po_chunk;

/*
 * Launch shape of a kernel.  The grid has one workgroup per tile of block*4 elements (each lane moves 4
 * consecutive elements per stream, one dwordx4 access).
 *   block        64, 128 or 256 threads (64, the default, measured fastest at every stage size; the near-memory
 *                tile order is defined for it alone)
 *   lds_bytes    0..65536, unused LDS reserved per workgroup to cap how many workgroups a CU
 *                holds at once (160 KiB of LDS per CU); 0 = no cap; PO_LDS_AUTO (-1, the default) = chosen at
 *                each call from the kernel, the number of state streams of the optimizer in use and the size
 *                of the stage (pipeoptim_auto_lds_bytes tells the value)
 *   chunk_elems  granularity of the chunk table: block*4 times a power of two, at most 2^30
 * The number of chunks times chunk_elems/(block*4) must stay below 2^31.
 */
typedef struct po_launch {
    int32_t block;
    int32_t lds_bytes;
    int64_t chunk_elems;
} po_launch;

#define PO_LDS_AUTO (-1)
enum { PO_KERNEL_KIND_FUSED = 0, PO_KERNEL_KIND_PREDICT = 1 };

typedef struct po_plan po_plan;   /* opaque */

/*
 * Build a plan for a stage: n_tensors tensors, tensor i having numel[i] fp32
 * elements at W[i], g[i], m[i], v[i] (device) and a What[i] buffer of numel[i]
 * elements of what_dtype.  numel, W, g, m, v, What are HOST arrays of length
 * n_tensors.  v may be NULL (plan for SGDM / Nesterov only) and m may be NULL (plan for RMSprop /
 * Adagrad only); a call with an optimizer whose state is missing fails.  numel[i] == 0 and n_tensors == 0
 * are legal.  No two buffers of the plan may overlap (checked: PO_EINVAL); g is only read;
 * W, m, v are updated in place.  Buffers aligned to 16 bytes take the vector
 * path; 4-byte (What bf16: 2-byte) alignment is accepted and takes a scalar
 * path for that tensor.  The tables are uploaded with one asynchronous copy each, enqueued on `hip_stream`
 * from pinned staging memory that the plan owns: the call does not wait for the device or for the stream.
 * A later launch of the plan on another stream is made to wait for the upload by the library (an event), so
 * the plan can be used on any stream of the device right away.  (That wait is an ordinary hipStreamWaitEvent: the
 * first launch on a stream other than the upload's must not be recorded under stream capture; launch once before
 * capturing, or create the plan on the stream that will be captured.)
 * The caller keeps all buffers alive and at the same addresses while the plan lives.
 */
int pipeoptim_plan_create(po_plan** out, int64_t n_tensors, const int64_t* numel,
                          float* const* W, const float* const* g, float* const* m, float* const* v,
                          void* const* What, int32_t what_dtype, void* hip_stream);

/*
 * As pipeoptim_plan_create, with the element type of the gradients chosen by grad_dtype: mixed-precision
 * training hands the optimizer bf16 gradients next to fp32 master weights and state.  A bf16 gradient is
 * widened exactly to fp32 before it enters Table 1's update; everything else is unchanged.  g[i] then
 * points to numel[i] bf16 values (2-byte aligned; 16-byte aligned for the vector path).
 */
int pipeoptim_plan_create_mixed(po_plan** out, int64_t n_tensors, const int64_t* numel,
                                float* const* W, const void* const* g, int32_t grad_dtype,
                                float* const* m, float* const* v, void* const* What, int32_t what_dtype,
                                void* hip_stream);

/* Frees the plan's tables.  Waits first for the two streams the plan used last (that of its latest launch and
 * that of its latest table upload), not for the device: launches of the plan that are still pending on any
 * other stream are the caller's to wait for.  NULL is a no-op. */
int pipeoptim_plan_destroy(po_plan* plan);

/* Replace one pointer column (which: 0 W, 1 g, 2 m, 3 v, 4 What) with n_tensors new device pointers
 * (host array), e.g. when gradient buffers are re-allocated between steps.  May be called every step: the new
 * descriptors go to the device with one asynchronous copy enqueued on `hip_stream`, ordered like any other work
 * there (after the launches already enqueued on it, before the later ones); nothing is waited for.  Uploads of one
 * plan land in call order whatever streams they are issued on (each is chained behind the previous one).  Launches of
 * the plan enqueued afterwards on another stream wait for the copy (an event); launches enqueued BEFORE the call
 * on another stream and still running are the caller's to order, as for any write to memory a kernel reads.
 * On failure the plan is left exactly as it was.  Clears the near-memory marks of pipeoptim_plan_localize, and those of
 * pipeoptim_plan_learn_layout unless only g or What move (see there).  Not meant
 * to be recorded under stream capture: the two staging buffers are recycled with host-side waits on their events. */
int pipeoptim_plan_set_pointers(po_plan* plan, int32_t which, void* const* ptrs, void* hip_stream);

/* Get / set the launch shape of the fused kernel.  A set-up call: if chunk_elems changes, set rebuilds the
 * chunk table, waits for the plan's latest launch and upload streams (a running launch may still read the old
 * table), and uploads the new one on the stream of the latest upload.  The prediction kernel shares the table:
 * if its tile no longer divides the new chunk_elems by a power of two, its block is reset to this launch's. */
int pipeoptim_plan_get_launch(const po_plan* plan, po_launch* out);
int pipeoptim_plan_set_launch(po_plan* plan, const po_launch* launch);

/* Host only: the lds_bytes a call resolves PO_LDS_AUTO to, for kernel (PO_KERNEL_KIND_*), optimizer and stage size. */
int pipeoptim_auto_lds_bytes(int32_t kernel, int32_t opt, int64_t n_params, int32_t* out);

/* Totals of a plan: parameters, chunk-table entries, tensors on the scalar (unaligned) path. */
int pipeoptim_plan_info(const po_plan* plan, int64_t* n_params, int64_t* n_chunks, int64_t* n_unaligned);

/*
 * Near-memory arena (nothing in the paper corresponds to it: it is this library's own placement of the memory that
 * the update of paper Table 1 / Eq. 1 / Eq. 5 streams through).  MI355X has two I/O dies with four XCCs and four HBM stacks each; physical memory alternates
 * between the dies in 8 KiB blocks (address bit 13 hashed with higher physical address bits), and an XCC reaches
 * the other die's memory more slowly and over a shared link.  An arena hands out device memory whose block-to-die
 * layout is known (it creates the memory in 2 MiB pieces with HIP's virtual memory management, finds each piece's
 * layout by timing loads, and sorts the pieces into two virtual ranges), so that the kernels can give every XCC
 * the tiles that live on its own die: see pipeoptim_plan_localize.  For callers that let the library place the
 * stage's tensors, in the way optimizers with flat parameter buffers do.
 *
 * pipeoptim_arena_create: reserves address space for capacity_bytes per layout class on the current device (an
 *   MI355X in one partition, else PO_EINVAL); physical memory is created as allocations need it.
 * pipeoptim_arena_alloc: n_buffers buffers of bytes[k] bytes (host arrays), all with the same layout, each 16 KiB
 *   aligned; meant for the streams of ONE tensor (W, g, m, v, What).  Buffers of 1 MiB and more are set apart by
 *   a further gap (pipeoptim_arena_set_skew, default 512 KiB, a multiple of 16 KiB) so that equal-sized streams do
 *   not meet in the same HBM stack at the same element offset.  Blocking (it may run timing kernels and waits
 *   for the device); nothing is ever freed before pipeoptim_arena_destroy.  PO_ENOMEM when a range is full.
 * pipeoptim_arena_near_half: *half = the XCC half (0: XCCs 0-3, 1: XCCs 4-7) whose die holds the 8 KiB block
 *   around ptr, or -1 if ptr is not inside memory the arena handed out.
 * pipeoptim_arena_info: bytes backed by physical memory, bytes handed out (gaps included), pieces given up because
 *   timing could not tell their layout, and the near / far load latency (cycles) of the piece timed last.
 * pipeoptim_arena_check: times every backed 2 MiB piece again, in place, and counts those whose faster block is not
 *   the one the arena's layout rule says is near (*n_disagree of the *n_timed pieces that could be told apart): a
 *   diagnostic of the placement, independent of the sorting pass.  Blocking; about 10 ms per GiB.
 * pipeoptim_arena_destroy: waits for the device, then unmaps and frees everything; destroy plans over the
 *   arena's memory first.  NULL is a no-op.
 * Calls on one arena must not overlap.
 */
typedef struct po_arena po_arena;   /* opaque */
int pipeoptim_arena_create(po_arena** out, int64_t capacity_bytes);
int pipeoptim_arena_alloc(po_arena* arena, int64_t n_buffers, const int64_t* bytes, void** ptrs);
int pipeoptim_arena_set_skew(po_arena* arena, int64_t skew_bytes);
int pipeoptim_arena_near_half(const po_arena* arena, const void* ptr, int32_t* half);
int pipeoptim_arena_info(const po_arena* arena, int64_t* backed_bytes, int64_t* used_bytes, int64_t* released_pieces,
                         int32_t* near_cycles, int32_t* far_cycles);
int pipeoptim_arena_check(po_arena* arena, int64_t* n_timed, int64_t* n_disagree);
int pipeoptim_arena_destroy(po_arena* arena);

/*
 * Marks every tensor of the plan whose fp32 streams (W, m, v, fp32 g, fp32 What) all came from one
 * pipeoptim_arena_alloc call of `arena` (same layout class, 16 KiB aligned); both kernels then process such a
 * tensor in the near-memory tile order: of 16 consecutive workgroups (two rounds over the 8 XCCs, which take
 * workgroups round-robin) the eight on XCCs 0-3 take the 8 KiB block of each stream that lies on their die, the
 * other eight the other block.  Only with 256-element tiles (block 64) and chunk_elems >= 4096; any other launch
 * shape, and every tensor not marked, keeps the plain order.  Results do not depend
 * on the order.  arena == NULL clears all marks; pipeoptim_plan_set_pointers clears them too.  *n_local_params
 * (may be NULL) receives the number of parameters marked.
 * On which XCC a launch's round starts depends on the hardware queue behind the stream.  This call finds out for
 * hip_stream with a tiny kernel; after that every launch of the plan reports where it started (one word written to
 * pinned host memory) and the next call uses what it finds there, so a plan that moves to another stream runs one
 * launch with the old value (slower, never wrong) before it follows.  A set-up call: waits for hip_stream (the
 * tiny kernel's answer), not for the device; the descriptors are then uploaded on hip_stream like in
 * pipeoptim_plan_set_pointers.
 */
int pipeoptim_plan_localize(po_plan* plan, const po_arena* arena, void* hip_stream, int64_t* n_local_params);

/*
 * The near-memory tile order for buffers the CALLER placed (e.g. plain PyTorch allocations): the library cannot choose
 * where they lie, but it can find out.  Times a few loads in every whole 2 MiB piece inside the union of the plan's fp32
 * buffers (loads only: nothing is written; two independent timings per piece must agree), and then decides chunk by
 * chunk of the chunk table which XCC half takes which 8 KiB of each 16 KiB of the chunk's elements: the assignment that
 * makes more of the chunk's bytes near wins (W, m, v weigh 8 bytes per element, g and an fp32 What 4; a stream that
 * starts on an 8 KiB boundary, as every large allocation does, votes with all of its bytes, one that starts o bytes
 * into a block with (8192 - o) : o, one 4 KiB off has no say).  Where all streams of a chunk agree every access is
 * near, where they split evenly nothing is lost against the plain order; measured on MI355X, plain PyTorch allocations
 * of 75 M to 738 M parameters: 0.73-0.91 of the traffic near instead of half, 3-5 % faster than the plain order.
 * Needs chunk_elems between 4096 and 524288 and 256-element tiles (block 64), else PO_EINVAL.
 * Results do not depend on the order.  A set-up call: waits for the device (the timing wants the memory system to
 * itself), about 10 ms per GiB of buffers.  pipeoptim_plan_set_pointers of W, m or v, a chunk_elems change and
 * pipeoptim_plan_localize drop what was learnt (learn again after them); new g or What pointers do not: the order was
 * decided mostly by the three heavier streams and stays in force.  *n_local_params (may be NULL) receives the
 * number of parameters in chunks that got an order of their own.
 */
int pipeoptim_plan_learn_layout(po_plan* plan, void* hip_stream, int64_t* n_local_params);

/*
 * Host-only (touches no device; testable without a GPU): the vote pipeoptim_plan_learn_layout takes for one chunk.
 * Stream j (at most 5) holds the chunk's `elems` fp32 elements from address first_byte[j] on and moves weight[j] bytes
 * of the call's traffic per element; piece_addr[k] (2 MiB aligned, ascending) are the pieces whose layout is known,
 * even_blocks_near[k] the XCC half (0, 1; -1 unknown) near to the piece's 8 KiB blocks with address bit 13 clear.
 * near[h] receives the bytes of traffic that giving the first 8 KiB of every 16 KiB of the chunk's elements to XCC
 * half h would make near; the larger one wins, bytes in pieces that are not listed count for neither.
 */
int pipeoptim_chunk_vote(int32_t n_streams, const uint64_t* first_byte, const int32_t* weight, int64_t elems,
                         int64_t n_pieces, const uint64_t* piece_addr, const int8_t* even_blocks_near, double* near);

/* Host-only: which memory pipeoptim_plan_learn_layout may time.  Given n_ranges byte ranges [lo[k], hi[k]) (the plan's
 * fp32 buffers; any order, may touch or overlap), the runs of whole 2 MiB-aligned pieces every byte of which lies in
 * at least one range: run j is [piece_lo[j], piece_hi[j]), ascending; *n_runs = their number (at most `capacity` are
 * written).  Nothing outside these runs is ever read by the timing. */
int pipeoptim_whole_pieces(int64_t n_ranges, const uint64_t* lo, const uint64_t* hi, uint64_t* piece_lo, uint64_t* piece_hi,
                           int64_t capacity, int64_t* n_runs);

/* Diagnostic: out[k] (k < capacity) = what pipeoptim_plan_learn_layout decided for chunk-table entry k: -1 plain order,
 * 0 / 1 the XCC half that takes the first 8 KiB of every 16 KiB of the chunk's elements; *n_chunks = entries in the table. */
int pipeoptim_plan_chunk_marks(const po_plan* plan, int8_t* out, int64_t capacity, int64_t* n_chunks);

/* Diagnostic: *share = the estimated share of the fused call's HBM bytes that are served by the memory of the die the
 * workgroup runs on: 0.5 in the plain order (every XCC's traffic is half near, half far), up to (all fp32 streams)
 * / (all streams) + half of the bf16 streams for a plan localized over an arena (0.98 for AdamW with bf16 What), and
 * what the votes of pipeoptim_plan_learn_layout added up to for a learnt order (0.71 when the four fp32 streams of each
 * tensor lie independently; pieces whose layout could not be told count as half near).  As of the last
 * pipeoptim_plan_localize / pipeoptim_plan_learn_layout call. */
int pipeoptim_plan_near_share(const po_plan* plan, double* share);

/* The XCC (0-7) on which the last launch of a localized plan that has reported so far started its round, i.e. the
 * value the next call will hand to its kernel; -1 for a plan that was never localized.  Does not wait for anything. */
int pipeoptim_plan_launch_phase(const po_plan* plan, int32_t* phase);

/* Parameters of the plan's tensors that are marked for the near-memory tile order right now. */
int pipeoptim_plan_local_params(const po_plan* plan, int64_t* n_local_params);

/* Host only: the launch shape a call of the given kernel (PO_KERNEL_KIND_*) and optimizer would run with
 * (PO_LDS_AUTO resolved for this plan, including whether it is localized). */
int pipeoptim_plan_effective_launch(const po_plan* plan, int32_t kernel, int32_t opt, po_launch* out);

/* Host only: the near-memory tile order.  *out = the tile (within its chunk) that the workgroup at position
 * tile_in_chunk processes when the first 8 KiB block of every 16 KiB group is near to XCC half first_block_half
 * (0 or 1).  A bijection on every aligned run of 16 positions. */
int pipeoptim_local_tile(uint32_t tile_in_chunk, int32_t first_block_half, uint32_t* out);

/* Host only: the rotation in front of it.  *out = the position (chunk * tiles per chunk + tile_in_chunk) that workgroup
 * id `workgroup` of a launch of n_slots workgroups (a multiple of 8) takes when the queue starts its launches on XCC
 * `phase` (0-7): position p then runs on XCC p mod 8. */
int pipeoptim_local_slot(uint32_t workgroup, uint32_t phase, uint32_t n_slots, uint32_t* out);

/*
 * The hot path.  For every element of every tensor of the plan, with dW_t from
 * paper Table 1 (built from the new gradient and the cached state):
 *     SGDM : g~ = g + wd*W;  m' = u*m + (1-tau)*g~;  dW = m'
 *     Adam : g~ = g + wd*W;  m' = b1*m + (1-b1)*g~;  v' = b2*v + (1-b2)*g~^2
 *            dW = (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps)
 *     AdamW: as Adam with g~ = g;  dW = r + wd*W  (prediction: r alone if !decay_in_prediction)
 *   and, beyond Table 1, by the same recipe:
 *     Nesterov: g~ = g + wd*W;  m' = u*m + g~;  dW = g~ + u*m'
 *     RMSprop : g~ = g + wd*W;  v' = alpha*v + (1-alpha)*g~^2;  dW = g~ / (sqrt(v') + eps)
 *     Adagrad : g~ = g + wd*W;  v' = v + g~^2;                  dW = g~ / (sqrt(v') + eps)
 *     W'   = W - lr*dW                      (paper Eq. 1)
 *     What = W - lr*s*dW                    (paper Eq. 5);  s == 0: What = W
 * in fp32 arithmetic.  W, m, v are overwritten with W', m', v'; What receives
 * the prediction (bf16: round-to-nearest-even).  t >= 1 is the 1-based step
 * index of the bias corrections; s >= 0 is the version difference of paper
 * Eq. 4.  Enqueues exactly one kernel on hip_stream and returns.  hip_stream must belong to the
 * device that was current when the plan was created, and that device must be current (else PO_EINVAL).
 */
int pipeoptim_step_predict(const po_plan* plan, const po_hyper* hyper, int64_t t, int32_t s,
                           void* hip_stream);

/*
 * For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The same update as pipeoptim_step_predict, for a ragged list handed over in the call itself instead
 * of a plan (arguments as in pipeoptim_plan_create, fp32 gradients; hyper, t, s as in pipeoptim_step_predict).
 * The call allocates nothing on the device and calls no allocating HIP routine (its argument checks use a little
 * ordinary host heap memory, freed before it returns): the tensor descriptors and the chunk table that a
 * plan keeps in memory of its own live here in a fixed device array inside the library (64 KiB + 512 KiB per
 * GPU the library runs on, held until the process ends).  The descriptors reach it inside kernel arguments, the
 * chunk table is built from them on the device, then the fused kernel runs: 2 + ceil(n_tensors / 48) small
 * kernels in front of the one that does the work, all enqueued on hip_stream, nothing waited for.
 * Limits: at most PO_STATIC_MAX_TENSORS tensors and PO_STATIC_MAX_CHUNKS chunk-table entries of 65,536 elements
 * (sum over tensors of ceil(numel / 65536); 4.2 G parameters in large tensors); beyond them PO_EINVAL, nothing
 * launched.  Launch shape: the default one (block 64, occupancy cap chosen for optimizer and stage size).
 * Every call on a GPU uses that GPU's one array: calls on the same stream follow each other safely; calls that
 * overlap in time on different streams of one GPU race on the tables and must be ordered by the caller.
 */
#define PO_STATIC_MAX_TENSORS 1024
#define PO_STATIC_MAX_CHUNKS 65536
int pipeoptim_step_predict_static(int64_t n_tensors, const int64_t* numel, float* const* W, const float* const* g,
                                  float* const* m, float* const* v, void* const* What, int32_t what_dtype,
                                  const po_hyper* hyper, int64_t t, int32_t s, void* hip_stream);

/*
 * Prediction alone, from the cached optimizer state: how paper Algorithm 1 sequences it (cached
 * state -> dW_t by Table 1 -> Eq. 5, ahead of the forward pass), for callers whose optimizer step
 * ran elsewhere or that need What again for another s.  Reads W, m (, v); reads no gradient;
 * writes only What:
 *     SGDM : dW = m
 *     Adam : dW = (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)        with m, v as stored
 *     AdamW: dW = that + wd*W   (r alone if !decay_in_prediction)
 *     What = W - lr*s*dW;  s == 0: What = W
 * t is the 1-based index of the step that produced the stored m, v.  Called right after
 * pipeoptim_step_predict(t, .) it predicts from the stepped weights: W' - lr*s*dW_t, which equals the
 * fused call's own prediction for s+1 (for AdamW up to the decay term being taken at W' instead of W).
 * With SGDM and the previous step's momentum it is SpecTrain's predictor (paper Eq. 6, first line).
 * Only the Table 1 optimizers have a direction that follows from the state alone; Nesterov, RMSprop and
 * Adagrad need the gradient and are rejected here (PO_EINVAL).
 * Enqueues exactly one kernel; uses the launch shape set with pipeoptim_plan_set_predict_launch (default: the
 * fused kernel's default shape, with the occupancy cap chosen for this kernel).
 */
int pipeoptim_predict(const po_plan* plan, const po_hyper* hyper, int64_t t, int32_t s, void* hip_stream);

/* Launch shape of pipeoptim_predict's kernel (same fields and limits; chunk_elems must equal the
 * plan's chunk_elems, i.e. the one of pipeoptim_plan_get_launch, or be 0 to mean that). */
int pipeoptim_plan_get_predict_launch(const po_plan* plan, po_launch* out);
int pipeoptim_plan_set_predict_launch(po_plan* plan, const po_launch* launch);

/* Paper Eq. 4: s = D - rank - 1 for stage `rank` (0-based) of a depth-D pipeline.  PO_EINVAL unless 0 <= rank < D. */
int pipeoptim_version_difference(int32_t D, int32_t rank, int32_t* s_out);

/* Host only: the fp32 coefficients pipeoptim_step_predict would launch with (validates hyper, t, s). */
int pipeoptim_coefficients(const po_hyper* hyper, int64_t t, int32_t s, po_coeffs* out);

/*
 * Host only: the chunk table for a ragged list.  Writes up to `capacity` entries to out (may be NULL
 * with capacity 0 to count) and the total to *n_chunks.  Tensors appear in list order, chunks of a
 * tensor in ascending order, empty tensors contribute none.
 */
int pipeoptim_chunk_table_build(int64_t n_tensors, const int64_t* numel, int64_t chunk_elems,
                                po_chunk* out, int64_t capacity, int64_t* n_chunks);

/* Measurement aid: dst[0..nbytes) = src[0..nbytes) with a plain streaming dwordx4 copy kernel (device
 * pointers, 16-byte aligned, nbytes a multiple of 16, below 2^41).  Gives the box's achievable
 * one-read-one-write bandwidth. */
int pipeoptim_probe_copy(void* dst, const void* src, int64_t nbytes, void* hip_stream);

/* Measurement aid: the same copy in the near-memory tile order, the yardstick for one read plus one write stream
 * with every XCC on its own die's memory.  dst and src: 16 KiB aligned, from ONE pipeoptim_arena_alloc call of
 * `arena`; nbytes a multiple of 16 KiB; lds_bytes (0..65536) caps the occupancy as in po_launch.  Like a localized
 * plan, it learns the XCC on which the stream's launches start from its own previous launch (run it twice). */
int pipeoptim_probe_copy_near(const po_arena* arena, void* dst, const void* src, int64_t nbytes, int32_t lds_bytes,
                              void* hip_stream);

/* Thread-local description of the last failure on this thread ("" if none). */
const char* pipeoptim_last_error(void);

/* Diagnostic: how many times this process's library has waited for the WHOLE device (hipDeviceSynchronize) so
 * far.  Only the arena calls and the fallbacks of pipeoptim_plan_destroy / pipeoptim_plan_set_launch (a stream
 * of the plan no longer exists) ever do; tests use the counter to show that the per-step calls do not. */
int pipeoptim_device_sync_count(int64_t* count);

#ifdef __cplusplus
}
#endif
#endif /* PIPEOPTIM_H */

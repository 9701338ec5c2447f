/*
 * zi.h — C ABI of the MI355X (gfx950) optimizer hot path for offloaded,
 * partitioned mixed-precision training.
 *
 * The library performs, on ONE GPU, the per-rank optimizer step over the model
 * states a data-parallel process owns (Section 2, "ZeRO": each process updates
 * only the optimizer states of the parameters it owns):
 *
 *   zi_grad_norm            global L2 norm of the low-precision gradients and
 *                           the inf/NaN flag of dynamic loss scaling;
 *   zi_adamw_step           fused AdamW over fp32 parameters, momentum and
 *                           variance with low-precision gradients, writing the
 *                           low-precision parameter copy (Section 3, "Memory
 *                           for Model States": which arrays exist and in which
 *                           precision; Section 2, "Adam Optimizer and Mixed
 *                           Precision Training": updates are done in fp32);
 *   zi_adamw_step_streamed  the same step when the fp32 states live in pinned
 *                           host memory and move through HBM in fixed-size
 *                           chunks, with reads, compute and writes overlapped
 *                           through a small ring of reused staging buffers
 *                           (Section 5.2.2: chunked step, overlap of reads,
 *                           writes and compute; Section 6.3: reused pinned
 *                           buffers).
 *
 * The step reads every state once and writes it once (Section 4.1, "AIT w.r.t.
 * Optimizer States"): 28 bytes per element here (read p, m, v 4 B each and g
 * 2 B; write p, m, v and the 2-byte copy).
 *
 * The paper cites Adam and mixed-precision training without printing their
 * equations.  The arithmetic is the standard definition, in this fixed binary32
 * order (round to nearest even, fused multiply-add only where fma is written):
 *
 *   g  = widen(g_lp) * gscale                gscale = clip / loss_scale
 *   [ZI_MODE_ADAM_L2 only]  g = fma(weight_decay, p, g)
 *   m' = fma(beta1, m, (1-beta1) * g)
 *   v' = fma(beta2, v, (1-beta2) * (g * g))
 *   d  = fma(sqrt(v'), 1/sqrt(1-beta2^step), eps)
 *   q  = m' / d
 *   pd = fma(-(lr*weight_decay), p, p)       [ZI_MODE_ADAMW; pd = p otherwise]
 *   p' = fma(-(lr/(1-beta1^step)), q, pd)
 *   p_lp = round_to_nearest_even(p')         bf16 or fp16, subnormals kept
 *
 * with norm = sqrt(sum g_lp^2) / loss_scale and
 * clip = max_grad_norm / (norm + 1e-6) if that is below 1, else 1.
 * All per-step scalars are evaluated in double and rounded once to fp32.
 * If any gradient is +-inf or NaN the step is skipped: no byte of any state
 * changes.
 *
 * General conventions
 *   - Every pointer is a plain address.  "device" = HBM of the current HIP
 *     device; "pinned host" = page-locked host memory (zi_pinned_alloc or any
 *     hipHostMalloc'd block).  The caller owns every buffer it passes; the
 *     library keeps nothing after a call returns, except inside a zi_engine.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *   - Functions return a zi_status; negative values are errors and leave every
 *     buffer untouched unless stated otherwise.  Nothing throws or aborts.
 *     zi_last_error() gives the text of the calling thread's last error.
 *   - Pointers must be aligned to their element size (4 bytes for p/m/v, 2
 *     bytes for g and p_lp); nothing more is required.  The step is fastest
 *     when all arrays of a tensor sit at the same offset from a 128-byte
 *     boundary, counted in elements (true for separately allocated arrays and
 *     for views that start at the same element of aligned buffers): then all
 *     of its traffic runs in whole 128-byte lines.  Other placements use the
 *     same kernel and give identical results, within a few percent of that
 *     speed.
 *   - Every array a kernel will touch is checked at its first and last byte before anything is launched:
 *     it must be device or page-locked host memory (both reachable by the GPU).  An ordinary host
 *     pointer is ZI_ERR_INVALID_ARG, never a GPU memory fault.
 *   - numel == 0 and n_tensors == 0 are valid and do nothing.
 *   - Threads: calls that do not share buffers or an engine may run concurrently from different
 *     threads.  An engine serves one call at a time.  zi_last_error() is per thread.
 *   - The library is gfx950-only and has no CPU fallback: without a usable HIP
 *     device every compute call returns ZI_ERR_HIP.
 */
#ifndef ZI_H
#define ZI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZI_OK = 0,
    ZI_SKIPPED_OVERFLOW = 1,   /* streamed step only: gradients held inf/NaN, nothing moved */
    ZI_ERR_INVALID_ARG = -1,
    ZI_ERR_UNSUPPORTED = -2,
    ZI_ERR_ALIGNMENT = -3,
    ZI_ERR_HIP = -4,
    ZI_ERR_NOMEM = -5,
    ZI_ERR_IO = -6
} zi_status;

typedef enum { ZI_BF16 = 0, ZI_FP16 = 1 } zi_lp_dtype;
typedef enum { ZI_MODE_ADAMW = 0, ZI_MODE_ADAM_L2 = 1 } zi_mode;

/* Hyper-parameters of one step.  Plain data, passed by pointer, read during the call only. */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int64_t step;          /* 1-based index of the step being taken; never modified */
    float loss_scale;      /* > 0 and finite; 1 = none; raw gradients are divided by it */
    float max_grad_norm;   /* <= 0: no clipping; needs a norm result to have any effect */
    int32_t mode;          /* zi_mode */
} zi_adamw_config;

/* Result of zi_grad_norm.  Lives in DEVICE memory, 8-byte aligned, 32 bytes.  The last two
 * fields are derived values the library writes together with `norm` so that the step's kernels
 * need not recompute them in every wavefront; a caller never sets them. */
typedef struct {
    double sumsq;          /* sum of squares of the raw (still loss-scaled) gradients */
    double norm;           /* sqrt(sumsq) / loss_scale; meaningful only if found_inf == 0 */
    uint32_t found_inf;    /* 1 if any gradient element is +-inf or NaN, else 0 */
    uint32_t scale_bits;   /* bit pattern of the (float) loss scale `norm` was divided by */
    double inv_norm;       /* 1 / (norm + 1e-6): the clip factor for a maximum norm of 1 */
} zi_norm_result;

/* One tensor of the owned partition.  All arrays hold numel elements. */
typedef struct {
    void* p;               /* fp32 master parameters, updated in place */
    void* m;               /* fp32 momentum, updated in place */
    void* v;               /* fp32 variance, updated in place */
    const void* g;         /* low-precision gradients, read only (device; the streamed calls also take host) */
    void* p_lp;            /* low-precision parameter copy, written; may be NULL (device; streamed: or host) */
    int64_t numel;
} zi_tensor;

/* Text of the calling thread's last error ("" if none).  Never NULL.  Host pointer, owned by the library. */
const char* zi_last_error(void);

/*
 * Bytes of device scratch zi_grad_norm needs (per-block partial sums; a fixed,
 * small size that does not grow with the inputs).  Never fails.
 */
size_t zi_norm_workspace_bytes(int64_t total_numel, int32_t n_tensors);

/*
 * Global gradient norm and overflow flag (the mixed-precision recipe of Section
 * 2 implies dynamic loss scaling; the rule used is the standard one):
 *   sumsq = sum over all tensors of g_lp^2 (accumulated in double),
 *   norm = sqrt(sumsq) / loss_scale, found_inf = any element with an all-ones
 *   exponent field.
 * Only t[i].g and t[i].numel are read (device pointers; p/m/v/p_lp ignored).
 * d_out: device, 8-byte aligned, written by the kernels on hip_stream.
 * d_workspace: device, 16-byte aligned, >= zi_norm_workspace_bytes(); contents
 * need no initialisation and are garbage afterwards.  Asynchronous: returns
 * once the work is enqueued.  Two calls that share a workspace must be ordered
 * on one stream.
 */
zi_status zi_grad_norm(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                       zi_norm_result* d_out, void* d_workspace, size_t workspace_bytes, void* hip_stream);

/*
 * zi_grad_norm for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * same result struct, same kernels; the per-block partials go to a fixed array of
 * ZI_NOALLOC_MAX_PARTIALS * 16 bytes (256 KiB) inside the library's device image, which every GPU the
 * library runs on holds until the process ends.  The call itself allocates nothing, on the device or
 * on the host.
 * Limit: at most ZI_NOALLOC_MAX_PARTIALS non-empty tensors per call (ZI_ERR_UNSUPPORTED beyond,
 * nothing launched); within it any sizes are accepted, long tensors simply get fewer workgroups so
 * that all partials of the call fit the array in one pass.  The sum is accumulated in double in a
 * different grouping than zi_grad_norm's when that happens (agreement ~1e-15 relative), and is
 * bit-identical otherwise.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different
 * streams or threads) race on it and give garbage; order them on one stream or with events.  Nothing in
 * the array needs clearing between calls: every partial the final pass reads was written by this call.
 * The device address of the array is looked up on the first call on each device (that first call must
 * not be under capture).  Asynchronous on hip_stream.
 */
#define ZI_NOALLOC_MAX_PARTIALS 16384
zi_status zi_grad_norm_noalloc(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                               zi_norm_result* d_out, void* hip_stream);

/*
 * Hook for a sharded run (Section 2, "ZeRO": every data-parallel process owns a slice of each
 * parameter and steps only that slice; the clip factor needs the norm over ALL slices).  Each rank
 * calls zi_grad_norm on its slice; the caller then combines the results across ranks, in place in
 * device memory, with whatever collective it uses (sumsq: sum, found_inf: max, 12 bytes in all);
 * zi_norm_refresh recomputes d_result->norm = sqrt(sumsq) / loss_scale from the combined sum, after
 * which zi_adamw_step proceeds as on one GPU.  The library itself issues no collective.
 * Asynchronous on hip_stream.
 */
zi_status zi_norm_refresh(zi_norm_result* d_result, float loss_scale, void* hip_stream);

/*
 * Fused AdamW step over HBM-resident state (Sections 3 and 4.1; equations in
 * the header comment).  All arrays of every tensor are device memory; p, m, v
 * are updated in place and p_lp (if not NULL) receives the low-precision copy.
 * No two arrays may overlap: within a tensor the five byte ranges are checked
 * pairwise (ZI_ERR_INVALID_ARG); arrays of different tensors must not overlap
 * either (not checked).
 * d_norm: device result of zi_grad_norm on the same gradients, or NULL.  With
 * NULL there is no overflow check and no clipping: gscale = 1 / loss_scale.
 * With a result, the kernels read it on the device: found_inf != 0 skips the
 * whole step, otherwise the clip factor follows from norm = sqrt(sumsq) /
 * cfg->loss_scale.  The result's own `norm` field is taken for that value only
 * when its `scale_bits` field says it was divided by cfg->loss_scale (the
 * library writes the two together); a result reduced with any other scale
 * has its norm derived again from `sumsq`, so the scale that was given to
 * zi_grad_norm cannot make the step clip wrongly.  A caller that edits
 * `sumsq` in place (a sharded run) calls zi_norm_refresh afterwards, which
 * rewrites `norm`, `scale_bits` and `inv_norm`.
 * Asynchronous on hip_stream; the return value is ZI_OK even when the device
 * will skip the step (read d_norm->found_inf to learn of it).
 */
zi_status zi_adamw_step(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, const zi_adamw_config* cfg,
                        const zi_norm_result* d_norm, void* hip_stream);

/*
 * Streaming engine: owns n_slots staging slots in HBM (each 4 arrays of
 * chunk_bytes_per_array: p, m, v, and one shared by staged gradients and a
 * staged low-precision copy), three HIP streams (host-to-device,
 * compute, device-to-host; all at default priority) and the events that order
 * slot reuse (Section 6.3: a small pool of reused buffers serves the whole
 * state).  Created once; step calls allocate no device or pinned memory and start no thread (the
 * ring's CPU threads are created with the ring and parked between calls; the host-side plan of a
 * call reuses buffers that grow only when a longer tensor list than ever before arrives).
 * chunk_bytes_per_array: positive multiple of 4096 (64 MiB is the usual value).
 * n_slots: 2..8.  device: HIP device ordinal.
 */
typedef struct zi_engine zi_engine;

zi_status zi_engine_create(zi_engine** out, int32_t device, size_t chunk_bytes_per_array, int32_t n_slots);
zi_status zi_engine_destroy(zi_engine* e);   /* NULL is accepted */

/*
 * AdamW step with p, m, v in PINNED HOST memory (or ordinary host memory if the
 * engine has a pinned ring, see zi_engine_set_option) and g, p_lp in device memory
 * (Section 5.2.2: the state is brought to the faster memory in chunks, one chunk
 * at a time, and written back, with reads, writes and compute overlapped).
 * Tensors larger than a chunk are split on chunk boundaries; consecutive small
 * tensors are packed into one slot.  Results are bit-identical to
 * zi_adamw_step on the same values.
 * The engine's streams first wait for the work already enqueued on hip_stream
 * (where the gradients and d_norm were produced).  If d_norm is given, its flag
 * is read back first; found_inf != 0 returns ZI_SKIPPED_OVERFLOW with no state
 * moved.  BLOCKING: returns after the last device-to-host copy has completed,
 * so the host arrays are valid on return; p_lp is complete as well.
 * On ZI_ERR_HIP part of the host state may already have been updated.
 */
zi_status zi_adamw_step_streamed(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                 const zi_adamw_config* cfg, const zi_norm_result* d_norm, void* hip_stream);

/*
 * Gradients and the low-precision copy need not be on the device for the streamed step: if
 * t[i].g (and / or t[i].p_lp) of zi_adamw_step_streamed is host memory (pinned, or ordinary with a
 * pinned ring), each chunk of gradients travels to HBM with its chunk of state, and the chunk of
 * the low-precision copy travels back with it (14 bytes per element each way instead of 12).
 * This is the gradient-side offload of Section 6.2 (gradients moved to slow memory during the
 * backward pass) seen from the optimizer step.  zi_grad_norm_streamed is the matching reduction:
 * as zi_grad_norm, but gradients in host memory are staged through the engine's slots chunk by
 * chunk (2 bytes per element over the link), overlapped with the reduction kernels; device-resident
 * gradients in the same list are reduced in place.  BLOCKING: returns when the result is in d_out.
 */
zi_status zi_grad_norm_streamed(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                                float loss_scale, zi_norm_result* d_out, void* d_workspace,
                                size_t workspace_bytes, void* hip_stream);

/*
 * Gradient offload as the gradients are produced (Section 6.2: during the backward pass each
 * gradient partition is moved to slow memory, overlapped with the computation that produces the
 * next one).  zi_grad_offload enqueues the copy of `bytes` from device memory d_src to PINNED host
 * memory h_dst on the engine's device-to-host stream, ordered after everything already enqueued on
 * producer_stream (an event recorded there), and returns at once: the producer stream is not
 * blocked and may go on with the next partition while this one drains.  d_src must stay untouched
 * until the copy is done.
 * Completion: zi_grad_offload_wait blocks the host until every offload issued so far has landed;
 * zi_grad_offload_order makes consumer_stream wait for them instead (no host blocking).
 * zi_grad_norm_streamed, zi_adamw_step_streamed and zi_adamw_step_cpu on the same engine order
 * themselves after outstanding offloads, so the host copies can be handed to them directly.
 * Calls on one engine must not overlap in time (an engine serves one call at a time).
 */
zi_status zi_grad_offload(zi_engine* e, const void* d_src, void* h_dst, size_t bytes, void* producer_stream);
zi_status zi_grad_offload_wait(zi_engine* e);
zi_status zi_grad_offload_order(zi_engine* e, void* consumer_stream);

/*
 * The step on the host CPUs with the link carrying only the 2-byte arrays (Section 5.2.2: with the
 * optimizer states in CPU memory the step runs on the CPUs; gradients come down, updated
 * low-precision parameters go up: 2 + 2 bytes per element over the link instead of 12 + 12).
 * p, m, v: host memory of any kind, updated in place by n_threads CPU threads (AVX2 / FMA / F16C,
 * the arithmetic of zi_host_adamw_step).  g, p_lp: DEVICE memory — each chunk of gradients is
 * fetched into the engine's pinned ring, stepped, and the chunk of the copy is shipped back, the
 * fetch of later chunks and the upload of earlier ones overlapping the CPUs' work — or host memory,
 * used in place.  Device-resident g / p_lp need ZI_OPT_HOST_RING_SLOTS >= 3.
 * d_norm: device result of zi_grad_norm or NULL; read back first; found_inf != 0 returns
 * ZI_SKIPPED_OVERFLOW with nothing touched.  The engine's streams first wait for hip_stream.
 * BLOCKING: on return the host state and p_lp are complete.  Results are bit-identical to
 * zi_adamw_step and zi_adamw_step_streamed on the same values.  This call is chosen explicitly;
 * no GPU entry point falls back to it.  ZI_ERR_UNSUPPORTED on a CPU without those instructions.
 */
zi_status zi_adamw_step_cpu(zi_engine* e, const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                            const zi_adamw_config* cfg, const zi_norm_result* d_norm, int32_t n_threads,
                            void* hip_stream);

/*
 * The same step with p, m, v in FILES (Section 5.2.2: with NVMe offload the state is brought to
 * faster memory and back in chunks, one chunk at a time; Section 6.3: bulk reads and writes issued
 * in parallel, into and out of reused pinned buffers, no further copies).  Each chunk is read by
 * the engine's CPU threads straight into a slot of the pinned ring (parallel pread), moved to HBM,
 * updated, moved back and written out (parallel pwrite); reads, host-link copies, the kernel and
 * writes of different chunks overlap.  Needs ZI_OPT_HOST_RING_SLOTS.
 * fd_*: descriptors open O_RDWR; the caller keeps and closes them.  off_*: byte offset of the
 * array inside its file (multiple of 4).  Descriptors opened with O_DIRECT are supported and
 * recommended for NVMe: then every offset must be a multiple of 4096, no two arrays may share a
 * 4096-byte block of a file, and transfers are rounded up to whole
 * blocks (a file whose last region is not a multiple of 4096 bytes grows to the block boundary).
 * Direct I/O passes through a small per-thread aligned buffer in ordinary memory, because memory
 * from the HIP page-locked allocator cannot itself be the target of direct I/O; buffered
 * descriptors read and write the pinned ring in place.
 * g, p_lp: device or host memory, as in zi_adamw_step_streamed (with O_DIRECT the device-resident one
 * of them, if any, must be 8-byte aligned).  Blocking; data is written with pwrite,
 * not synced (call fsync/fdatasync if durability is needed).  Results are bit-identical to
 * zi_adamw_step on the same values.  A bad descriptor is ZI_ERR_INVALID_ARG; a failed or short read
 * or write is ZI_ERR_IO with the errno text in zi_last_error(), and part of the state may then
 * already have been updated.
 */
typedef struct {
    int32_t fd_p, fd_m, fd_v;
    int32_t reserved;
    int64_t off_p, off_m, off_v;
    const void* g;
    void* p_lp;
    int64_t numel;
} zi_file_tensor;

zi_status zi_adamw_step_files(zi_engine* e, const zi_file_tensor* t, int32_t n_tensors, zi_lp_dtype dt,
                              const zi_adamw_config* cfg, const zi_norm_result* d_norm, void* hip_stream);

/* Figures of the engine's last streamed step (host memory, filled by the call). */
typedef struct {
    double seconds;            /* first host-to-device issue .. last device-to-host completion */
    uint64_t bytes_h2d;
    uint64_t bytes_d2h;
    int64_t n_slot_uses;       /* chunk-slots processed */
    int64_t n_copies;          /* hipMemcpyAsync calls issued */
    int64_t n_kernels;         /* kernel launches */
    uint64_t bytes_staged_host; /* bytes copied by CPU threads through the pinned ring (both ways) */
} zi_stream_stats;

zi_status zi_engine_last_stats(const zi_engine* e, zi_stream_stats* out);

/*
 * Engine options.
 * ZI_OPT_SKIP_KERNEL = 1 runs the identical copy pipeline without launching the
 * update (a measurement aid like the calls of zi_probe.h: the time of the pipeline with the update
 * removed).
 * ZI_OPT_MAX_INFLIGHT selects how the host paces the pipeline.  0 (default, needs n_slots >= 3): a slot
 * use is issued when the copy-out of the use two positions back starts (its update is done);
 * the two directions of the link then run side by side one chunk apart and the update of the chunk
 * in between is hidden.  k >= 1: before issuing a slot use the host waits for the use k positions
 * back to FINISH (k = 2 also keeps the directions in lockstep but exposes the update once per chunk;
 * k = n_slots lets the copy-in stream run a whole slot ahead, which measured slower and unsteady).
 * ZI_OPT_HOST_RING_SLOTS = n gives the engine a ring of n pinned host slots
 * (each shaped like an HBM slot: 4 arrays of the chunk size) and two small CPU thread pools.  With it,
 * zi_adamw_step_streamed also accepts p, m, v in ORDINARY (pageable) host
 * memory: each chunk is copied into a ring slot by CPU threads, moved to HBM
 * and back by the copy engines, and copied out again, all stages overlapped
 * (Section 6.3, pinned memory management layer: a small reused pinned pool
 * serves model states far larger than what can be page-locked).  Results are
 * bit-identical to the pinned path.  Without a ring, pageable state is refused.
 */
typedef enum {
    ZI_OPT_SKIP_KERNEL = 0,
    ZI_OPT_HOST_RING_SLOTS = 1,    /* 0 = none (default); 2..16: allocate a pinned ring of that many slots */
    ZI_OPT_HOST_COPY_THREADS = 2,  /* 1..64 CPU threads per direction for the ring (default 6) */
    ZI_OPT_MAX_INFLIGHT = 3        /* 0 (default pacing) or 1..n_slots */
} zi_engine_option;
zi_status zi_engine_set_option(zi_engine* e, int32_t option, int64_t value);

/*
 * Chunk plan of the streamed step, as a pure host function (no GPU needed):
 * how a tensor list maps onto slot uses.  Segment i says that elements
 * [elem_offset, elem_offset + count) of tensor `tensor` travel in slot use
 * `slot_use` at element offset `slot_offset` inside the slot's arrays.
 * Writes at most `cap` segments to `out` (may be NULL when cap == 0) and always
 * stores the totals.  chunk_elems = chunk_bytes_per_array / 4.
 */
typedef struct {
    int32_t tensor;
    int32_t reserved;
    int64_t elem_offset;
    int64_t count;
    int64_t slot_use;
    int64_t slot_offset;
} zi_chunk_segment;

zi_status zi_plan_chunks(const int64_t* numel, int32_t n_tensors, int64_t chunk_elems, zi_chunk_segment* out,
                         int64_t cap, int64_t* n_segments_out, int64_t* n_slot_uses_out);

/*
 * Launch plan of zi_adamw_step, as a pure host function (no GPU needed; nothing is dereferenced, only
 * the addresses and lengths of t[] are used).  One item per non-empty tensor: the number of leading
 * elements handled one by one before the 4-element lane vectors start (0..63, chosen so that as much
 * of the tensor's traffic as possible starts on 128-byte lines), its tiles of 512 elements, and the
 * launch it belongs to.  Tensors of 2^22 elements or more get a launch of their own (`alone`);
 * shorter ones share launches of up to 32 tensors.  Writes at most `cap` items and always the totals.
 */
typedef struct {
    int32_t tensor;        /* index into t[] */
    int32_t head;          /* leading elements handled one by one */
    int64_t n_tiles;
    int64_t first_tile;    /* first workgroup of this tensor within its launch */
    int32_t launch;        /* 0-based, in issue order */
    int32_t alone;         /* 1 if the launch holds this tensor only */
} zi_step_plan_item;

zi_status zi_plan_step(const zi_tensor* t, int32_t n_tensors, zi_step_plan_item* out, int64_t cap,
                       int64_t* n_items_out, int64_t* n_launches_out);

/*
 * The step on the host CPUs, for state, gradients and copy that all live in HOST memory (any host
 * memory).  This is the paper's own placement of the offloaded step (Section 5.2.2: with optimizer
 * states in CPU memory the step uses the CPUs' aggregate compute and memory bandwidth; only 2 bytes
 * of gradient per element come down the link and 2 bytes of low-precision parameter go up).  These
 * two calls are chosen explicitly by the caller: no GPU entry point ever falls back to them, and
 * they touch no GPU.  Same arithmetic in the same order as the GPU kernels (AVX2 / FMA / F16C
 * vector code, n_threads threads, blocks of 2^18 elements); ZI_ERR_UNSUPPORTED on a CPU without
 * those instructions.  Blocking.
 * zi_host_grad_norm: as zi_grad_norm, result written to HOST memory h_out; block partials are
 * added in block order, so the result does not depend on n_threads.
 * zi_host_adamw_step: as zi_adamw_step; h_norm is a HOST result or NULL; returns
 * ZI_SKIPPED_OVERFLOW (nothing touched) if h_norm->found_inf is set.
 */
zi_status zi_host_grad_norm(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, float loss_scale,
                            zi_norm_result* h_out, int32_t n_threads);
zi_status zi_host_adamw_step(const zi_tensor* t, int32_t n_tensors, zi_lp_dtype dt, const zi_adamw_config* cfg,
                             const zi_norm_result* h_norm, int32_t n_threads);

/* Pinned (page-locked, device-visible) host memory.  zi_pinned_free(NULL) is accepted. */
zi_status zi_pinned_alloc(void** out, size_t bytes);
zi_status zi_pinned_free(void* ptr);

#ifdef __cplusplus
}
#endif
#endif /* ZI_H */

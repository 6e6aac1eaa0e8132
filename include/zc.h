/*
 * zc — one rank's sharded mixed-precision optimizer step on MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only.  Every pointer is marked HOST or
 * DEVICE below.  The caller owns every data buffer; the library owns only what
 * a *_create call returns and the small reduction workspaces (64 KiB per device
 * and stream) it allocates on first use of zc_grad_sqnorm.
 *
 * Stream semantics: every call that takes `hip_stream` (a hipStream_t passed
 * as void*, NULL = the null stream) only enqueues work on it and returns; no
 * call synchronises the device.  zc_offload_adam_step uses two extra internal
 * copy streams that are fenced against `hip_stream` at entry and exit, so the
 * caller sees ordinary in-order stream behaviour.
 *
 * Errors: every call returns a zc_status.  Argument errors are detected before
 * anything is launched and leave all memory untouched.  zc_last_error() gives
 * a thread-local text for the most recent failure on the calling thread.
 *
 * Context in the paper (arXiv 2504.09983): the passes it describes schedule
 * all-gathers, releases and optimizer-state transfers *around* this path; the
 * path itself is "parameter updates" on the GPU (Evaluation: Efficiency;
 * Adaptive Offloading) over fp32 master parameters and Adam states with bf16
 * compute copies (Experimental settings), evenly partitioned across ranks
 * (Optimizations: Fully-sharded approach).
 */
#ifndef ZC_H
#define ZC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZC_OK = 0,
    ZC_ERR_INVALID_ARG = 1, /* NULL where required, negative size, bad hyper-parameter */
    ZC_ERR_ALIGNMENT = 2,   /* pointer not aligned to its element type */
    ZC_ERR_HIP = 3,         /* a HIP runtime call failed; text has the HIP error */
    ZC_ERR_UNSUPPORTED = 4, /* valid request this build cannot serve */
    ZC_ERR_NOMEM = 5        /* host or device allocation failed */
} zc_status;

typedef enum { ZC_F32 = 0, ZC_BF16 = 1 } zc_dtype;
typedef enum { ZC_ADAMW = 0, ZC_ADAM_L2 = 1 } zc_mode;

/*
 * Hyper-parameters of one step.  `step` is 1-based and supplied by the caller
 * (the library keeps no counter).  `grad_scale` multiplies every gradient
 * before use (1.0f = none; used for loss-scale removal and clipping).
 * Constraints: lr finite, 0 <= beta1 < 1, 0 <= beta2 < 1, eps >= 0,
 * weight_decay finite, grad_scale finite, step >= 1, mode in zc_mode.
 */
typedef struct {
    float lr;
    float beta1;
    float beta2;
    float eps;
    float weight_decay;
    float grad_scale;
    int64_t step;
    int32_t mode;
    int32_t reserved; /* must be 0 */
} zc_adam_hparams;

/* One contiguous piece of the gathered buffer and where it goes. */
typedef struct {
    int64_t src_offset; /* bf16 elements from the start of the gathered buffer */
    void *dst;          /* DEVICE, 2-byte aligned, room for numel bf16 values */
    int64_t numel;      /* bf16 elements, >= 0 */
} zc_segment;

typedef struct zc_unshard_plan zc_unshard_plan;
typedef struct zc_offload_ctx zc_offload_ctx;

/* Library version, major*10000 + minor*100 + patch. */
int zc_version(void);

/* Text of the last failure on this thread ("" if none).  Static storage. */
const char *zc_last_error(void);

/*
 * Fused Adam / AdamW update over a flat fp32 partition, in place (paper:
 * "parameter updates" kept on the GPU, Evaluation: Adaptive Offloading; fp32
 * parameters, gradients and Adam states, Experimental settings).
 *
 * Per element i, with t = hp->step, bc1 = 1-beta1^t, bc2 = 1-beta2^t:
 *   g  = upcast(g[i]) * grad_scale            (ZC_ADAM_L2: g += wd * p[i])
 *   m[i] = beta1*m[i] + (1-beta1)*g
 *   v[i] = beta2*v[i] + (1-beta2)*g*g
 *   p[i] = p[i]*(1 - lr*wd) [ZC_ADAMW only] - (lr/bc1) * m[i] / (sqrt(v[i]/bc2) + eps)
 *   bf16_out[i] = round-to-nearest-even bf16 of the stored p[i]   (if not NULL)
 *
 * p, m, v      DEVICE fp32[n], 4-byte aligned, updated in place.
 * g            DEVICE, fp32[n] (ZC_F32, 4-byte aligned) or bf16[n] bit
 *              patterns (ZC_BF16, 2-byte aligned); read only.
 * bf16_out     DEVICE uint16[n] or NULL.  No two of p, m, v, g, bf16_out may
 *              share a byte (checked; ZC_ERR_INVALID_ARG).
 * skip_flag    DEVICE int32 or NULL; when *skip_flag != 0 at execution time
 *              the step leaves every buffer untouched (overflowed step).
 * n            elements, >= 0 (0 is a no-op); any size up to 2^40.
 * Vector (128-bit) access is used when p, m, v are 16-byte aligned and g,
 * bf16_out are aligned to 4 elements, also when all of them reach that alignment
 * after the same 1-3 leading elements (a range cut out of a larger partition);
 * otherwise a slower one-element-per-lane kernel runs.
 * Placement: for partitions of a few GB the rate depends on how far apart p, m
 * and v lie in device memory (measured on MI355X over 4 GB arrays: 0.78 of the
 * HBM peak back to back, 0.82 at 32 GiB or more, 0.85 at 16 or 20 GiB between
 * neighbours); a caller that carves them out of one arena does well to put other
 * long-lived buffers between them.  Arrays of tens of GB are affected less (0.81-0.82
 * in most runs, 0.78 seen once).  zc_adam_step_packed below has no such dependence.
 * Returns ZC_ERR_INVALID_ARG / ZC_ERR_ALIGNMENT before launching anything.
 */
zc_status zc_adam_step(float *p, float *m, float *v, const void *g, zc_dtype g_dtype,
                       int64_t n, const zc_adam_hparams *hp, uint16_t *bf16_out,
                       const int32_t *skip_flag, void *hip_stream);

/*
 * The same step with per-range hyper-parameters and a device-side gradient scale
 * (weight decay is usually switched off for norm vectors and biases; the clipping
 * coefficient and the loss scale are known on the GPU before they are on the host).
 *   ranges[r]      HOST, sorted by begin, non-overlapping, inside [0, n): elements
 *                  [begin, end) use lr = hp->lr * lr_scale (one fp32 product) and
 *                  the range's weight_decay; elements outside every range use *hp
 *   grad_scale_dev DEVICE float or NULL: gradients are multiplied by
 *                  fl32(hp->grad_scale * *grad_scale_dev), read at execution time
 * Everything else as zc_adam_step.  Each stretch is one launch; the result is
 * bit-identical to calling zc_adam_step on the stretches one by one.
 */
typedef struct {
    int64_t begin;
    int64_t end;
    float lr_scale;
    float weight_decay;
} zc_param_range;
zc_status zc_adam_step_groups(float *p, float *m, float *v, const void *g, zc_dtype g_dtype,
                              int64_t n, const zc_adam_hparams *hp, const zc_param_range *ranges,
                              int64_t nranges, uint16_t *bf16_out, const int32_t *skip_flag,
                              const float *grad_scale_dev, void *hip_stream);

/*
 * Packed optimizer state (not in the paper, which says nothing about how a rank
 * lays out its fp32 master parameters and Adam buffers; Experimental settings
 * only fixes that they are fp32 and per rank).  p, m and v are private to the
 * optimizer, so the library may choose their layout: one array in which granules
 * of ZC_PACKED_GRANULE elements of p, m and v follow each other,
 *   [p 0..G) [m 0..G) [v 0..G) [p G..2G) [m G..2G) [v G..2G) ...
 * i.e. p[e] = state[e + 2*G*(e / G)], m[e] one granule and v[e] two granules behind
 * it.  The update then reads and writes ONE contiguous stream of state instead of
 * three that lie gigabytes apart, which measured 2-4 % faster on MI355X (0.83-0.85
 * of the HBM peak instead of 0.80-0.82) and does not depend on where an allocator
 * happened to put three separate arrays.  The arithmetic, the bf16 copy, the skip
 * flag, the ranges and the device-side scale are those of zc_adam_step_groups,
 * and the results are bit-identical to it element by element.
 *
 * zc_packed_state_numel(n): floats the packed array of an n-element partition
 *   holds (3 * ceil(n / G) * G; 0 for n <= 0).
 * zc_state_pack: state <- p, m, v (DEVICE fp32[n], 4-byte aligned; a NULL source
 *   stands for zeros); the padding behind element n of the last granule is zeroed.
 * zc_state_unpack: p, m, v <- state; NULL destinations are skipped.
 * zc_adam_step_packed: one step over the whole partition.
 *   state  DEVICE fp32[zc_packed_state_numel(n)], 128-byte aligned, updated in
 *          place; the padding is never read or written.
 *   g, bf16_out, hp, ranges, skip_flag, grad_scale_dev, n: as zc_adam_step_groups
 *          (flat arrays indexed by element; ranges may be NULL with nranges 0).
 * 128-bit accesses are used for every stretch whose g and bf16_out reach 16- and
 * 8-byte alignment at an element index that is a multiple of 4; other stretches and
 * the non-default "adam.arith" variants run one element per lane.
 * state must not overlap g, bf16_out, p, m or v (checked; ZC_ERR_INVALID_ARG).
 * All calls are asynchronous on hip_stream and allocate nothing.
 */
#define ZC_PACKED_GRANULE 8192
int64_t zc_packed_state_numel(int64_t n);
zc_status zc_state_pack(const float *p, const float *m, const float *v, int64_t n, float *state,
                        void *hip_stream);
zc_status zc_state_unpack(const float *state, int64_t n, float *p, float *m, float *v,
                          void *hip_stream);
zc_status zc_adam_step_packed(float *state, const void *g, zc_dtype g_dtype, int64_t n,
                              const zc_adam_hparams *hp, const zc_param_range *ranges,
                              int64_t nranges, uint16_t *bf16_out, const int32_t *skip_flag,
                              const float *grad_scale_dev, void *hip_stream);

/*
 * Gradient-clipping coefficient and loss-scale removal on the GPU, from the
 * squared norm that zc_grad_sqnorm wrote (of the still loss-scaled gradients):
 *   norm = sqrt(*sqnorm) * inv_loss_scale
 *   *scale_out = fl32(inv_loss_scale * min(1, max_norm / (norm + 1e-6)))   (max_norm = 0: no clipping)
 * sqnorm, scale_out DEVICE float.  The result is what zc_adam_step_groups takes
 * as grad_scale_dev, so norm -> coefficient -> step needs no host round trip.
 */
zc_status zc_clip_scale(const float *sqnorm, float max_norm, float inv_loss_scale,
                        float *scale_out, void *hip_stream);

/*
 * Standalone fp32 -> bf16 copy into the all-gather send buffer (paper: bf16
 * compute copies of fp32 masters, Experimental settings; the shards are what
 * the all-gather sends, Fully-sharded approach).  Round-to-nearest-even; NaN
 * stays NaN with the quiet bit set; no flush of subnormals.  Bit-identical to
 * the bf16_out of zc_adam_step for the same fp32 input.
 * src DEVICE fp32[n]; dst DEVICE uint16[n]; must not overlap.
 */
zc_status zc_cast_bf16(const float *src, uint16_t *dst, int64_t n, void *hip_stream);

/*
 * Host-only helper: flat even partition of `ntensors` tensors over `world`
 * ranks (paper: each parameter evenly partitioned across all GPUs,
 * Fully-sharded approach; here applied to the flattened concatenation).
 * offsets_out[t] = sum of numels[0..t); *total_out = T = sum of all numels;
 * *shard_numel_out = ceil(ceil(T/world)/shard_align)*shard_align.  The
 * gathered buffer has world * shard_numel elements; elements >= T are padding.
 * All pointers HOST.  Touches no GPU.
 */
zc_status zc_flat_layout(const int64_t *numels, int64_t ntensors, int32_t world,
                         int64_t shard_align, int64_t *offsets_out,
                         int64_t *shard_numel_out, int64_t *total_out);

/*
 * Host-only helper: per-tensor even partition, the layout the paper states
 * literally (every parameter tensor evenly partitioned across all GPUs,
 * Fully-sharded approach) with the all-gathers of a group of tensors fused into
 * one buffer (Proactive prefetching, Fuse).  Tensor t is cut into `world` slices
 * of s_t = ceil(ceil(n_t/world)/align)*align elements, the part beyond n_t being
 * padding; a rank's send buffer is its slices of all tensors back to back
 * (*send_numel_out = sum of s_t elements); the gathered buffer is the `world`
 * send buffers in rank order.  For segment k = t*world + r the tables receive
 *   src_offsets_out[k] = r * send_numel + (sum of s_t' for t' < t)
 *   dst_offsets_out[k] = r * s_t        (element offset inside tensor t)
 *   seg_numels_out[k]  = real elements rank r holds of tensor t (0 = padding only)
 * which, with dst = tensor base + dst offset, is a zc_segment table for
 * zc_unshard_plan_create.  All pointers HOST, tables of ntensors*world entries.
 */
zc_status zc_per_tensor_layout(const int64_t *numels, int64_t ntensors, int32_t world,
                               int64_t align, int64_t *src_offsets_out, int64_t *dst_offsets_out,
                               int64_t *seg_numels_out, int64_t *send_numel_out);

/*
 * Unshard: copy pieces of the gathered flat bf16 buffer (what the all-gather
 * produced: the large buffer B_ag of Proactive prefetching / Selective
 * unsharding) into separately allocated per-layer tensors.  Bit copy.
 *
 * zc_unshard_plan_create validates the HOST segment table (offsets and sizes
 * inside [0, gathered_numel], non-NULL 2-byte-aligned dst for non-empty
 * segments), and uploads a descriptor table to the current device.
 * Destination ranges must not overlap each other (checked at creation) or the
 * gathered buffer (checked at every zc_unshard); ZC_ERR_INVALID_ARG otherwise.
 * The plan stays valid until destroyed; dst pointers are captured.
 * zc_unshard enqueues one kernel; `gathered` is DEVICE uint16[gathered_numel],
 * 2-byte aligned.  An empty plan (nsegs == 0 or all numel == 0) is a no-op.
 */
zc_status zc_unshard_plan_create(const zc_segment *segs, int64_t nsegs,
                                 int64_t gathered_numel, zc_unshard_plan **out);
zc_status zc_unshard(const zc_unshard_plan *plan, const uint16_t *gathered, void *hip_stream);
zc_status zc_unshard_plan_destroy(zc_unshard_plan *plan);

/*
 * Offloaded step (paper: Adaptive offloading moves optimizer-state fragments
 * to host memory and overlaps the copies with computation while the update
 * itself stays on the GPU).  Elements [0, n_resident) of the partition live
 * in DEVICE arrays p_dev/m_dev/v_dev; elements [n_resident, n_resident +
 * n_streamed) live in pinned HOST arrays p_host/m_host/v_host and cross the
 * host link once in each direction.  Three transports, chosen by the knob
 * "offload.zero_copy" (results are bit-identical to zc_adam_step over the
 * concatenation either way):
 *   1 (default)  the update kernel reads and writes the pinned host arrays
 *                directly through the link; one launch on `hip_stream`, no
 *                staging memory, no copy engines.  A resident prefix is updated
 *                by a second launch on an internal stream that forks from and
 *                rejoins `hip_stream` inside the call.
 *   0            staged ring: host -> staging slot -> kernel -> host in chunks
 *                of chunk_bytes per array through num_buffers slots, copies on
 *                two internal streams (hipMemcpyAsync) and the kernel on
 *                `hip_stream`, fenced by events.  With "offload.max_ahead" = 1
 *                (default) this transport blocks the calling thread while it
 *                feeds the ring; the results are still ordered on `hip_stream`.
 *   2            staged reads, direct writes: chunks are copied host -> staging
 *                slot on one internal stream, the kernel reads the slot and
 *                stores the new state straight into the host arrays.  Same
 *                host-blocking rule as 0.  Measured slower than 1.
 *
 * zc_offload_create   chunk_bytes: bytes per fp32 array per chunk, a positive
 *                     multiple of 4096 (64 MiB in the reference workload);
 *                     num_buffers in [1, 8].  Creates two streams and the events.
 *                     The staging ring of 3*num_buffers*chunk_bytes of device
 *                     memory is allocated by the first call that stages (transports
 *                     0 and 2, zc_offload_probe_link; ZC_ERR_NOMEM if it does not
 *                     fit) and never by the default transport.
 * zc_offload_adam_step
 *   p_dev,m_dev,v_dev DEVICE fp32[n_resident] (may be NULL when n_resident==0)
 *   p_host,...        HOST fp32[n_streamed], allocated with hipHostMalloc (or
 *                     torch pin_memory); checked, unpinned -> INVALID_ARG.
 *   g_dev             DEVICE, n_resident + n_streamed elements of g_dtype.
 *   bf16_out_dev      DEVICE uint16[n_resident + n_streamed] or NULL.
 *   A context serves one step at a time; concurrent calls on one context race.
 *   The host arrays must not be touched by the host until `hip_stream` has
 *   passed the call.
 */
zc_status zc_offload_create(int64_t chunk_bytes, int32_t num_buffers, zc_offload_ctx **out);
zc_status zc_offload_adam_step(zc_offload_ctx *ctx, float *p_dev, float *m_dev, float *v_dev,
                               int64_t n_resident, float *p_host, float *m_host,
                               float *v_host, int64_t n_streamed, const void *g_dev,
                               zc_dtype g_dtype, const zc_adam_hparams *hp,
                               uint16_t *bf16_out_dev, const int32_t *skip_flag,
                               void *hip_stream);
zc_status zc_offload_destroy(zc_offload_ctx *ctx);

/*
 * Adaptive offloading of optimizer-state fragments (paper: Adaptive offloading,
 * Algorithm 2, and the reload rule of the paragraph after it), as a host-only
 * planner over a profiled schedule.
 *   p_mem[i]      profiled memory in use before operator i, optimizer states not
 *                 counted; operators [0, n_forward) are the forward pass, the
 *                 rest the backward pass
 *   frag_bytes[f] size of optimizer-state fragment f; their sum is M_opt
 *   mem_limit     M
 * Copies out are started at the very beginning for the shortest prefix of
 * fragments that lets the largest p_mem fit; a fragment is waited for and freed
 * (ZC_OP_SYNC_FREE) right before the first operator that needs its room; in the
 * backward pass a copy back (ZC_OP_RELOAD) starts as soon as the largest p_mem
 * from that operator to the end leaves room for it; every reload is waited for
 * (ZC_OP_SYNC_RELOAD) at the end.  Fragments leave and return in list order.
 * out receives at most `capacity` entries, *out_len the length of the schedule
 * (n_ops + 4*nfrags always suffices).  ZC_ERR_UNSUPPORTED when an operator does
 * not fit even with every fragment offloaded.  All pointers HOST.
 */
typedef enum {
    ZC_OP_COMPUTE = 0,    /* index = operator */
    ZC_OP_OFFLOAD = 1,    /* index = fragment: start the asynchronous copy to the host */
    ZC_OP_SYNC_FREE = 2,  /* wait for that copy, then the device memory may be reused */
    ZC_OP_RELOAD = 3,     /* start the asynchronous copy back */
    ZC_OP_SYNC_RELOAD = 4 /* wait for the copy back */
} zc_op_kind;
typedef struct {
    int32_t kind;
    int32_t index;
} zc_sched_op;
zc_status zc_plan_adaptive_offload(const int64_t *p_mem, int64_t n_ops, int64_t n_forward,
                                   const int64_t *frag_bytes, int64_t nfrags, int64_t mem_limit,
                                   zc_sched_op *out, int64_t capacity, int64_t *out_len);

/*
 * Proactive prefetching (paper: Proactive prefetching, Algorithm 1) with Fuse, as a
 * host-only planner.  The schedule o_0..o_{n-1} is walked from the back; an
 * all-gather keeps moving towards the front together with the other unscheduled
 * ones while the profiled memory before its predecessor plus their buffers stays
 * below mem_limit and their total stays below prefetch_limit; when that fails the
 * group is placed and the all-gather opens the next group if it fits alone, else
 * it stays where it is.  A placed group is fused pairwise in schedule order while
 * T_c(V1) + T_c(V2) > alpha * T_c(V1 + V2), T_c being the profiled table
 * (tc_sizes increasing, tc_times; linear between samples, flat below the first,
 * last slope beyond the last).
 *   is_allgather[i], bag_bytes[i] (B_ag, > 0 for all-gathers), p_mem[i] (P_mem)
 *   order_out[k]   operator at position k of the new schedule
 *   group_out[k]   -1 for other operators; all-gathers with equal ids are fused
 * All pointers HOST, tables of n_ops entries.
 */
zc_status zc_plan_prefetch(const int32_t *is_allgather, const int64_t *bag_bytes,
                           const int64_t *p_mem, int64_t n_ops, int64_t mem_limit,
                           int64_t prefetch_limit, const int64_t *tc_sizes,
                           const double *tc_times, int64_t n_tc, double alpha,
                           int32_t *order_out, int32_t *group_out);

/*
 * Selective unsharding (paper: Selective unsharding): which gathered parameters to
 * keep unsharded until the update, within `budget` bytes of memory left after
 * prefetching.  Parameters are taken in order of communication time saved per byte,
 * T_c(B_ag)/B_ag, highest first (smaller buffers first among equals), each one that
 * still fits.  chosen_out receives the indices in the order chosen (room for n),
 * *n_chosen_out their count.  All pointers HOST.
 */
zc_status zc_select_unsharded(const int64_t *bag_bytes, int64_t n, const int64_t *tc_sizes,
                              const double *tc_times, int64_t n_tc, int64_t budget,
                              int32_t *chosen_out, int64_t *n_chosen_out);

/*
 * Replay a schedule on HIP streams: operator i becomes a stand-in kernel that
 * occupies `hip_stream` for op_ms[i] milliseconds (NULL = no kernels), copies run
 * on the context's two copy streams, the wait operators become cross-stream event
 * waits.  With poison_freed != 0 a freed fragment's device memory is overwritten,
 * so a later use without reload shows.  The schedule is validated first
 * (operators in order, each fragment offload -> free -> reload -> wait, all
 * fragments back at the end).  frags[f].dev DEVICE, frags[f].host pinned HOST,
 * bytes a multiple of 4.  Enqueues and returns.
 */
typedef struct {
    void *dev;
    void *host;
    int64_t bytes;
} zc_fragment;
zc_status zc_schedule_run(zc_offload_ctx *ctx, const zc_sched_op *ops, int64_t nops,
                          const float *op_ms, int64_t n_ops, const zc_fragment *frags,
                          int64_t nfrags, int32_t poison_freed, void *hip_stream);

/*
 * Pinned host memory of exactly `bytes` bytes for the offloaded partitions
 * (hipHostMalloc; page-locked, device-accessible, 4 KiB aligned).  A convenience
 * for callers whose allocator rounds pinned requests up (a 35 GB array then
 * costs 64 GB).  *out (HOST) is owned by the caller and released with
 * zc_host_free; NULL is a no-op there.  Failure -> ZC_ERR_NOMEM, *out = NULL.
 */
zc_status zc_host_alloc(int64_t bytes, void **out);
zc_status zc_host_free(void *ptr);

/*
 * Measurement helper: the practical host-link ceiling next to which the offloaded
 * step is reported.  Copies `bytes` from pinned HOST memory into the context's
 * staging ring (mode 0), from the ring to pinned HOST memory (mode 1), or both at
 * once on the context's two copy streams (mode 2), in chunk_bytes pieces, and
 * returns the wall time in *ms_out (HOST).  Blocks until the copies are done.
 * The data copied is meaningless; host_src is only read, host_dst only written.
 */
zc_status zc_offload_probe_link(zc_offload_ctx *ctx, const void *host_src, void *host_dst,
                                int64_t bytes, int32_t mode, float *ms_out);

/*
 * Gradient accumulation into the fp32 gradient partition (paper: fp32 gradients
 * are kept, Experimental settings; with gradient accumulation several forward/
 * backward passes add into them before one update, Selective unsharding):
 *   acc[i] = acc[i] + upcast(micro[i]) * scale      (one rounding to fp32)
 * acc DEVICE fp32[n], updated in place; micro DEVICE fp32[n] or bf16[n], read
 * only, must not alias acc; scale finite (1/accumulation-steps, loss-scale
 * removal).  The accumulated fp32 partition is then the g of zc_grad_sqnorm and
 * zc_adam_step (ZC_F32).  n == 0 is a no-op.
 */
zc_status zc_grad_accumulate(float *acc, const void *micro, zc_dtype micro_dtype, int64_t n,
                             float scale, void *hip_stream);

/*
 * Squared L2 norm of the gradient partition and a non-finite flag (the
 * overflow check and clipping input that precede a mixed-precision step; not
 * in the paper, which only states that fp32 gradients are kept).
 * g DEVICE fp32[n] or bf16[n]; sqnorm_out DEVICE float; found_inf_out DEVICE
 * int32, set to 1 when any element is NaN/Inf else 0.  Deterministic for a
 * given n (fixed reduction tree); fp32 arithmetic only within groups of at most
 * 8 squares, double from there on, so *sqnorm_out lies within one fp32 ulp of the
 * exactly rounded sum.  n == 0 writes 0 and 0.
 * The per-workgroup partial sums live in a 64 KiB device workspace that the
 * library allocates on the first call on a (device, stream) pair and keeps, so
 * calls on different streams do not interfere.  That first call must happen
 * outside a graph capture (inside one it returns ZC_ERR_UNSUPPORTED and enqueues
 * nothing).
 */
zc_status zc_grad_sqnorm(const void *g, zc_dtype g_dtype, int64_t n, float *sqnorm_out,
                         int32_t *found_inf_out, void *hip_stream);

/*
 * zc_grad_sqnorm for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels, same result bit for bit; the per-workgroup partial sums go to a fixed
 * 64 KiB array (4096 entries of 16 bytes) inside the library's device image
 * instead of an allocated workspace, so this call never allocates or frees
 * memory.  The grid is capped at 4096 workgroups, which serves every n up to the
 * library's limit of 2^40 elements; a larger n is refused with
 * ZC_ERR_UNSUPPORTED before anything is enqueued.  Each GPU holds one copy of
 * the array for the life of the process; its address is looked up once per
 * device on the first call made with that device current.  The array needs no
 * clearing (every entry read was written by the same call), but all calls on a
 * GPU share it whatever their stream: two calls whose kernels can overlap on one
 * GPU race and give garbage; order them on one stream or with events.
 */
zc_status zc_grad_sqnorm_static(const void *g, zc_dtype g_dtype, int64_t n, float *sqnorm_out,
                                int32_t *found_inf_out, void *hip_stream);

/*
 * Tuning knobs for measurement sweeps.  The knobs belong to the calling thread:
 * zc_tune_set changes what later calls made by the same thread launch, and no
 * other thread's; a thread that never calls it launches the defaults, whatever
 * other threads have set.  Unknown key -> ZC_ERR_INVALID_ARG.  Keys:
 *   "adam.rows"        128-bit vectors per lane per tile: 1 (default), 2 or 4
 *   "adam.block"       threads per workgroup: 64 (default), 128 or 256
 *   "adam.waves_per_cu" cap on resident waves per compute unit, enforced through an
 *                      unused dynamic-LDS request; 0 = no cap; -1 (default) = 13 with
 *                      bf16 gradients, 12 with fp32 gradients
 *   "adam.nontemporal" 0 = ordinary loads and stores, 1 = both non-temporal, 2 = loads only,
 *                      3 = stores only, 4 (default) = non-temporal loads and write-through
 *                      streaming stores (buffer stores with the nt and sc1 bits)
 *   "adam.arith"       0 = fp32 only, 1 = fp64 multiply-adds with fp32 sqrt/div,
 *                      2 = fp64 throughout
 *   "copy.waves_per_cu", "cast.waves_per_cu", "accum.waves_per_cu"  the same cap for
 *                      unshard (16), the cast (20) and gradient accumulation (24)
 *   "reduce.unroll"    128-bit loads in flight per lane in zc_grad_sqnorm: 2, 4 or 8 (default)
 *   "reduce.blocks_per_cu" persistent 256-thread workgroups per compute unit in
 *                      zc_grad_sqnorm: 1-16, default 2
 *   "copy.nontemporal"  cast, unshard, accumulation: 0 = ordinary accesses, 1 = non-temporal,
 *                      2 (default) = non-temporal loads and write-through streaming stores
 *   "launch.max_grid"  workgroups per launch (default 2^30, and never more than fit into
 *                      2^32 - 1 threads); larger jobs are cut into several launches
 *   "offload.zero_copy" 0 = staged ring, 1 = kernel reads/writes pinned host (default),
 *                      2 = staged reads + kernel writes pinned host
 *   "offload.zc_waves_per_cu"  resident-wave cap of the zero-copy kernel (0 = none)
 *   "offload.zc_block", "offload.zc_rows"  its threads per workgroup (256) and rows (2)
 *   "offload.max_ahead" 1 (default) = the staged ring blocks the host so that it never runs
 *                      more than num_buffers chunks ahead of finished copy-backs (deep copy
 *                      queues were measured to halve the link rate); 0 = enqueue everything
 *   "offload.d2h_on_compute" 1 = the staged ring copies back on `hip_stream`
 *   "offload.overlap_resident" 1 (default) = in the zero-copy transport the resident prefix runs on
 *                      an internal stream beside the link-bound launch, joined before the call returns
 *   "offload.poison"   1 = every ring slot is overwritten with 0xDEADBEEF once its chunk has
 *                      left it (a test aid: a missing fence then shows up as garbage)
 */
zc_status zc_tune_set(const char *key, int64_t value);
zc_status zc_tune_get(const char *key, int64_t *value_out);

#ifdef __cplusplus
}
#endif
#endif /* ZC_H */

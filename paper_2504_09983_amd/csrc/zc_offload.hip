// Offloaded optimizer step: fp32 p/m/v of the streamed suffix live in pinned
// host memory and cross the host link once in each direction per step.
//
// Paper context (Adaptive offloading): optimizer-state fragments are copied
// asynchronously so that transfers overlap with computation, memory is only
// reused after the copy has completed, and the update itself runs on the GPU.
//
// Three transports are built.
//
// Zero-copy (default): the fused update kernel is pointed at the pinned host
// arrays.  Its 128-bit loads become link reads, its stores link writes, both
// directions are busy at once, and nothing is staged in HBM.
//
// Staged ring: fixed-size chunks pass through a ring of device slots, driven by
// three HIP streams at default priority:
//
//   h2d stream : wait(slot free) -> 3 x hipMemcpyAsync host->slot -> record(loaded)
//   caller's   : wait(loaded)    -> fused update kernel on slot   -> record(updated)
//   d2h stream : wait(updated)   -> 3 x hipMemcpyAsync slot->host -> record(slot free)
//
// Staged reads, direct writes: the h2d stream of the ring feeds the slots, the update
// kernel reads a slot and stores the new state straight into the host arrays (no
// copy-back stream).  Measured 43 GB/s each way against 46 for zero-copy: kept as a
// measured alternative, not the default.
//
// Measured on MI355X the ring reaches the plain-memcpy ceiling of the link when
// the caller synchronises between steps.  The runtime executes the copy-backs as
// copy kernels of its own, and with several steps queued those now and then
// (about one process in five) run at ~10 GB/s, halving the step rate; the
// zero-copy kernel holds ~95 % of the ceiling every time, which is why it is the
// default.
#include <chrono>
#include <new>
#include <vector>

#include "zc_internal.h"

struct zc_offload_ctx {
    int64_t chunk_bytes = 0;
    int64_t chunk_elems = 0;
    int num_buffers = 0;
    int device = 0;
    float *staging = nullptr;  // num_buffers * 3 * chunk_elems floats; allocated by the first call that stages
    hipStream_t h2d = nullptr, d2h = nullptr;
    hipEvent_t entry = nullptr, done = nullptr;
    hipEvent_t loaded[8] = {}, updated[8] = {}, freed[8] = {};
    std::vector<hipEvent_t> pool;  // extra events for schedule replay, grown on demand
};

namespace zc {

static void destroy_ctx(zc_offload_ctx *c)
{
    if (!c)
        return;
    if (c->h2d) {
        (void)hipStreamSynchronize(c->h2d);
        (void)hipStreamDestroy(c->h2d);
    }
    if (c->d2h) {
        (void)hipStreamSynchronize(c->d2h);
        (void)hipStreamDestroy(c->d2h);
    }
    for (int i = 0; i < 8; ++i) {
        if (c->loaded[i]) (void)hipEventDestroy(c->loaded[i]);
        if (c->updated[i]) (void)hipEventDestroy(c->updated[i]);
        if (c->freed[i]) (void)hipEventDestroy(c->freed[i]);
    }
    for (hipEvent_t e : c->pool)
        (void)hipEventDestroy(e);
    if (c->entry) (void)hipEventDestroy(c->entry);
    if (c->done) (void)hipEventDestroy(c->done);
    if (c->staging) (void)hipFree(c->staging);
    delete c;
}

// Accessors for the schedule executor, which lives in another translation unit.
hipStream_t offload_h2d_stream(zc_offload_ctx *ctx) { return ctx->h2d; }
hipStream_t offload_d2h_stream(zc_offload_ctx *ctx) { return ctx->d2h; }
int offload_device(zc_offload_ctx *ctx) { return ctx->device; }

zc_status offload_events(zc_offload_ctx *ctx, int64_t count, hipEvent_t **out)
{
    try {
        while ((int64_t)ctx->pool.size() < count) {
            hipEvent_t e = nullptr;
            ZC_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            ctx->pool.push_back(e);
        }
    } catch (const std::bad_alloc &) {
        return fail(ZC_ERR_NOMEM, "cannot grow the event pool");
    }
    *out = ctx->pool.data();
    return ZC_OK;
}

// The staging ring is only needed by the two staged transports and the link probe; the
// default zero-copy transport never touches it, so it is allocated by the first call that
// stages (not capturable: that call allocates) and kept until the context is destroyed.
static zc_status require_staging(zc_offload_ctx *ctx)
{
    if (ctx->staging)
        return ZC_OK;
    const size_t bytes = (size_t)ctx->chunk_bytes * 3 * (size_t)ctx->num_buffers;
    const hipError_t e = hipMalloc(reinterpret_cast<void **>(&ctx->staging), bytes);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        ctx->staging = nullptr;
        return fail(ZC_ERR_NOMEM, "staging ring of %zu bytes does not fit", bytes);
    }
    if (e != hipSuccess)
        return hip_fail(e, "hipMalloc(staging ring)");
    return ZC_OK;
}

// Pinned host memory is reported as hipMemoryTypeHost; pageable memory either
// fails the query or is reported as unregistered.
static zc_status require_pinned(const void *ptr, const char *name)
{
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // clear the sticky error of the failed query
        return fail(ZC_ERR_INVALID_ARG, "%s is not pinned host memory (hipHostMalloc it)", name);
    }
    if (attr.type != hipMemoryTypeHost)
        return fail(ZC_ERR_INVALID_ARG, "%s is not pinned host memory (memory type %d)", name,
                    (int)attr.type);
    return ZC_OK;
}

}  // namespace zc

extern "C" {

zc_status zc_offload_create(int64_t chunk_bytes, int32_t num_buffers, zc_offload_ctx **out)
{
    using namespace zc;
    if (!out)
        return fail(ZC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (chunk_bytes <= 0 || chunk_bytes % 4096 != 0)
        return fail(ZC_ERR_INVALID_ARG, "chunk_bytes must be a positive multiple of 4096");
    if (chunk_bytes > (int64_t(1) << 32))
        return fail(ZC_ERR_UNSUPPORTED, "chunk_bytes above 4 GiB");
    if (num_buffers < 1 || num_buffers > 8)
        return fail(ZC_ERR_INVALID_ARG, "num_buffers must be in [1, 8]");
    zc_offload_ctx *c = new (std::nothrow) zc_offload_ctx;
    if (!c)
        return fail(ZC_ERR_NOMEM, "cannot allocate the context");
    c->chunk_bytes = chunk_bytes;
    c->chunk_elems = chunk_bytes / 4;
    c->num_buffers = num_buffers;
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->h2d, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->d2h, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->entry, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->done, hipEventDisableTiming);
    for (int i = 0; i < num_buffers && e == hipSuccess; ++i) {
        e = hipEventCreateWithFlags(&c->loaded[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->updated[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->freed[i], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        const zc_status st = hip_fail(e, "creating the offload context");
        destroy_ctx(c);
        return st;
    }
    *out = c;
    return ZC_OK;
}

zc_status zc_offload_destroy(zc_offload_ctx *ctx)
{
    zc::destroy_ctx(ctx);
    return ZC_OK;
}

zc_status zc_host_alloc(int64_t bytes, void **out)
{
    using namespace zc;
    if (!out)
        return fail(ZC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (bytes <= 0)
        return fail(ZC_ERR_INVALID_ARG, "bytes must be positive");
    void *ptr = nullptr;
    const hipError_t e = hipHostMalloc(&ptr, (size_t)bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ZC_ERR_NOMEM, "hipHostMalloc(%lld bytes): %s", (long long)bytes, hipGetErrorString(e));
    }
    *out = ptr;
    return ZC_OK;
}

zc_status zc_host_free(void *ptr)
{
    using namespace zc;
    if (!ptr)
        return ZC_OK;
    ZC_HIP(hipHostFree(ptr));
    return ZC_OK;
}

zc_status zc_offload_probe_link(zc_offload_ctx *ctx, const void *host_src, void *host_dst, int64_t bytes,
                                int32_t mode, float *ms_out)
{
    using namespace zc;
    if (!ctx || !ms_out)
        return fail(ZC_ERR_INVALID_ARG, "ctx / ms_out is NULL");
    if (bytes <= 0 || mode < 0 || mode > 2)
        return fail(ZC_ERR_INVALID_ARG, "need bytes > 0 and mode in {0, 1, 2}");
    const bool do_h2d = mode == 0 || mode == 2, do_d2h = mode == 1 || mode == 2;
    if (do_h2d) {
        if (!host_src)
            return fail(ZC_ERR_INVALID_ARG, "host_src is NULL");
        ZC_TRY(require_pinned(host_src, "host_src"));
    }
    if (do_d2h) {
        if (!host_dst)
            return fail(ZC_ERR_INVALID_ARG, "host_dst is NULL");
        ZC_TRY(require_pinned(host_dst, "host_dst"));
    }
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev != ctx->device)
        return fail(ZC_ERR_INVALID_ARG, "context belongs to device %d", ctx->device);
    // The staging ring is only a landing zone here: slots are reused without fences
    // because nobody reads what the probe copies.
    ZC_TRY(require_staging(ctx));
    const int64_t cb = ctx->chunk_bytes;
    const int64_t slots = (int64_t)ctx->num_buffers * 3;
    char *stage = reinterpret_cast<char *>(ctx->staging);
    ZC_HIP(hipStreamSynchronize(ctx->h2d));
    ZC_HIP(hipStreamSynchronize(ctx->d2h));
    const auto t0 = std::chrono::steady_clock::now();
    int64_t k = 0;
    for (int64_t off = 0; off < bytes; off += cb, ++k) {
        const size_t cnt = (size_t)((bytes - off) < cb ? (bytes - off) : cb);
        // the two directions use different halves of the ring where it has room for both
        const int64_t up = k % slots, down = (k + slots / 2) % slots;
        if (do_h2d)
            ZC_HIP(hipMemcpyAsync(stage + up * cb, static_cast<const char *>(host_src) + off, cnt,
                                  hipMemcpyHostToDevice, ctx->h2d));
        if (do_d2h)
            ZC_HIP(hipMemcpyAsync(static_cast<char *>(host_dst) + off, stage + down * cb, cnt,
                                  hipMemcpyDeviceToHost, ctx->d2h));
    }
    ZC_HIP(hipStreamSynchronize(ctx->h2d));
    ZC_HIP(hipStreamSynchronize(ctx->d2h));
    const auto t1 = std::chrono::steady_clock::now();
    *ms_out = std::chrono::duration<float, std::milli>(t1 - t0).count();
    return ZC_OK;
}

zc_status zc_offload_adam_step(zc_offload_ctx *ctx, float *p_dev, float *m_dev, float *v_dev,
                               int64_t n_resident, float *p_host, float *m_host, float *v_host,
                               int64_t n_streamed, const void *g_dev, zc_dtype g_dtype,
                               const zc_adam_hparams *hp, uint16_t *bf16_out_dev,
                               const int32_t *skip_flag, void *hip_stream)
{
    using namespace zc;
    if (!ctx)
        return fail(ZC_ERR_INVALID_ARG, "ctx is NULL");
    if (n_resident < 0 || n_streamed < 0)
        return fail(ZC_ERR_INVALID_ARG, "n_resident and n_streamed must be >= 0");
    if (n_resident > kMaxElements || n_streamed > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "partition exceeds 2^40 elements");
    ZC_TRY(check_dtype(g_dtype));
    ZC_TRY(check_hparams(hp));
    const int64_t n = n_resident + n_streamed;
    if (n == 0)
        return ZC_OK;
    if (!g_dev)
        return fail(ZC_ERR_INVALID_ARG, "g_dev is NULL");
    const int64_t g_size = g_dtype == ZC_BF16 ? 2 : 4;
    if (!aligned_to(g_dev, (uintptr_t)g_size))
        return fail(ZC_ERR_ALIGNMENT, "g_dev is not aligned to its element size");
    if (bf16_out_dev && !aligned_to(bf16_out_dev, 2))
        return fail(ZC_ERR_ALIGNMENT, "bf16_out_dev must be 2-byte aligned");
    if (skip_flag && !aligned_to(skip_flag, 4))
        return fail(ZC_ERR_ALIGNMENT, "skip_flag must be 4-byte aligned");
    if (n_resident > 0) {
        if (!p_dev || !m_dev || !v_dev)
            return fail(ZC_ERR_INVALID_ARG, "resident p/m/v must not be NULL when n_resident > 0");
        if (!aligned_to(p_dev, 4) || !aligned_to(m_dev, 4) || !aligned_to(v_dev, 4))
            return fail(ZC_ERR_ALIGNMENT, "resident p/m/v must be 4-byte aligned");
    }
    if (n_streamed > 0) {
        if (!p_host || !m_host || !v_host)
            return fail(ZC_ERR_INVALID_ARG, "host p/m/v must not be NULL when n_streamed > 0");
        if (!aligned_to(p_host, 4) || !aligned_to(m_host, 4) || !aligned_to(v_host, 4))
            return fail(ZC_ERR_ALIGNMENT, "host p/m/v must be 4-byte aligned");
        if (p_host == m_host || p_host == v_host || m_host == v_host)
            return fail(ZC_ERR_INVALID_ARG, "host p, m, v must be distinct buffers");
    }
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev != ctx->device)
        return fail(ZC_ERR_INVALID_ARG, "context was created on device %d, current device is %d",
                    ctx->device, dev);
    if (n_streamed > 0) {
        ZC_TRY(require_pinned(p_host, "p_host"));
        ZC_TRY(require_pinned(m_host, "m_host"));
        ZC_TRY(require_pinned(v_host, "v_host"));
    }

    hipStream_t stream = (hipStream_t)hip_stream;

    const char *g_tail = static_cast<const char *>(g_dev) + n_resident * g_size;
    uint16_t *out_tail = bf16_out_dev ? bf16_out_dev + n_resident : nullptr;

    if (tune().offload_zero_copy == 1 && n_streamed > 0) {
        // The update kernel itself reads and writes the pinned host arrays through the
        // link: no staging, no copy engines, one launch.  The link is the bound, so the
        // HBM-motivated cap on resident waves is lifted (more requests in flight).
        float *pd = nullptr, *md = nullptr, *vd = nullptr;
        ZC_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&pd), p_host, 0));
        ZC_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&md), m_host, 0));
        ZC_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&vd), v_host, 0));
        const bool side = n_resident > 0 && tune().offload_overlap_resident != 0;
        if (side) {
            // The resident prefix is bound by HBM, the streamed suffix by the link: run the
            // prefix on an internal stream next to the long link-bound launch instead of in
            // front of it (fork after what the caller has enqueued, join before returning).
            ZC_HIP(hipEventRecord(ctx->entry, stream));
            ZC_HIP(hipStreamWaitEvent(ctx->h2d, ctx->entry, 0));
        }
        // Prefix first: its short-lived workgroups take the compute units at once and hand
        // them over to the link-bound launch as they retire.
        if (n_resident > 0)
            ZC_TRY(launch_adam(p_dev, m_dev, v_dev, g_dev, g_dtype, n_resident, hp, bf16_out_dev, skip_flag,
                               side ? ctx->h2d : stream));
        // Launch shape for the link (knobs offload.zc_block / zc_rows / zc_waves_per_cu):
        // four-wave workgroups of two rows, no cap.  A sweep over
        // 64-256 threads, 1-4 rows and caps of 0-32 waves moved the rate between 43.9 and
        // 46.4 GB/s each way; the link, not the shape, is the bound.
        // Stores to host memory leave the chip whatever their cache policy; plain non-temporal
        // ones measured 1 % faster over the link than the write-through form used in HBM.
        const int link_nt = tune().adam_nontemporal == 4 ? 1 : (int)tune().adam_nontemporal;
        const AdamShape link_shape{(int)tune().offload_zc_rows, (int)tune().offload_zc_block, link_nt};
        ZC_TRY(launch_adam(pd, md, vd, g_tail, g_dtype, n_streamed, hp, out_tail, skip_flag, stream,
                           (int)tune().offload_zc_waves_per_cu, nullptr, nullptr, &link_shape));
        if (side) {
            ZC_HIP(hipEventRecord(ctx->done, ctx->h2d));
            ZC_HIP(hipStreamWaitEvent(stream, ctx->done, 0));
        }
        return ZC_OK;
    }

    if (n_streamed > 0)
        ZC_TRY(require_staging(ctx));   // before anything is enqueued: a failure leaves memory untouched

    // Resident prefix: one ordinary launch on the caller's stream.
    if (n_resident > 0)
        ZC_TRY(launch_adam(p_dev, m_dev, v_dev, g_dev, g_dtype, n_resident, hp, bf16_out_dev, skip_flag,
                           stream));
    if (n_streamed == 0)
        return ZC_OK;

    // Fence the copy streams behind whatever the caller has already enqueued.
    ZC_HIP(hipEventRecord(ctx->entry, stream));
    ZC_HIP(hipStreamWaitEvent(ctx->h2d, ctx->entry, 0));
    ZC_HIP(hipStreamWaitEvent(ctx->d2h, ctx->entry, 0));

    const int64_t ce = ctx->chunk_elems;
    const int nb = ctx->num_buffers;
    const int64_t nchunks = (n_streamed + ce - 1) / ce;

    // Transport 2 (staged reads, direct writes): a copy engine brings each chunk into a ring
    // slot (large read requests on the link), the update kernel reads the slot from HBM and
    // stores the new state straight into the pinned host arrays; nothing is copied back by
    // the runtime, and a slot is free again as soon as its kernel has finished.
    // Transport 0 (staged ring): the kernel updates the slot in place and a third stream
    // copies it back.
    const bool direct_writes = tune().offload_zero_copy == 2;
    float *pd = nullptr, *md = nullptr, *vd = nullptr;
    if (direct_writes) {
        ZC_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&pd), p_host, 0));
        ZC_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&md), m_host, 0));
        ZC_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&vd), v_host, 0));
    }
    for (int64_t k = 0; k < nchunks; ++k) {
        const int slot = (int)(k % nb);
        const int64_t off = k * ce;
        const int64_t cnt = (n_streamed - off) < ce ? (n_streamed - off) : ce;
        const size_t bytes = (size_t)cnt * 4;
        float *sp = ctx->staging + (int64_t)slot * 3 * ce;
        float *sm = sp + ce;
        float *sv = sm + ce;

        if (k >= nb) {
            // Optional host throttle: do not run more than num_buffers chunks ahead of the
            // slots that have been released (the event still holds chunk k - nb's record).
            if (tune().offload_max_ahead > 0)
                ZC_HIP(hipEventSynchronize(ctx->freed[slot]));
            ZC_HIP(hipStreamWaitEvent(ctx->h2d, ctx->freed[slot], 0));
        }
        ZC_HIP(hipMemcpyAsync(sp, p_host + off, bytes, hipMemcpyHostToDevice, ctx->h2d));
        ZC_HIP(hipMemcpyAsync(sm, m_host + off, bytes, hipMemcpyHostToDevice, ctx->h2d));
        ZC_HIP(hipMemcpyAsync(sv, v_host + off, bytes, hipMemcpyHostToDevice, ctx->h2d));
        ZC_HIP(hipEventRecord(ctx->loaded[slot], ctx->h2d));
        ZC_HIP(hipStreamWaitEvent(stream, ctx->loaded[slot], 0));

        uint16_t *out_k = out_tail ? out_tail + off : nullptr;
        hipStream_t releases = stream;           // the stream whose progress frees the slot
        if (direct_writes) {
            const AdamOut to_host{pd + off, md + off, vd + off};
            ZC_TRY(launch_adam(sp, sm, sv, g_tail + off * g_size, g_dtype, cnt, hp, out_k, skip_flag, stream,
                               (int)tune().offload_zc_waves_per_cu, nullptr, &to_host));
        } else {
            ZC_TRY(launch_adam(sp, sm, sv, g_tail + off * g_size, g_dtype, cnt, hp, out_k, skip_flag, stream));
            ZC_HIP(hipEventRecord(ctx->updated[slot], stream));
            if (!tune().offload_d2h_on_compute) {    // else: copy back in order behind the kernel
                releases = ctx->d2h;
                ZC_HIP(hipStreamWaitEvent(ctx->d2h, ctx->updated[slot], 0));
            }
            ZC_HIP(hipMemcpyAsync(p_host + off, sp, bytes, hipMemcpyDeviceToHost, releases));
            ZC_HIP(hipMemcpyAsync(m_host + off, sm, bytes, hipMemcpyDeviceToHost, releases));
            ZC_HIP(hipMemcpyAsync(v_host + off, sv, bytes, hipMemcpyDeviceToHost, releases));
        }
        if (tune().offload_poison)
            ZC_TRY(launch_poison(sp, 3 * ce, releases));
        ZC_HIP(hipEventRecord(ctx->freed[slot], releases));
    }
    if (!direct_writes) {
        // The caller's stream resumes only after the last copy-back has landed.
        ZC_HIP(hipEventRecord(ctx->done, ctx->d2h));
        ZC_HIP(hipStreamWaitEvent(stream, ctx->done, 0));
    }
    return ZC_OK;
}

}  // extern "C"

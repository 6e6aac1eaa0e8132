// Error reporting, tuning knobs, device queries and the host-only layout helper.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "zc_internal.h"

namespace zc {

static thread_local char g_err[512] = "";

zc_status fail(zc_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

zc_status hip_fail(hipError_t e, const char *what)
{
    return fail(ZC_ERR_HIP, "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
}

void clear_error() { g_err[0] = '\0'; }

// One set of knobs per calling thread: a sweep on one thread never changes the kernels another
// thread launches, and a thread that never calls zc_tune_set always launches the defaults.
Tune &tune()
{
    static thread_local Tune t;
    return t;
}

zc_status num_cus(int *out)
{
    static std::mutex mu;
    static int cached[64];
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64)
        return fail(ZC_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int cus = 0;
        ZC_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (cus <= 0)
            return fail(ZC_ERR_HIP, "device %d reports %d compute units", dev, cus);
        cached[dev] = cus;
    }
    *out = cached[dev];
    return ZC_OK;
}

zc_status occupancy_cap_lds(int waves_per_cu, int block_threads, size_t *lds_bytes)
{
    *lds_bytes = 0;
    if (waves_per_cu <= 0)
        return ZC_OK;
    static std::mutex mu;
    static int lds_per_cu[64];
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64)
        return fail(ZC_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    {
        std::lock_guard<std::mutex> lock(mu);
        if (lds_per_cu[dev] == 0) {
            int bytes = 0;
            ZC_HIP(hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev));
            if (bytes <= 0)
                bytes = 64 * 1024;
            lds_per_cu[dev] = bytes;
        }
    }
    const int waves_per_block = (block_threads + 63) / 64;
    int blocks = waves_per_cu / waves_per_block;
    if (blocks < 1)
        blocks = 1;
    // Largest request that still lets `blocks` workgroups share one CU's LDS.
    size_t bytes = (size_t)lds_per_cu[dev] / (size_t)blocks;
    bytes &= ~(size_t)255;
    if (bytes > 64 * 1024)
        bytes = 64 * 1024;  // default per-workgroup limit for dynamic LDS
    *lds_bytes = bytes;
    return ZC_OK;
}

zc_status check_dtype(zc_dtype t)
{
    if (t != ZC_F32 && t != ZC_BF16)
        return fail(ZC_ERR_INVALID_ARG, "g_dtype %d is neither ZC_F32 nor ZC_BF16", (int)t);
    return ZC_OK;
}

zc_status check_hparams(const zc_adam_hparams *hp)
{
    if (!hp)
        return fail(ZC_ERR_INVALID_ARG, "hp is NULL");
    if (!std::isfinite(hp->lr))
        return fail(ZC_ERR_INVALID_ARG, "lr must be finite");
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f))
        return fail(ZC_ERR_INVALID_ARG, "beta1 must be in [0, 1)");
    if (!(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(ZC_ERR_INVALID_ARG, "beta2 must be in [0, 1)");
    if (!(hp->eps >= 0.0f) || !std::isfinite(hp->eps))
        return fail(ZC_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (!std::isfinite(hp->weight_decay))
        return fail(ZC_ERR_INVALID_ARG, "weight_decay must be finite");
    if (!std::isfinite(hp->grad_scale))
        return fail(ZC_ERR_INVALID_ARG, "grad_scale must be finite");
    if (hp->step < 1)
        return fail(ZC_ERR_INVALID_ARG, "step is 1-based, got %lld", (long long)hp->step);
    if (hp->mode != ZC_ADAMW && hp->mode != ZC_ADAM_L2)
        return fail(ZC_ERR_INVALID_ARG, "mode %d is neither ZC_ADAMW nor ZC_ADAM_L2", (int)hp->mode);
    if (hp->reserved != 0)
        return fail(ZC_ERR_INVALID_ARG, "reserved field must be 0");
    return ZC_OK;
}

struct Knob {
    const char *key;
    int64_t Tune::*field;
    int64_t lo, hi;
};

static const Knob kKnobs[] = {
    {"adam.rows", &Tune::adam_rows, 1, 4},
    {"adam.block", &Tune::adam_block, 64, 256},
    {"adam.waves_per_cu", &Tune::adam_waves_per_cu, -1, 64},
    {"adam.nontemporal", &Tune::adam_nontemporal, 0, 4},
    {"adam.arith", &Tune::adam_arith, 0, 2},
    {"reduce.unroll", &Tune::reduce_unroll, 2, 8},
    {"reduce.blocks_per_cu", &Tune::reduce_blocks_per_cu, 1, 16},
    {"copy.waves_per_cu", &Tune::copy_waves_per_cu, 0, 64},
    {"cast.waves_per_cu", &Tune::cast_waves_per_cu, 0, 64},
    {"accum.waves_per_cu", &Tune::accum_waves_per_cu, 0, 64},
    {"copy.nontemporal", &Tune::copy_nontemporal, 0, 2},
    {"launch.max_grid", &Tune::launch_max_grid, 1, int64_t(1) << 30},
    {"offload.zero_copy", &Tune::offload_zero_copy, 0, 2},
    {"offload.zc_waves_per_cu", &Tune::offload_zc_waves_per_cu, 0, 64},
    {"offload.zc_block", &Tune::offload_zc_block, 64, 256},
    {"offload.zc_rows", &Tune::offload_zc_rows, 1, 4},
    {"offload.max_ahead", &Tune::offload_max_ahead, 0, 1},
    {"offload.d2h_on_compute", &Tune::offload_d2h_on_compute, 0, 1},
    {"offload.poison", &Tune::offload_poison, 0, 1},
    {"offload.overlap_resident", &Tune::offload_overlap_resident, 0, 1},
};

static const Knob *find_knob(const char *key)
{
    if (!key)
        return nullptr;
    for (const Knob &k : kKnobs)
        if (std::strcmp(k.key, key) == 0)
            return &k;
    return nullptr;
}

}  // namespace zc

extern "C" {

int zc_version(void) { return 20100; }   // 2.1.0: packed optimizer state

const char *zc_last_error(void) { return zc::g_err; }

zc_status zc_tune_set(const char *key, int64_t value)
{
    const zc::Knob *k = zc::find_knob(key);
    if (!k)
        return zc::fail(ZC_ERR_INVALID_ARG, "unknown tuning key '%s'", key ? key : "(null)");
    const bool pow2 = value > 0 && (value & (value - 1)) == 0;
    if (value < k->lo || value > k->hi ||
        ((k->field == &zc::Tune::adam_rows || k->field == &zc::Tune::adam_block ||
          k->field == &zc::Tune::reduce_unroll || k->field == &zc::Tune::offload_zc_block ||
          k->field == &zc::Tune::offload_zc_rows) && !pow2))
        return zc::fail(ZC_ERR_INVALID_ARG, "value %lld out of range for '%s'", (long long)value, key);
    zc::tune().*(k->field) = value;
    return ZC_OK;
}

zc_status zc_tune_get(const char *key, int64_t *value_out)
{
    const zc::Knob *k = zc::find_knob(key);
    if (!k || !value_out)
        return zc::fail(ZC_ERR_INVALID_ARG, "unknown tuning key or NULL output");
    *value_out = zc::tune().*(k->field);
    return ZC_OK;
}

zc_status zc_flat_layout(const int64_t *numels, int64_t ntensors, int32_t world, int64_t shard_align,
                         int64_t *offsets_out, int64_t *shard_numel_out, int64_t *total_out)
{
    if (ntensors < 0 || world < 1 || shard_align < 1)
        return zc::fail(ZC_ERR_INVALID_ARG, "need ntensors >= 0, world >= 1, shard_align >= 1");
    if (shard_align > zc::kMaxElements)
        return zc::fail(ZC_ERR_UNSUPPORTED, "shard_align exceeds 2^40 elements");
    if (ntensors > 0 && (!numels || !offsets_out))
        return zc::fail(ZC_ERR_INVALID_ARG, "numels / offsets_out is NULL");
    if (!shard_numel_out || !total_out)
        return zc::fail(ZC_ERR_INVALID_ARG, "shard_numel_out / total_out is NULL");
    const int64_t limit = zc::kMaxElements * 64;
    int64_t running = 0;
    for (int64_t t = 0; t < ntensors; ++t) {
        if (numels[t] < 0)
            return zc::fail(ZC_ERR_INVALID_ARG, "numels[%lld] is negative", (long long)t);
        if (numels[t] > limit - running)
            return zc::fail(ZC_ERR_UNSUPPORTED, "total size exceeds 2^46 elements");
        running += numels[t];
    }
    // Write outputs only after the whole table has been validated.
    running = 0;
    for (int64_t t = 0; t < ntensors; ++t) {
        offsets_out[t] = running;
        running += numels[t];
    }
    const int64_t per_rank = (running + world - 1) / world;
    *shard_numel_out = (per_rank + shard_align - 1) / shard_align * shard_align;
    *total_out = running;
    return ZC_OK;
}

zc_status zc_per_tensor_layout(const int64_t *numels, int64_t ntensors, int32_t world, int64_t align,
                               int64_t *src_offsets_out, int64_t *dst_offsets_out,
                               int64_t *seg_numels_out, int64_t *send_numel_out)
{
    if (ntensors < 0 || world < 1 || align < 1)
        return zc::fail(ZC_ERR_INVALID_ARG, "need ntensors >= 0, world >= 1, align >= 1");
    if (align > zc::kMaxElements)
        return zc::fail(ZC_ERR_UNSUPPORTED, "align exceeds 2^40 elements");
    if (ntensors > 0 && (!numels || !src_offsets_out || !dst_offsets_out || !seg_numels_out))
        return zc::fail(ZC_ERR_INVALID_ARG, "numels or an output table is NULL");
    if (!send_numel_out)
        return zc::fail(ZC_ERR_INVALID_ARG, "send_numel_out is NULL");
    const int64_t limit = zc::kMaxElements * 64;
    // Pass 1: validate and size one rank's send buffer.
    int64_t send = 0;
    for (int64_t t = 0; t < ntensors; ++t) {
        if (numels[t] < 0)
            return zc::fail(ZC_ERR_INVALID_ARG, "numels[%lld] is negative", (long long)t);
        if (numels[t] > limit)
            return zc::fail(ZC_ERR_UNSUPPORTED, "tensor %lld exceeds 2^46 elements", (long long)t);
        const int64_t slice = ((numels[t] + world - 1) / world + align - 1) / align * align;
        if (slice > (limit - send))
            return zc::fail(ZC_ERR_UNSUPPORTED, "send buffer exceeds 2^46 elements");
        send += slice;
    }
    if (send > limit / world)
        return zc::fail(ZC_ERR_UNSUPPORTED, "gathered buffer exceeds 2^46 elements");
    // Pass 2: one segment per (tensor, rank); ranks that hold only padding get numel 0.
    int64_t inside = 0;
    for (int64_t t = 0; t < ntensors; ++t) {
        const int64_t n = numels[t];
        const int64_t slice = ((n + world - 1) / world + align - 1) / align * align;
        for (int32_t r = 0; r < world; ++r) {
            const int64_t first = (int64_t)r * slice;
            int64_t count = n - first;
            if (count > slice)
                count = slice;
            if (count < 0)
                count = 0;
            const int64_t k = t * world + r;
            src_offsets_out[k] = (int64_t)r * send + inside;
            dst_offsets_out[k] = count > 0 ? first : 0;
            seg_numels_out[k] = count;
        }
        inside += slice;
    }
    *send_numel_out = send;
    return ZC_OK;
}

}  // extern "C"

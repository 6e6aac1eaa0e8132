// Internal declarations shared by the translation units of libzc.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zc.h"

namespace zc {

// Records a message for zc_last_error() and returns `code`.
zc_status fail(zc_status code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
zc_status hip_fail(hipError_t e, const char *what);
void clear_error();

#define ZC_HIP(call)                                   \
    do {                                               \
        hipError_t zc_e_ = (call);                     \
        if (zc_e_ != hipSuccess)                       \
            return ::zc::hip_fail(zc_e_, #call);       \
    } while (0)

#define ZC_TRY(call)                 \
    do {                             \
        zc_status zc_s_ = (call);    \
        if (zc_s_ != ZC_OK)          \
            return zc_s_;            \
    } while (0)

struct Tune {
    int64_t adam_rows = 1;
    int64_t adam_block = 64;
    int64_t adam_waves_per_cu = -1;   // -1: chosen per variant at launch
    int64_t adam_nontemporal = 4;     // non-temporal loads, write-through streaming stores
    int64_t adam_arith = 2;
    int64_t reduce_unroll = 8;
    int64_t reduce_blocks_per_cu = 2;
    int64_t copy_waves_per_cu = 16;
    int64_t cast_waves_per_cu = 20;
    int64_t accum_waves_per_cu = 24;
    int64_t copy_nontemporal = 2;     // the same for cast, unshard and accumulation
    int64_t launch_max_grid = int64_t(1) << 30;
    int64_t offload_zero_copy = 1;   // 0 staged ring, 1 zero-copy kernel, 2 staged reads + direct writes
    int64_t offload_zc_waves_per_cu = 0;
    int64_t offload_zc_block = 256;  // launch shape of the link-bound zero-copy kernel
    int64_t offload_zc_rows = 2;
    int64_t offload_max_ahead = 1;
    int64_t offload_d2h_on_compute = 0;
    int64_t offload_overlap_resident = 1;   // zero-copy: resident prefix on a side stream
    int64_t offload_poison = 0;      // overwrite every ring slot once its chunk has left it
};
Tune &tune();

// Compute units of the current device (cached per device ordinal).
zc_status num_cus(int *out);

// Dynamic-LDS request (bytes, never touched by the kernel) that limits a kernel
// with `block_threads` threads per workgroup to about `waves_per_cu` resident
// waves per compute unit; 0 waves means no cap (0 bytes).
zc_status occupancy_cap_lds(int waves_per_cu, int block_threads, size_t *lds_bytes);

// Host-side validation shared by the resident and the offloaded step.
zc_status check_hparams(const zc_adam_hparams *hp);
zc_status check_dtype(zc_dtype t);

// Enqueue the fused update over n elements; arguments already validated.
// waves_per_cu < 0 takes the "adam.waves_per_cu" knob, otherwise overrides it.
// grad_scale_dev (DEVICE, may be NULL) multiplies hp->grad_scale at execution time.
// out_of_place (may be NULL): the new p, m, v go to these arrays instead of back into
// p, m, v, which are then only read.
struct AdamOut {
    float *p, *m, *v;
};
// shape (may be NULL): rows per lane, threads per workgroup and access mode for this launch
// instead of the "adam.rows" / "adam.block" / "adam.nontemporal" knobs (the link-bound launches of the offloaded step want a
// different shape than the HBM-bound ones).
struct AdamShape {
    int rows, block;
    int nontemporal;   // a value of "adam.nontemporal"
};
zc_status launch_adam(float *p, float *m, float *v, const void *g, zc_dtype g_dtype, int64_t n,
                      const zc_adam_hparams *hp, uint16_t *bf16_out, const int32_t *skip_flag,
                      hipStream_t stream, int waves_per_cu = -1, const float *grad_scale_dev = nullptr,
                      const AdamOut *out_of_place = nullptr, const AdamShape *shape = nullptr);

// Fill `words` 32-bit words at dst (DEVICE) with 0xDEADBEEF on `stream`.
zc_status launch_poison(void *dst, int64_t words, hipStream_t stream);

#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC__)
// Streaming stores that leave the L2 at once: buffer stores with the non-temporal and the
// device-scope (sc1) bits set.  An ordinary or merely non-temporal store stays in the XCD's
// L2 as a dirty line and is written back whenever the cache evicts it, at a moment unrelated
// to the stream; written through right away, the stores of a tile reach DRAM together, which
// measured 1-3 % faster and made the rate depend less on where the caller's arrays lie
// relative to each other.  The descriptor covers exactly the bytes the workgroup may write
// (base and size must be uniform across the wave), so the hardware drops anything beyond.
constexpr int kBufferFlags = 0x00020000;      // raw buffer, 32-bit data format (gfx9 family)
constexpr int kAuxStreamOut = 2 | 16;         // nt | sc1
typedef uint32_t stream_u32x4 __attribute__((vector_size(16)));
typedef uint32_t stream_u32x2 __attribute__((vector_size(8)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t stream_out_rsrc(void *base, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, kBufferFlags);
}
#endif

// Workgroups one launch may have: the "launch.max_grid" knob, and never so many that the
// launch would exceed 2^32 - 1 threads in x.  The dispatch packet counts threads in 32 bits,
// and a larger launch does not fail: it silently runs the count modulo 2^32.
inline int64_t max_workgroups_per_launch(int64_t knob, int block_threads)
{
    const int64_t hw = int64_t(0xFFFFFFFFu) / block_threads;
    return knob < hw ? knob : hw;
}

inline bool aligned_to(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr int64_t kMaxElements = int64_t(1) << 40;

}  // namespace zc

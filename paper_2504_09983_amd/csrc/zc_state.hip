// Packing three state arrays into the granule-interleaved layout of zc_adam_step_packed and
// back.  Both are plain streaming copies (24 bytes per element) that run once when a partition
// is created, loaded from or written to a checkpoint; they use 128-bit accesses when every
// array allows it and fall back to one element per lane otherwise.
#include "zc_internal.h"

namespace zc {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kStateGranuleShift = 13;
constexpr int64_t kStateGranule = int64_t(1) << kStateGranuleShift;
static_assert(kStateGranule == ZC_PACKED_GRANULE, "the header and the kernels must agree on the granule");

// Index of p[e] in the packed array; m[e] is one granule and v[e] two granules behind it.
__device__ __forceinline__ int64_t state_at(int64_t e)
{
    return e + ((e >> kStateGranuleShift) << (kStateGranuleShift + 1));
}

// The ragged end and misaligned arrays: elements [lo, hi), one per lane (W = 1), grid-stride.
// PACK: state <- p, m, v, a NULL source or an element at or beyond n giving 0.
// else: p, m, v <- state, NULL destinations skipped (hi <= n).
template <typename T, bool PACK>
__global__ __launch_bounds__(256) void state_copy_kernel(float *state, float *p, float *m, float *v,
                                                         int64_t lo, int64_t hi, int64_t n)
{
    constexpr int W = sizeof(T) / 4;
    const int64_t stride = (int64_t)gridDim.x * 256 * W;
    for (int64_t e = lo + ((int64_t)blockIdx.x * 256 + threadIdx.x) * W; e < hi; e += stride) {
        T *sp = reinterpret_cast<T *>(state + state_at(e));
        T *sm = reinterpret_cast<T *>(state + state_at(e) + kStateGranule);
        T *sv = reinterpret_cast<T *>(state + state_at(e) + 2 * kStateGranule);
        if constexpr (PACK) {
            const bool inside = e + W <= n;
            T zero = {};
            *sp = (p && inside) ? *reinterpret_cast<const T *>(p + e) : zero;
            *sm = (m && inside) ? *reinterpret_cast<const T *>(m + e) : zero;
            *sv = (v && inside) ? *reinterpret_cast<const T *>(v + e) : zero;
        } else {
            if (p)
                *reinterpret_cast<T *>(p + e) = *sp;
            if (m)
                *reinterpret_cast<T *>(m + e) = *sm;
            if (v)
                *reinterpret_cast<T *>(v + e) = *sv;
        }
    }
}

// The wide path: one-wave workgroups in tile order, kStateRows 16-byte vectors per lane and
// array, all loads of a tile issued before its stores, non-temporal both ways.  Elements
// [0, 4 * nvec); `tile0` is the tile of workgroup 0.
constexpr int kStateRows = 4;

template <bool PACK>
__global__ __launch_bounds__(64) void state_tile_kernel(float *state, float *p, float *m, float *v,
                                                        int64_t nvec, int64_t tile0)
{
    const int64_t first = (tile0 + blockIdx.x) * (64 * kStateRows) + threadIdx.x;
    f32x4 a[kStateRows], b[kStateRows], c[kStateRows];
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < kStateRows; ++r) {
        const int64_t i = first + r * 64;
        if (i < nvec) {
            const int64_t at = state_at(i << 2);
            if constexpr (PACK) {
                a[r] = p ? __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p) + i) : zero;
                b[r] = m ? __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(m) + i) : zero;
                c[r] = v ? __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(v) + i) : zero;
            } else {
                if (p) a[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(state + at));
                if (m) b[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(state + at + kStateGranule));
                if (v) c[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(state + at + 2 * kStateGranule));
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kStateRows; ++r) {
        const int64_t i = first + r * 64;
        if (i < nvec) {
            const int64_t at = state_at(i << 2);
            if constexpr (PACK) {
                __builtin_nontemporal_store(a[r], reinterpret_cast<f32x4 *>(state + at));
                __builtin_nontemporal_store(b[r], reinterpret_cast<f32x4 *>(state + at + kStateGranule));
                __builtin_nontemporal_store(c[r], reinterpret_cast<f32x4 *>(state + at + 2 * kStateGranule));
            } else {
                if (p) __builtin_nontemporal_store(a[r], reinterpret_cast<f32x4 *>(p) + i);
                if (m) __builtin_nontemporal_store(b[r], reinterpret_cast<f32x4 *>(m) + i);
                if (v) __builtin_nontemporal_store(c[r], reinterpret_cast<f32x4 *>(v) + i);
            }
        }
    }
}

template <bool PACK>
static zc_status run_state_copy(float *state, float *p, float *m, float *v, int64_t n, hipStream_t stream)
{
    int cus = 0;
    ZC_TRY(num_cus(&cus));
    const bool vec = (!p || aligned_to(p, 16)) && (!m || aligned_to(m, 16)) && (!v || aligned_to(v, 16));
    // whole vectors inside n take the wide kernel; the ragged end (and, when packing, the
    // padding up to the end of the last granule) goes element by element
    const int64_t wide_end = vec ? (n & ~int64_t(3)) : 0;
    const int64_t end = PACK ? ((n + kStateGranule - 1) >> kStateGranuleShift << kStateGranuleShift) : n;
    auto blocks_for = [&](int64_t lanes) {
        int64_t b = (lanes + 255) / 256;
        const int64_t cap = (int64_t)cus * 16;
        return dim3((unsigned)(b < 1 ? 1 : (b > cap ? cap : b)));
    };
    if (wide_end > 0) {
        const int64_t nvec = wide_end >> 2;
        const int64_t ntiles = (nvec + 64 * kStateRows - 1) / (64 * kStateRows);
        size_t lds = 0;
        ZC_TRY(occupancy_cap_lds((int)tune().copy_waves_per_cu, 64, &lds));
        const int64_t per_launch = max_workgroups_per_launch(tune().launch_max_grid, 64);
        for (int64_t tile0 = 0; tile0 < ntiles; tile0 += per_launch) {
            const int64_t count = (ntiles - tile0) < per_launch ? (ntiles - tile0) : per_launch;
            hipLaunchKernelGGL((state_tile_kernel<PACK>), dim3((unsigned)count), dim3(64), lds, stream, state, p, m,
                               v, nvec, tile0);
        }
    }
    if (end > wide_end)
        hipLaunchKernelGGL((state_copy_kernel<float, PACK>), blocks_for(end - wide_end), dim3(256), 0, stream,
                           state, p, m, v, wide_end, end, n);
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

static zc_status check_state_args(const float *state, const float *p, const float *m, const float *v,
                                  int64_t n)
{
    if (n < 0)
        return fail(ZC_ERR_INVALID_ARG, "n is negative (%lld)", (long long)n);
    if (n > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "n exceeds 2^40 elements");
    if (n == 0)
        return ZC_OK;
    if (!state)
        return fail(ZC_ERR_INVALID_ARG, "state must not be NULL when n > 0");
    if (!aligned_to(state, 128))
        return fail(ZC_ERR_ALIGNMENT, "state must be 128-byte aligned");
    if (!aligned_to(p, 4) || !aligned_to(m, 4) || !aligned_to(v, 4))
        return fail(ZC_ERR_ALIGNMENT, "p, m, v must be 4-byte aligned");
    const uintptr_t s_lo = (uintptr_t)state, s_hi = s_lo + (uintptr_t)zc_packed_state_numel(n) * 4;
    const float *arrays[3] = {p, m, v};
    for (int a = 0; a < 3; ++a) {
        if (!arrays[a])
            continue;
        const uintptr_t lo = (uintptr_t)arrays[a], hi = lo + (uintptr_t)n * 4;
        if (lo < s_hi && s_lo < hi)
            return fail(ZC_ERR_INVALID_ARG, "p, m, v must not overlap the packed state");
        for (int b = a + 1; b < 3; ++b) {
            if (!arrays[b])
                continue;
            const uintptr_t lo2 = (uintptr_t)arrays[b], hi2 = lo2 + (uintptr_t)n * 4;
            if (lo < hi2 && lo2 < hi)
                return fail(ZC_ERR_INVALID_ARG, "p, m, v must not overlap each other");
        }
    }
    return ZC_OK;
}

}  // namespace zc

extern "C" zc_status zc_state_pack(const float *p, const float *m, const float *v, int64_t n, float *state,
                                   void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_state_args(state, p, m, v, n));
    if (n == 0)
        return ZC_OK;
    return run_state_copy<true>(state, const_cast<float *>(p), const_cast<float *>(m), const_cast<float *>(v), n,
                                (hipStream_t)hip_stream);
}

extern "C" zc_status zc_state_unpack(const float *state, int64_t n, float *p, float *m, float *v,
                                     void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_state_args(state, p, m, v, n));
    if (n == 0 || (!p && !m && !v))
        return ZC_OK;
    return run_state_copy<false>(const_cast<float *>(state), p, m, v, n, (hipStream_t)hip_stream);
}

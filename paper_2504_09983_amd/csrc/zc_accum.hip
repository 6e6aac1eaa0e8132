// Gradient accumulation into the fp32 gradient partition:
//   acc[i] += upcast(micro[i]) * scale
// (paper: fp32 gradients are kept per rank, Experimental settings; with
// gradient accumulation several forward/backward passes add into them before
// one parameter update, Selective unsharding).  Streaming, 10 bytes per element
// with bf16 micro-gradients (2 + 4 read, 4 written), same tile shape as the
// other kernels: single-wave workgroups, one tile each, capped resident waves.
#include "zc_internal.h"

namespace zc {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kAccBlock = 64;
constexpr int kAccRows = 4;

// The sum is formed in fp64 (the product of two fp32 values is exact there) and
// rounded to fp32 once.
__device__ __forceinline__ float acc_elem(float a, float g, double scale)
{
    return (float)((double)a + (double)g * scale);
}

// Requires acc 16-byte aligned and micro aligned to 4 elements.
// STREAM: the sums are written with write-through streaming stores (stream_out_rsrc) instead
// of plain non-temporal ones.
template <bool G_BF16, bool STREAM>
__global__ __launch_bounds__(kAccBlock) void accumulate_vec_kernel(float *__restrict__ acc,
                                                                   const void *__restrict__ micro,
                                                                   int64_t n, int64_t tile0, double scale)
{
    const int64_t nvec = n >> 2;
    f32x4 *a4 = reinterpret_cast<f32x4 *>(acc);
    const int64_t tile = tile0 + blockIdx.x;
    const int64_t first = tile * (kAccBlock * kAccRows) + threadIdx.x;
    f32x4 av[kAccRows], gv[kAccRows];
#pragma unroll
    for (int r = 0; r < kAccRows; ++r) {
        const int64_t i = first + r * kAccBlock;
        if (i < nvec) {
            av[r] = __builtin_nontemporal_load(a4 + i);
            if constexpr (G_BF16) {
                const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(micro) + i);
                gv[r].x = __uint_as_float(w.x << 16);
                gv[r].y = __uint_as_float(w.x & 0xFFFF0000u);
                gv[r].z = __uint_as_float(w.y << 16);
                gv[r].w = __uint_as_float(w.y & 0xFFFF0000u);
            } else {
                gv[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(micro) + i);
            }
        }
    }
    const int64_t tile_first = tile * (kAccBlock * kAccRows);
    int64_t room = nvec - tile_first;
    room = room < 0 ? 0 : (room > kAccBlock * kAccRows ? kAccBlock * kAccRows : room);
    const __amdgpu_buffer_rsrc_t ra = stream_out_rsrc(a4 + tile_first, room * 16);
#pragma unroll
    for (int r = 0; r < kAccRows; ++r) {
        const int64_t i = first + r * kAccBlock;
        if (i < nvec) {
            f32x4 o;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                o[k] = acc_elem(av[r][k], gv[r][k], scale);
            if constexpr (STREAM)
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(stream_u32x4, o), ra,
                                                       (int)(threadIdx.x + r * kAccBlock) * 16, 0, kAuxStreamOut);
            else
                __builtin_nontemporal_store(o, a4 + i);
        }
    }
    const int64_t i = (nvec << 2) + threadIdx.x;
    if (tile == 0 && threadIdx.x < 4 && i < n) {
        float g;
        if constexpr (G_BF16)
            g = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(micro)[i] << 16);
        else
            g = reinterpret_cast<const float *>(micro)[i];
        acc[i] = acc_elem(acc[i], g, scale);
    }
}

template <bool G_BF16>
__global__ __launch_bounds__(256) void accumulate_scalar_kernel(float *__restrict__ acc,
                                                                const void *__restrict__ micro, int64_t n,
                                                                double scale)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        float g;
        if constexpr (G_BF16)
            g = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(micro)[i] << 16);
        else
            g = reinterpret_cast<const float *>(micro)[i];
        acc[i] = acc_elem(acc[i], g, scale);
    }
}

}  // namespace zc

extern "C" zc_status zc_grad_accumulate(float *acc, const void *micro, zc_dtype micro_dtype, int64_t n,
                                        float scale, void *hip_stream)
{
    using namespace zc;
    if (n < 0)
        return fail(ZC_ERR_INVALID_ARG, "n is negative (%lld)", (long long)n);
    if (n > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "n exceeds 2^40 elements");
    ZC_TRY(check_dtype(micro_dtype));
    if (scale != scale || scale - scale != 0.0f)
        return fail(ZC_ERR_INVALID_ARG, "scale must be finite");
    if (n == 0)
        return ZC_OK;
    if (!acc || !micro)
        return fail(ZC_ERR_INVALID_ARG, "acc and micro must not be NULL when n > 0");
    const bool bf16 = micro_dtype == ZC_BF16;
    if (!aligned_to(acc, 4))
        return fail(ZC_ERR_ALIGNMENT, "acc must be 4-byte aligned");
    if (!aligned_to(micro, bf16 ? 2 : 4))
        return fail(ZC_ERR_ALIGNMENT, "micro is not aligned to its element size");
    if ((const void *)acc == micro)
        return fail(ZC_ERR_INVALID_ARG, "acc and micro must be distinct buffers");
    hipStream_t stream = (hipStream_t)hip_stream;
    if (aligned_to(acc, 16) && aligned_to(micro, bf16 ? 8 : 16)) {
        const int64_t nvec = n >> 2;
        const int64_t tile_vecs = kAccBlock * kAccRows;
        int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;
        if (ntiles == 0)
            ntiles = 1;
        size_t lds = 0;
        ZC_TRY(occupancy_cap_lds((int)tune().accum_waves_per_cu, kAccBlock, &lds));
        const int64_t kAccMaxGrid = max_workgroups_per_launch(tune().launch_max_grid, kAccBlock);
        for (int64_t tile0 = 0; tile0 < ntiles; tile0 += kAccMaxGrid) {
            const int64_t count = (ntiles - tile0) < kAccMaxGrid ? (ntiles - tile0) : kAccMaxGrid;
            const bool stream_out = tune().copy_nontemporal == 2;
#define ZC_ACC(GB, ST)                                                                                  \
    hipLaunchKernelGGL((accumulate_vec_kernel<GB, ST>), dim3((unsigned)count), dim3(kAccBlock), lds, stream, \
                       acc, micro, n, tile0, (double)scale)
            if (bf16) {
                if (stream_out) ZC_ACC(true, true);
                else ZC_ACC(true, false);
            } else {
                if (stream_out) ZC_ACC(false, true);
                else ZC_ACC(false, false);
            }
#undef ZC_ACC
        }
    } else {
        int cus = 0;
        ZC_TRY(num_cus(&cus));
        int64_t blocks = (n + 255) / 256;
        if (blocks > (int64_t)cus * 32)
            blocks = (int64_t)cus * 32;
        if (bf16)
            hipLaunchKernelGGL(accumulate_scalar_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream,
                               acc, micro, n, (double)scale);
        else
            hipLaunchKernelGGL(accumulate_scalar_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream,
                               acc, micro, n, (double)scale);
    }
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

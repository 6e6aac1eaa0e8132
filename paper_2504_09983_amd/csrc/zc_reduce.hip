// Squared gradient norm and non-finite check over a flat partition.
//
// Streaming read (2 or 4 bytes per element).  Each lane keeps four fp32
// partial sums per tile (one per vector slot, 4-8 terms each) and folds them into a
// double once per tile, a wave folds the lanes' doubles with cross-lane
// shuffles (DPP / permute on gfx950), waves meet in LDS, every workgroup writes
// one double partial, and a single small workgroup folds the partials in a
// fixed order, so the result is deterministic for a given n.
#include <map>
#include <mutex>
#include <new>
#include <utility>

#include "zc_internal.h"

namespace zc {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxPartials = 4096;

struct Partial {
    double sum;
    uint32_t bad;
    uint32_t pad;
};

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ uint32_t wave_or(uint32_t x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x |= (uint32_t)__shfl_xor((int)x, off, 64);
    return x;
}

__device__ __forceinline__ void block_fold(double sum, uint32_t bad, Partial *out)
{
    __shared__ double s_sum[4];
    __shared__ uint32_t s_bad[4];
    sum = wave_sum(sum);
    bad = wave_or(bad);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        s_sum[wave] = sum;
        s_bad[wave] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        Partial r;
        r.sum = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
        r.bad = s_bad[0] | s_bad[1] | s_bad[2] | s_bad[3];
        r.pad = 0;
        *out = r;
    }
}


constexpr int kFoldLoads = 4;  // loads whose squares are summed in fp32 before going to double

// bf16 input, 8 elements (16 bytes) per lane per load, UNROLL loads issued back to back.
// Requires 16-byte alignment.  fp32 sums run over the squares of at most kFoldLoads loads
// (8 terms in each of four accumulators) and are folded into the lane's double sum from
// there, so the result stays within an fp32 rounding of the exact sum whatever UNROLL is.
template <int UNROLL>
__global__ __launch_bounds__(256) void sqnorm_bf16_kernel(const uint16_t *__restrict__ g, int64_t n,
                                                          Partial *__restrict__ partials)
{
    const int64_t nvec = n >> 3;
    const u32x4 *g4 = reinterpret_cast<const u32x4 *>(g);
    double sum = 0.0;
    uint32_t worst = 0;  // running max of |bits| per half-word; >= 0x7F80 means Inf/NaN
    const int64_t tile_vecs = 256 * UNROLL;
    const int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t first = tile * tile_vecs + threadIdx.x;
        u32x4 w[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = first + u * 256;
            w[u] = i < nvec ? __builtin_nontemporal_load(g4 + i) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int q = 0; q < UNROLL; q += kFoldLoads) {
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
            for (int u = q; u < q + kFoldLoads && u < UNROLL; ++u) {
                const uint32_t ws[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
                float lo[4], hi[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    lo[k] = __uint_as_float(ws[k] << 16);
                    hi[k] = __uint_as_float(ws[k] & 0xFFFF0000u);
                }
                a0 = fmaf(lo[0], lo[0], a0);
                a1 = fmaf(hi[0], hi[0], a1);
                a2 = fmaf(lo[1], lo[1], a2);
                a3 = fmaf(hi[1], hi[1], a3);
                a0 = fmaf(lo[2], lo[2], a0);
                a1 = fmaf(hi[2], hi[2], a1);
                a2 = fmaf(lo[3], lo[3], a2);
                a3 = fmaf(hi[3], hi[3], a3);
            }
            const float group_sum = (a0 + a1) + (a2 + a3);
            // A NaN or Inf element makes its group's fp32 sum non-finite; so does the square of
            // a finite value above 1.8e19, which must not raise the flag.  Only such a group
            // looks at its elements one by one (they are still in registers).
            if (!(fabsf(group_sum) <= 3.4028234e38f)) {
#pragma unroll
                for (int u = q; u < q + kFoldLoads && u < UNROLL; ++u) {
                    const uint32_t ws[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        worst = max(worst, max(ws[k] & 0x7FFFu, (ws[k] >> 16) & 0x7FFFu));
                }
            }
            sum += ((double)a0 + (double)a1) + ((double)a2 + (double)a3);
        }
    }
    // The last n % 8 elements, one lane each, in workgroup 0.
    const int64_t t = (nvec << 3) + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < 8 && t < n) {
        const uint32_t b = g[t];
        const float x = __uint_as_float(b << 16);
        sum += (double)x * (double)x;
        worst = max(worst, b & 0x7FFFu);
    }
    block_fold(sum, worst >= 0x7F80u ? 1u : 0u, partials + blockIdx.x);
}

// fp32 input, 4 elements per lane per load (4 terms in each accumulator per group).
// Requires 16-byte alignment.
template <int UNROLL>
__global__ __launch_bounds__(256) void sqnorm_f32_kernel(const float *__restrict__ g, int64_t n,
                                                         Partial *__restrict__ partials)
{
    const int64_t nvec = n >> 2;
    const f32x4 *g4 = reinterpret_cast<const f32x4 *>(g);
    double sum = 0.0;
    uint32_t worst = 0;
    const int64_t tile_vecs = 256 * UNROLL;
    const int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t first = tile * tile_vecs + threadIdx.x;
        f32x4 x[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = first + u * 256;
            x[u] = i < nvec ? __builtin_nontemporal_load(g4 + i) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int q = 0; q < UNROLL; q += kFoldLoads) {
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
            for (int u = q; u < q + kFoldLoads && u < UNROLL; ++u) {
                a0 = fmaf(x[u].x, x[u].x, a0);
                a1 = fmaf(x[u].y, x[u].y, a1);
                a2 = fmaf(x[u].z, x[u].z, a2);
                a3 = fmaf(x[u].w, x[u].w, a3);
            }
            const float group_sum = (a0 + a1) + (a2 + a3);
            if (!(fabsf(group_sum) <= 3.4028234e38f)) {   // see the bf16 kernel: only then look closer
#pragma unroll
                for (int u = q; u < q + kFoldLoads && u < UNROLL; ++u)
                    worst = max(max(worst, __float_as_uint(x[u].x) & 0x7FFFFFFFu),
                                max(__float_as_uint(x[u].y) & 0x7FFFFFFFu,
                                    max(__float_as_uint(x[u].z) & 0x7FFFFFFFu,
                                        __float_as_uint(x[u].w) & 0x7FFFFFFFu)));
            }
            sum += ((double)a0 + (double)a1) + ((double)a2 + (double)a3);
        }
    }
    const int64_t t = (nvec << 2) + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < 4 && t < n) {
        const float x = g[t];
        sum += (double)x * (double)x;
        worst = max(worst, __float_as_uint(x) & 0x7FFFFFFFu);
    }
    block_fold(sum, worst >= 0x7F800000u ? 1u : 0u, partials + blockIdx.x);
}

// Any natural alignment.
template <bool G_BF16>
__global__ __launch_bounds__(256) void sqnorm_scalar_kernel(const void *__restrict__ g, int64_t n,
                                                            Partial *__restrict__ partials)
{
    double sum = 0.0;
    uint32_t bad = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        float x;
        if constexpr (G_BF16)
            x = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(g)[i] << 16);
        else
            x = reinterpret_cast<const float *>(g)[i];
        sum += (double)x * (double)x;
        bad |= (__float_as_uint(x) & 0x7FFFFFFFu) >= 0x7F800000u ? 1u : 0u;
    }
    block_fold(sum, bad, partials + blockIdx.x);
}

// One workgroup folds `count` partials in a fixed order.  A non-finite input
// makes the sum non-finite by itself; fp32 overflow of the final value gives inf.
__global__ __launch_bounds__(256) void sqnorm_final_kernel(const Partial *__restrict__ partials,
                                                           int count, float *__restrict__ sqnorm_out,
                                                           int32_t *__restrict__ found_inf_out)
{
    double sum = 0.0;
    uint32_t bad = 0;
    for (int i = threadIdx.x; i < count; i += 256) {
        sum += partials[i].sum;
        bad |= partials[i].bad;
    }
    __shared__ Partial total;
    block_fold(sum, bad, &total);
    __syncthreads();
    if (threadIdx.x == 0) {
        *sqnorm_out = (float)total.sum;
        *found_inf_out = total.bad ? 1 : 0;
    }
}

// Workspace for the partials: one 64 KiB buffer per (device, stream), allocated on the first
// call that names that pair and kept until the process ends, so that calls enqueued on
// different streams never share partial sums.  A stream handle that is destroyed and handed
// out again simply finds its predecessor's buffer.
static zc_status partials_buffer(hipStream_t stream, Partial **out)
{
    static std::mutex mu;
    static std::map<std::pair<int, hipStream_t>, Partial *> bufs;
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_pair(dev, stream);
    auto it = bufs.find(key);
    if (it == bufs.end()) {
        hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &capturing) != hipSuccess)
            (void)hipGetLastError();
        if (capturing != hipStreamCaptureStatusNone)
            return fail(ZC_ERR_UNSUPPORTED, "the first zc_grad_sqnorm on a stream allocates its workspace: "
                                            "call it once on this stream before capturing");
        if (bufs.size() >= 1024)
            return fail(ZC_ERR_NOMEM, "more than 1024 (device, stream) pairs have called zc_grad_sqnorm");
        Partial *buf = nullptr;
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&buf), sizeof(Partial) * kMaxPartials);
        if (e != hipSuccess)
            return hip_fail(e, "hipMalloc(reduction workspace)");
        try {
            it = bufs.emplace(key, buf).first;
        } catch (const std::bad_alloc &) {
            (void)hipFree(buf);
            return fail(ZC_ERR_NOMEM, "cannot record the reduction workspace");
        }
    }
    *out = it->second;
    return ZC_OK;
}

// Argument checks shared by both entry points; nothing is enqueued here.
static zc_status check_sqnorm_args(const void *g, zc_dtype g_dtype, int64_t n, float *sqnorm_out,
                                   int32_t *found_inf_out)
{
    if (n < 0)
        return fail(ZC_ERR_INVALID_ARG, "n is negative (%lld)", (long long)n);
    if (n > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "n exceeds 2^40 elements");
    ZC_TRY(check_dtype(g_dtype));
    if (!sqnorm_out || !found_inf_out)
        return fail(ZC_ERR_INVALID_ARG, "sqnorm_out and found_inf_out must not be NULL");
    if (!aligned_to(sqnorm_out, 4) || !aligned_to(found_inf_out, 4))
        return fail(ZC_ERR_ALIGNMENT, "outputs must be 4-byte aligned");
    if (n > 0 && !g)
        return fail(ZC_ERR_INVALID_ARG, "g is NULL");
    if (n > 0 && !aligned_to(g, g_dtype == ZC_BF16 ? 2 : 4))
        return fail(ZC_ERR_ALIGNMENT, "g is not aligned to its element size");
    return ZC_OK;
}

// The two launches (partials, then the fixed-order fold) over a partials buffer of
// kMaxPartials entries.  Every workgroup overwrites its own entry and the fold reads only
// the entries written by this call, so the buffer needs no clearing between calls.
static zc_status enqueue_sqnorm(const void *g, bool bf16, int64_t n, float *sqnorm_out,
                                int32_t *found_inf_out, hipStream_t stream, Partial *partials)
{
    int cus = 0;
    ZC_TRY(num_cus(&cus));
    int blocks = 0;
    if (n > 0) {
        const Tune &t = tune();
        const int unroll = (int)t.reduce_unroll;      // 128-bit loads in flight per lane
        const int64_t per_lane = (bf16 ? 8 : 4) * unroll;
        const int64_t want = (n / per_lane + 255) / 256;
        int64_t cap = (int64_t)cus * t.reduce_blocks_per_cu;
        if (cap > kMaxPartials)
            cap = kMaxPartials;
        blocks = (int)(want < 1 ? 1 : (want > cap ? cap : want));
        if (aligned_to(g, 16)) {
#define ZC_SQNORM(KERNEL, TYPE)                                                                          \
    do {                                                                                                 \
        if (unroll == 2)                                                                                 \
            hipLaunchKernelGGL(KERNEL<2>, dim3(blocks), dim3(256), 0, stream, static_cast<const TYPE *>(g), n, partials); \
        else if (unroll == 8)                                                                            \
            hipLaunchKernelGGL(KERNEL<8>, dim3(blocks), dim3(256), 0, stream, static_cast<const TYPE *>(g), n, partials); \
        else                                                                                             \
            hipLaunchKernelGGL(KERNEL<4>, dim3(blocks), dim3(256), 0, stream, static_cast<const TYPE *>(g), n, partials); \
    } while (0)
            if (bf16)
                ZC_SQNORM(sqnorm_bf16_kernel, uint16_t);
            else
                ZC_SQNORM(sqnorm_f32_kernel, float);
#undef ZC_SQNORM
        } else {
            if (bf16)
                hipLaunchKernelGGL(sqnorm_scalar_kernel<true>, dim3(blocks), dim3(256), 0, stream, g, n,
                                   partials);
            else
                hipLaunchKernelGGL(sqnorm_scalar_kernel<false>, dim3(blocks), dim3(256), 0, stream, g, n,
                                   partials);
        }
        ZC_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(sqnorm_final_kernel, dim3(1), dim3(256), 0, stream, partials, blocks, sqnorm_out,
                       found_inf_out);
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

// Partials buffer of zc_grad_sqnorm_static: one fixed array in the library's device image,
// so that entry point never allocates.  Every GPU the library runs on holds its own copy at
// its own address; host code must use the address hipGetSymbolAddress returns for the
// current device, never the symbol itself.
static __device__ __align__(256) unsigned char scratch[sizeof(Partial) * kMaxPartials];

static zc_status static_partials(Partial **out)
{
    static std::mutex mu;
    static Partial *ptr_of_device[64];
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64)
        return fail(ZC_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {
        void *ptr = nullptr;
        ZC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr)
            return fail(ZC_ERR_HIP, "hipGetSymbolAddress gave no address for the static partials buffer");
        ptr_of_device[dev] = static_cast<Partial *>(ptr);
    }
    *out = ptr_of_device[dev];
    return ZC_OK;
}

}  // namespace zc

extern "C" zc_status zc_grad_sqnorm(const void *g, zc_dtype g_dtype, int64_t n, float *sqnorm_out,
                                    int32_t *found_inf_out, void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_sqnorm_args(g, g_dtype, n, sqnorm_out, found_inf_out));
    hipStream_t stream = (hipStream_t)hip_stream;
    Partial *partials = nullptr;
    ZC_TRY(partials_buffer(stream, &partials));
    return enqueue_sqnorm(g, g_dtype == ZC_BF16, n, sqnorm_out, found_inf_out, stream, partials);
}

extern "C" zc_status zc_grad_sqnorm_static(const void *g, zc_dtype g_dtype, int64_t n, float *sqnorm_out,
                                           int32_t *found_inf_out, void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_sqnorm_args(g, g_dtype, n, sqnorm_out, found_inf_out));
    Partial *partials = nullptr;
    ZC_TRY(static_partials(&partials));
    return enqueue_sqnorm(g, g_dtype == ZC_BF16, n, sqnorm_out, found_inf_out, (hipStream_t)hip_stream,
                          partials);
}

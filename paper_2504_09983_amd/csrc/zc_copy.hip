// Standalone fp32 -> bf16 cast and the segmented unshard copy.
//
// Both are pure streaming kernels (6 and 4 bytes per element, no reuse), built
// on 128-bit accesses with a wave touching contiguous 1 KiB (fp32 / bf16 body)
// per instruction.  Workgroups are single waves that each own one small tile and
// are dispatched in tile order; the number of resident waves per CU is capped
// (unused dynamic LDS) because on MI355X a mixed read/write stream loses
// bandwidth when too many DRAM pages are open at once.  Loads are non-temporal,
// stores are written through the L2 at once (stream_out_rsrc in zc_internal.h).
#include <algorithm>
#include <new>
#include <utility>
#include <vector>

#include "zc_internal.h"

namespace zc {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT, typename T>
__device__ __forceinline__ T ldc(const T *ptr)
{
    if constexpr (NT)
        return __builtin_nontemporal_load(ptr);
    else
        return *ptr;
}

template <bool NT, typename T>
__device__ __forceinline__ void stc(T *ptr, T val)
{
    if constexpr (NT)
        __builtin_nontemporal_store(val, ptr);
    else
        *ptr = val;
}

// Round-to-nearest-even fp32 -> bf16 bits; NaN kept (quiet bit set); no flush.
__device__ __forceinline__ uint32_t cast_rne(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x40u;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? quiet : rounded;
}

constexpr int kCopyBlock = 64;  // one wave per workgroup: finest dispatch granularity
constexpr int kCastRows = 4;    // 4 x 256 elements per workgroup tile

// Requires src 16-byte and dst 8-byte aligned.  One tile per workgroup; `tile0`
// is the tile of workgroup 0 (launches are cut to keep the grid below 2^31).
// NT: 0 = ordinary accesses, 1 = non-temporal loads and stores, 2 = non-temporal loads and
// write-through streaming stores (stream_out_rsrc).
template <int NT>
__global__ __launch_bounds__(kCopyBlock) void cast_vec_kernel(const float *__restrict__ src,
                                                              uint16_t *__restrict__ dst, int64_t n,
                                                              int64_t tile0)
{
    const int64_t nvec = n >> 2;
    const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src);
    u32x2 *d2 = reinterpret_cast<u32x2 *>(dst);
    const int64_t tile = tile0 + blockIdx.x;
    const int64_t first = tile * (kCopyBlock * kCastRows) + threadIdx.x;
    f32x4 x[kCastRows];
#pragma unroll
    for (int r = 0; r < kCastRows; ++r) {
        const int64_t i = first + r * kCopyBlock;
        if (i < nvec)
            x[r] = ldc<(NT != 0)>(s4 + i);
    }
    const int64_t tile_first = tile * (kCopyBlock * kCastRows);
    int64_t room = nvec - tile_first;
    room = room < 0 ? 0 : (room > kCopyBlock * kCastRows ? kCopyBlock * kCastRows : room);
    const __amdgpu_buffer_rsrc_t rd = stream_out_rsrc(d2 + tile_first, room * 8);
#pragma unroll
    for (int r = 0; r < kCastRows; ++r) {
        const int64_t i = first + r * kCopyBlock;
        if (i < nvec) {
            u32x2 w;
            w.x = cast_rne(x[r].x) | (cast_rne(x[r].y) << 16);
            w.y = cast_rne(x[r].z) | (cast_rne(x[r].w) << 16);
            if constexpr (NT == 2) {
                stream_u32x2 o;
                o[0] = w.x;
                o[1] = w.y;
                __builtin_amdgcn_raw_buffer_store_b64(o, rd, (int)(threadIdx.x + r * kCopyBlock) * 8, 0, kAuxStreamOut);
            } else {
                stc<(NT != 0)>(d2 + i, w);
            }
        }
    }
    const int64_t i = (nvec << 2) + threadIdx.x;
    if (tile == 0 && threadIdx.x < 4 && i < n)
        dst[i] = (uint16_t)cast_rne(src[i]);
}

__global__ __launch_bounds__(256) void cast_scalar_kernel(const float *__restrict__ src,
                                                          uint16_t *__restrict__ dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        dst[i] = (uint16_t)cast_rne(src[i]);
}

// ---------------------------------------------------------------------------
// Unshard.  A segment is cut into tiles of kTileVecs 16-byte vectors of its
// destination-aligned body; the first tile of a segment also copies the (< 8
// element) unaligned head and tail.  Workgroups find their segment by binary
// search over the prefix sum of tiles per segment.
// ---------------------------------------------------------------------------

constexpr int64_t kTileVecs = 256;  // 4 KiB per tile
constexpr int kUnroll = 4;          // kTileVecs / kCopyBlock threads

struct SegDesc {
    int64_t src_offset;
    uint16_t *dst;
    int64_t numel;
    int64_t first_tile;
};

// align_class: 0 = source 16-byte aligned, 1 = 4-byte aligned, 2 = 2-byte aligned.
template <int ALIGN, bool NT>
__device__ __forceinline__ u32x4 load_src_vec(const uint16_t *s)
{
    u32x4 w;
    if constexpr (ALIGN == 0) {
        const u32x4 *q = reinterpret_cast<const u32x4 *>(s);
        if constexpr (NT)
            w = __builtin_nontemporal_load(q);
        else
            w = *q;
    } else if constexpr (ALIGN == 1) {
        const uint32_t *q = reinterpret_cast<const uint32_t *>(s);
        w.x = q[0];
        w.y = q[1];
        w.z = q[2];
        w.w = q[3];
    } else {
        w.x = (uint32_t)s[0] | ((uint32_t)s[1] << 16);
        w.y = (uint32_t)s[2] | ((uint32_t)s[3] << 16);
        w.z = (uint32_t)s[4] | ((uint32_t)s[5] << 16);
        w.w = (uint32_t)s[6] | ((uint32_t)s[7] << 16);
    }
    return w;
}

// One tile of the aligned body: every load of the tile is issued before the first store.
// The alignment class is the same for the whole wave, so the caller branches once and the
// loads of a tile issue back to back (with the class tested per load the compiler waited
// after each of them).  The per-vector bounds test stays on full tiles as well: a variant
// without it measured 2.7 % slower.
template <int ALIGN, int NT>
__device__ __forceinline__ void copy_tile(const uint16_t *sb, u32x4 *db, int64_t t, int64_t body_vecs)
{
    const int64_t first = t * kTileVecs + threadIdx.x;
    u32x4 w[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
        const int64_t i = first + k * kCopyBlock;
        if (i < body_vecs)
            w[k] = load_src_vec<ALIGN, (NT != 0)>(sb + (i << 3));
    }
    int64_t room = body_vecs - t * kTileVecs;      // uniform: the segment and its tile are per workgroup
    room = room < 0 ? 0 : (room > kTileVecs ? kTileVecs : room);
    const __amdgpu_buffer_rsrc_t rd = stream_out_rsrc(db + t * kTileVecs, room * 16);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
        const int64_t i = first + k * kCopyBlock;
        if (i < body_vecs) {
            if constexpr (NT == 2) {
                stream_u32x4 o;
                o[0] = w[k].x;
                o[1] = w[k].y;
                o[2] = w[k].z;
                o[3] = w[k].w;
                __builtin_amdgcn_raw_buffer_store_b128(o, rd, (int)(threadIdx.x + k * kCopyBlock) * 16, 0, kAuxStreamOut);
            } else {
                stc<(NT != 0)>(db + i, w[k]);
            }
        }
    }
}

constexpr int kHintShift = 10;  // one hint per 1024 tiles

// `hint[k]` is the segment that owns tile k << kHintShift, so the search for a
// tile's segment starts in a range that is almost always a single segment: one
// dependent load instead of log2(nsegs) of them before the wave can issue its copy.
template <int NT>
__global__ __launch_bounds__(kCopyBlock) void unshard_kernel(const uint16_t *__restrict__ gathered,
                                                             const SegDesc *__restrict__ segs,
                                                             const int32_t *__restrict__ hint,
                                                             int64_t nsegs, int64_t tile0)
{
    const int64_t tile = tile0 + blockIdx.x;
    {
        // Largest s with segs[s].first_tile <= tile (empty segments share their
        // successor's first_tile and are skipped by taking the last match).
        const int64_t grp = tile >> kHintShift;
        int64_t lo = hint[grp], hi = (int64_t)hint[grp + 1] + 1;
        if (hi > nsegs)
            hi = nsegs;
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (segs[mid].first_tile <= tile)
                lo = mid;
            else
                hi = mid;
        }
        const SegDesc d = segs[lo];
        const int64_t t = tile - d.first_tile;
        const uint16_t *src = gathered + d.src_offset;
        uint16_t *dst = d.dst;
        const int64_t n = d.numel;

        int64_t head = (int64_t)(((16u - (unsigned)(reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u) >> 1);
        if (head > n)
            head = n;
        const int64_t body_vecs = (n - head) >> 3;
        const int64_t tail = n - head - (body_vecs << 3);

        if (t == 0) {
            if ((int64_t)threadIdx.x < head)
                dst[threadIdx.x] = src[threadIdx.x];
            const int64_t tail_at = head + (body_vecs << 3);
            if ((int64_t)threadIdx.x < tail)
                dst[tail_at + threadIdx.x] = src[tail_at + threadIdx.x];
        }

        const uint16_t *sb = src + head;
        u32x4 *db = reinterpret_cast<u32x4 *>(dst + head);
        const uintptr_t sa = reinterpret_cast<uintptr_t>(sb);
        if ((sa & 15u) == 0)
            copy_tile<0, NT>(sb, db, t, body_vecs);
        else if ((sa & 3u) == 0)
            copy_tile<1, NT>(sb, db, t, body_vecs);
        else
            copy_tile<2, NT>(sb, db, t, body_vecs);
    }
}

}  // namespace zc

struct zc_unshard_plan {
    std::vector<std::pair<uintptr_t, uintptr_t>> dst_ranges;  // [lo, hi) of every non-empty destination, sorted
    zc::SegDesc *segs_dev = nullptr;
    int32_t *hint_dev = nullptr;
    int64_t nsegs = 0;
    int64_t ntiles = 0;
    int64_t gathered_numel = 0;
    int device = 0;
};

extern "C" {

zc_status zc_cast_bf16(const float *src, uint16_t *dst, int64_t n, void *hip_stream)
{
    using namespace zc;
    if (n < 0)
        return fail(ZC_ERR_INVALID_ARG, "n is negative (%lld)", (long long)n);
    if (n > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "n exceeds 2^40 elements");
    if (n == 0)
        return ZC_OK;
    if (!src || !dst)
        return fail(ZC_ERR_INVALID_ARG, "src and dst must not be NULL when n > 0");
    if (!aligned_to(src, 4))
        return fail(ZC_ERR_ALIGNMENT, "src must be 4-byte aligned");
    if (!aligned_to(dst, 2))
        return fail(ZC_ERR_ALIGNMENT, "dst must be 2-byte aligned");
    const uintptr_t s0 = (uintptr_t)src, d0 = (uintptr_t)dst;
    if (s0 < d0 + 2 * (uintptr_t)n && d0 < s0 + 4 * (uintptr_t)n)
        return fail(ZC_ERR_INVALID_ARG, "src and dst overlap");
    hipStream_t stream = (hipStream_t)hip_stream;
    int cus = 0;
    ZC_TRY(num_cus(&cus));
    const Tune &t = tune();
    if (aligned_to(src, 16) && aligned_to(dst, 8)) {
        const int64_t nvec = n >> 2;
        const int64_t tile_vecs = kCopyBlock * kCastRows;
        int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;
        if (ntiles == 0)
            ntiles = 1;  // workgroup 0 also owns the n % 4 tail
        size_t lds = 0;
        ZC_TRY(occupancy_cap_lds((int)t.cast_waves_per_cu, kCopyBlock, &lds));
        const int64_t kMaxGrid = max_workgroups_per_launch(t.launch_max_grid, kCopyBlock);
        for (int64_t tile0 = 0; tile0 < ntiles; tile0 += kMaxGrid) {
            const int64_t count = (ntiles - tile0) < kMaxGrid ? (ntiles - tile0) : kMaxGrid;
            if (t.copy_nontemporal == 2)
                hipLaunchKernelGGL(cast_vec_kernel<2>, dim3((unsigned)count), dim3(kCopyBlock), lds,
                                   stream, src, dst, n, tile0);
            else if (t.copy_nontemporal == 1)
                hipLaunchKernelGGL(cast_vec_kernel<1>, dim3((unsigned)count), dim3(kCopyBlock), lds,
                                   stream, src, dst, n, tile0);
            else
                hipLaunchKernelGGL(cast_vec_kernel<0>, dim3((unsigned)count), dim3(kCopyBlock), lds,
                                   stream, src, dst, n, tile0);
        }
    } else {
        int64_t blocks = (n + 255) / 256;
        if (blocks > (int64_t)cus * 32)
            blocks = (int64_t)cus * 32;
        hipLaunchKernelGGL(cast_scalar_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, dst, n);
    }
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

zc_status zc_unshard_plan_create(const zc_segment *segs, int64_t nsegs, int64_t gathered_numel,
                                 zc_unshard_plan **out)
{
    using namespace zc;
    if (!out)
        return fail(ZC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (nsegs < 0 || gathered_numel < 0)
        return fail(ZC_ERR_INVALID_ARG, "nsegs and gathered_numel must be >= 0");
    if (nsegs > 0 && !segs)
        return fail(ZC_ERR_INVALID_ARG, "segs is NULL");
    if (gathered_numel > kMaxElements * 64)
        return fail(ZC_ERR_UNSUPPORTED, "gathered buffer exceeds 2^46 elements");
    if (nsegs > 0x7FFFFFFF)
        return fail(ZC_ERR_UNSUPPORTED, "more than 2^31 segments");

    std::vector<SegDesc> table;
    try {
        table.reserve((size_t)nsegs);
    } catch (const std::bad_alloc &) {
        return fail(ZC_ERR_NOMEM, "cannot allocate the host segment table");
    }
    int64_t ntiles = 0;
    for (int64_t s = 0; s < nsegs; ++s) {
        const zc_segment &g = segs[s];
        if (g.numel < 0 || g.src_offset < 0)
            return fail(ZC_ERR_INVALID_ARG, "segment %lld: negative offset or size", (long long)s);
        if (g.numel > gathered_numel || g.src_offset > gathered_numel - g.numel)
            return fail(ZC_ERR_INVALID_ARG, "segment %lld: [%lld, +%lld) leaves the gathered buffer of %lld",
                        (long long)s, (long long)g.src_offset, (long long)g.numel,
                        (long long)gathered_numel);
        if (g.numel > 0 && !g.dst)
            return fail(ZC_ERR_INVALID_ARG, "segment %lld: dst is NULL", (long long)s);
        if (g.numel > 0 && !aligned_to(g.dst, 2))
            return fail(ZC_ERR_ALIGNMENT, "segment %lld: dst must be 2-byte aligned", (long long)s);
        SegDesc d;
        d.src_offset = g.src_offset;
        d.dst = static_cast<uint16_t *>(g.dst);
        d.numel = g.numel;
        d.first_tile = ntiles;
        if (g.numel > 0) {
            int64_t head = (int64_t)(((16u - (unsigned)((uintptr_t)g.dst & 15u)) & 15u) >> 1);
            if (head > g.numel)
                head = g.numel;
            const int64_t body_vecs = (g.numel - head) >> 3;
            const int64_t tiles = (body_vecs + kTileVecs - 1) / kTileVecs;
            ntiles += tiles > 0 ? tiles : 1;  // head / tail need a tile even with no body
        }
        table.push_back(d);
    }

    // Destinations must not overlap each other: sort their byte ranges and compare neighbours.
    std::vector<std::pair<uintptr_t, uintptr_t>> ranges;
    try {
        ranges.reserve(table.size());
        for (const SegDesc &d : table)
            if (d.numel > 0)
                ranges.emplace_back(reinterpret_cast<uintptr_t>(d.dst),
                                    reinterpret_cast<uintptr_t>(d.dst) + 2 * (uintptr_t)d.numel);
    } catch (const std::bad_alloc &) {
        return fail(ZC_ERR_NOMEM, "cannot allocate the destination range table");
    }
    std::sort(ranges.begin(), ranges.end());
    for (size_t k = 1; k < ranges.size(); ++k)
        if (ranges[k].first < ranges[k - 1].second)
            return fail(ZC_ERR_INVALID_ARG, "two destinations overlap (bytes [%#llx, %#llx) and [%#llx, %#llx))",
                        (unsigned long long)ranges[k - 1].first, (unsigned long long)ranges[k - 1].second,
                        (unsigned long long)ranges[k].first, (unsigned long long)ranges[k].second);

    // hint[k] = last segment whose first tile is <= k << kHintShift, for k = 0 .. groups
    const int64_t groups = (ntiles >> kHintShift) + 1;
    std::vector<int32_t> hints;
    try {
        hints.resize((size_t)groups + 1);
    } catch (const std::bad_alloc &) {
        return fail(ZC_ERR_NOMEM, "cannot allocate the host hint table");
    }
    {
        int64_t seg = 0;
        for (int64_t k = 0; k <= groups; ++k) {
            const int64_t tile = k << kHintShift;
            while (seg + 1 < nsegs && table[(size_t)seg + 1].first_tile <= tile)
                ++seg;
            hints[(size_t)k] = (int32_t)seg;
        }
    }

    zc_unshard_plan *plan = new (std::nothrow) zc_unshard_plan;
    if (!plan)
        return fail(ZC_ERR_NOMEM, "cannot allocate the plan");
    plan->dst_ranges.swap(ranges);
    plan->nsegs = nsegs;
    plan->ntiles = ntiles;
    plan->gathered_numel = gathered_numel;
    hipError_t e = hipGetDevice(&plan->device);
    if (e == hipSuccess && nsegs > 0) {
        e = hipMalloc(reinterpret_cast<void **>(&plan->segs_dev), sizeof(SegDesc) * (size_t)nsegs);
        if (e == hipSuccess)
            e = hipMemcpy(plan->segs_dev, table.data(), sizeof(SegDesc) * (size_t)nsegs,
                          hipMemcpyHostToDevice);
        if (e == hipSuccess)
            e = hipMalloc(reinterpret_cast<void **>(&plan->hint_dev), sizeof(int32_t) * hints.size());
        if (e == hipSuccess)
            e = hipMemcpy(plan->hint_dev, hints.data(), sizeof(int32_t) * hints.size(),
                          hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        if (plan->hint_dev)
            (void)hipFree(plan->hint_dev);
        if (plan->segs_dev)
            (void)hipFree(plan->segs_dev);
        delete plan;
        return hip_fail(e, "uploading the unshard descriptor table");
    }
    *out = plan;
    return ZC_OK;
}

zc_status zc_unshard(const zc_unshard_plan *plan, const uint16_t *gathered, void *hip_stream)
{
    using namespace zc;
    if (!plan)
        return fail(ZC_ERR_INVALID_ARG, "plan is NULL");
    if (plan->ntiles == 0)
        return ZC_OK;
    if (!gathered)
        return fail(ZC_ERR_INVALID_ARG, "gathered is NULL");
    if (!aligned_to(gathered, 2))
        return fail(ZC_ERR_ALIGNMENT, "gathered must be 2-byte aligned");
    {
        // The gathered buffer must not overlap any destination: find the first destination
        // that ends behind its start and see whether it begins before its end.
        const uintptr_t lo = reinterpret_cast<uintptr_t>(gathered);
        const uintptr_t hi = lo + 2 * (uintptr_t)plan->gathered_numel;
        auto it = std::upper_bound(plan->dst_ranges.begin(), plan->dst_ranges.end(), lo,
                                   [](uintptr_t v, const std::pair<uintptr_t, uintptr_t> &r) { return v < r.second; });
        if (it != plan->dst_ranges.end() && it->first < hi)
            return fail(ZC_ERR_INVALID_ARG, "the gathered buffer overlaps a destination");
    }
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev != plan->device)
        return fail(ZC_ERR_INVALID_ARG, "plan was created on device %d, current device is %d",
                    plan->device, dev);
    const Tune &t = tune();
    size_t lds = 0;
    ZC_TRY(occupancy_cap_lds((int)t.copy_waves_per_cu, kCopyBlock, &lds));
    const int64_t kMaxGrid = max_workgroups_per_launch(t.launch_max_grid, kCopyBlock);
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int64_t tile0 = 0; tile0 < plan->ntiles; tile0 += kMaxGrid) {
        const int64_t left = plan->ntiles - tile0;
        const int64_t count = left < kMaxGrid ? left : kMaxGrid;
        if (t.copy_nontemporal == 2)
            hipLaunchKernelGGL(unshard_kernel<2>, dim3((unsigned)count), dim3(kCopyBlock), lds, stream,
                               gathered, plan->segs_dev, plan->hint_dev, plan->nsegs, tile0);
        else if (t.copy_nontemporal == 1)
            hipLaunchKernelGGL(unshard_kernel<1>, dim3((unsigned)count), dim3(kCopyBlock), lds, stream,
                               gathered, plan->segs_dev, plan->hint_dev, plan->nsegs, tile0);
        else
            hipLaunchKernelGGL(unshard_kernel<0>, dim3((unsigned)count), dim3(kCopyBlock), lds, stream,
                               gathered, plan->segs_dev, plan->hint_dev, plan->nsegs, tile0);
    }
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

zc_status zc_unshard_plan_destroy(zc_unshard_plan *plan)
{
    using namespace zc;
    if (!plan)
        return ZC_OK;
    hipError_t e = hipSuccess;
    if (plan->hint_dev)
        e = hipFree(plan->hint_dev);
    if (plan->segs_dev) {
        const hipError_t e2 = hipFree(plan->segs_dev);
        if (e == hipSuccess)
            e = e2;
    }
    delete plan;
    if (e != hipSuccess)
        return hip_fail(e, "hipFree(descriptor table)");
    return ZC_OK;
}

}  // extern "C"

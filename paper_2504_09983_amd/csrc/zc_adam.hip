// Fused Adam / AdamW update (+ optional bf16 copy) over a flat fp32 partition.
//
// One streaming pass: every element's p, m, v (fp32) and g (fp32 or bf16) is
// read once and p, m, v (+ bf16 p) written once.  Nothing is reused, nothing is
// a contraction, so the kernel is HBM-bound and built around 128-bit accesses:
// a wave reads one contiguous 1 KiB row per instruction (lane l owns elements
// 4l..4l+3 of the row), a workgroup owns ROWS rows of 4*BLOCK elements, and
// all loads of a tile are issued before any arithmetic.  Measured on MI355X the
// mixed read/write stream runs fastest with one-wave workgroups of one row,
// dispatched in tile order, and only ~12 waves resident per CU; more waves in
// flight widen the window of DRAM pages touched at once and cost bandwidth.  The
// resident-wave count is capped by asking for a slice of LDS that is never used.
// Loads are non-temporal; stores are written through the L2 at once (buffer
// stores with the nt and sc1 bits), so that a tile's results reach DRAM together
// instead of whenever the cache evicts them.
//
// p, m and v come either as three arrays or as one packed state array in which granules
// of 8192 elements of p, m and v follow each other (zc_adam_step_packed): the same kernel
// with one more index computation per lane.  The resident waves then work on one contiguous
// stretch of state instead of three that lie gigabytes apart, which measured 2-4 % faster.
//
// The arithmetic (paper: Adam with momentum and variance buffers in fp32 next
// to fp32 master parameters; Experimental settings, Adaptive offloading) is
// bias-corrected Adam with epsilon outside the square root and, in ZC_ADAMW
// mode, decoupled weight decay applied to the old parameter.  It is hidden
// behind the memory traffic, so the default evaluates it in fp64.
#include <cmath>

#include "zc_internal.h"

namespace zc {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct AdamScalars {
    double b1, omb1, b2, omb2, step_size, inv_sqrt_bc2, eps, decay, wd, gscale;
    float b1f, omb1f, b2f, omb2f, step_sizef, inv_sqrt_bc2f, epsf, lrwdf, wdf, gscalef;
    int l2;
};

// Device-resident controls read at execution time: a skip flag (overflowed step) and
// an extra gradient scale (clipping coefficient / loss-scale removal computed on the GPU).
struct DevCtl {
    const int32_t *skip;
    const float *gscale;
};

// Packed state (zc_adam_step_packed): p, m and v of one partition interleaved in granules of
// ZC_PACKED_GRANULE elements, [p granule 0][m granule 0][v granule 0][p granule 1]...  Element e
// of p sits at state[packed_at(e)], its m one granule and its v two granules behind it.
constexpr int kGranuleShift = 13;
constexpr int64_t kGranule = int64_t(1) << kGranuleShift;
constexpr int64_t kGranuleVecs = kGranule / 4;
static_assert(kGranule == ZC_PACKED_GRANULE, "the header and the kernels must agree on the granule");

__host__ __device__ __forceinline__ int64_t packed_at(int64_t e)
{
    return e + ((e >> kGranuleShift) << (kGranuleShift + 1));
}
// the same for an index in 16-byte vectors
__host__ __device__ __forceinline__ int64_t packed_vec_at(int64_t gv)
{
    return gv + ((gv >> (kGranuleShift - 2)) << (kGranuleShift - 1));
}

static AdamScalars make_scalars(const zc_adam_hparams *hp)
{
    AdamScalars s;
    const double lr = hp->lr, b1 = hp->beta1, b2 = hp->beta2, wd = hp->weight_decay;
    const double t = (double)hp->step;
    const double bc1 = 1.0 - std::pow(b1, t);
    const double bc2 = 1.0 - std::pow(b2, t);
    s.b1 = b1;
    s.omb1 = 1.0 - b1;
    s.b2 = b2;
    s.omb2 = 1.0 - b2;
    s.step_size = lr / bc1;
    s.inv_sqrt_bc2 = 1.0 / std::sqrt(bc2);
    s.eps = hp->eps;
    s.decay = 1.0 - lr * wd;
    s.wd = wd;
    s.gscale = hp->grad_scale;
    s.b1f = (float)s.b1;
    s.omb1f = (float)s.omb1;
    s.b2f = (float)s.b2;
    s.omb2f = (float)s.omb2;
    s.step_sizef = (float)s.step_size;
    s.inv_sqrt_bc2f = (float)s.inv_sqrt_bc2;
    s.epsf = (float)s.eps;
    s.lrwdf = (float)(lr * wd);
    s.wdf = (float)wd;
    s.gscalef = (float)s.gscale;
    s.l2 = hp->mode == ZC_ADAM_L2;
    return s;
}

// ARITH 0: fp32 throughout (fused multiply-adds, correctly rounded sqrt / div).
// ARITH 1: multiply-adds in fp64 (full rate on gfx950), sqrt and divide in fp32.
// ARITH 2 (default): fp64 throughout; m and v as unfused IEEE double expressions.
template <int ARITH>
__device__ __forceinline__ void adam_elem(float &p, float &m, float &v, float g, const AdamScalars &s)
{
    if constexpr (ARITH == 0) {
        float gf = g * s.gscalef;
        if (s.l2)
            gf = fmaf(s.wdf, p, gf);
        const float mn = fmaf(s.omb1f, gf, s.b1f * m);
        const float vn = fmaf(s.omb2f * gf, gf, s.b2f * v);
        const float denom = fmaf(sqrtf(vn), s.inv_sqrt_bc2f, s.epsf);
        const float upd = mn / denom;
        // p*(1 - lr*wd) evaluated as p - (lr*wd)*p: the tiny factor keeps its
        // relative accuracy, which (1 - lr*wd) rounded to fp32 would not.
        const float pd = s.l2 ? p : fmaf(-s.lrwdf, p, p);
        p = fmaf(-s.step_sizef, upd, pd);
        m = mn;
        v = vn;
    } else if constexpr (ARITH == 1) {
        double gd = (double)g * s.gscale;
        if (s.l2)
            gd = fma(s.wd, (double)p, gd);
        const float mn = (float)fma(s.omb1, gd, s.b1 * (double)m);
        const float vn = (float)fma(s.omb2 * gd, gd, s.b2 * (double)v);
        const double pd = s.l2 ? (double)p : (double)p * s.decay;
        const float denom = fmaf(sqrtf(vn), s.inv_sqrt_bc2f, s.epsf);
        const float upd = mn / denom;
        p = (float)fma(-s.step_size, (double)upd, pd);
        m = mn;
        v = vn;
    } else {
        // The definition evaluated in IEEE double, every product and sum rounded on its
        // own (contraction into fused multiply-adds is switched off for this block), then
        // one rounding to fp32 per stored value:
        //   m = b1*m + (1-b1)*g,  v = b2*v + ((1-b2)*g)*g
        // so m and v reproduce bit for bit on any IEEE machine that evaluates the same
        // expression in double.
        float mn, vn;
        {
#pragma clang fp contract(off)
            double gd = (double)g * s.gscale;
            if (s.l2) {
                const double wp = s.wd * (double)p;
                gd = gd + wp;
            }
            const double m_keep = s.b1 * (double)m;
            const double m_add = s.omb1 * gd;
            mn = (float)(m_keep + m_add);
            const double v_keep = s.b2 * (double)v;
            const double v_add = (s.omb2 * gd) * gd;
            vn = (float)(v_keep + v_add);
        }
        const double pd = s.l2 ? (double)p : (double)p * s.decay;
        const double denom = fma(sqrt((double)vn), s.inv_sqrt_bc2, s.eps);
        p = (float)(pd - s.step_size * (double)mn / denom);
        m = mn;
        v = vn;
    }
}

// fp32 -> bf16 bits, round-to-nearest-even, NaN kept quiet, no flush.
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x40u;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? quiet : rounded;
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *ptr)
{
    if constexpr (NT)
        return __builtin_nontemporal_load(ptr);
    else
        return *ptr;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(T *ptr, T val)
{
    if constexpr (NT)
        __builtin_nontemporal_store(val, ptr);
    else
        *ptr = val;
}

// NT: 0 = ordinary loads and stores, 1 = both non-temporal, 2 = loads only, 3 = stores only,
// 4 = non-temporal loads and write-through streaming stores (stream_out_rsrc, zc_internal.h).
// PACKED: p4 == po4 is the packed state array (m4, v4, mo4, vo4 unused) and gv0 the index, in
// vectors of the flat partition, of the stretch's first element; g and out2 stay flat.  A tile
// may straddle a granule boundary (a stretch can start anywhere), so every lane maps its own
// vector and the store descriptors span the tile's first to its last packed vector.
template <int ROWS, int BLOCK, bool G_BF16, int NT, int ARITH, bool GUARD, bool PACKED = false>
__device__ __forceinline__ void adam_tile(const f32x4 *p4, const f32x4 *m4, const f32x4 *v4,
                                          f32x4 *po4, f32x4 *mo4, f32x4 *vo4,
                                          const void *__restrict__ g, u32x2 *__restrict__ out2,
                                          int64_t first, int64_t nvec, const AdamScalars &s_in, DevCtl ctl,
                                          int64_t gv0 = 0)
{
    // The skip flag and the device-side scale are fetched together with the data and only
    // used after the tile's loads have been issued, so their latency hides behind them.
    const int32_t skip_now = ctl.skip ? *ctl.skip : 0;
    const float dev_scale = ctl.gscale ? *ctl.gscale : 1.0f;
    constexpr bool NTL = NT == 1 || NT == 2 || NT == 4, NTS = NT == 1 || NT == 3;
    // mode 4: one descriptor per output array over this workgroup's tile (uniform values)
    typedef stream_u32x4 u32x4v;
    typedef stream_u32x2 u32x2v;
    constexpr int64_t kTileVecs = (int64_t)BLOCK * ROWS;
    const int64_t tile_first = first - threadIdx.x;
    f32x4 pv[ROWS], mv[ROWS], vv[ROWS], gv[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int64_t i = first + (int64_t)r * BLOCK;
        if (!GUARD || i < nvec) {
            if constexpr (PACKED) {
                const f32x4 *at = p4 + packed_vec_at(gv0 + i);
                pv[r] = ld<NTL>(at);
                mv[r] = ld<NTL>(at + kGranuleVecs);
                vv[r] = ld<NTL>(at + 2 * kGranuleVecs);
            } else {
                pv[r] = ld<NTL>(p4 + i);
                mv[r] = ld<NTL>(m4 + i);
                vv[r] = ld<NTL>(v4 + i);
            }
            if constexpr (G_BF16) {
                const u32x2 w = ld<NTL>(reinterpret_cast<const u32x2 *>(g) + i);
                gv[r].x = __uint_as_float(w.x << 16);
                gv[r].y = __uint_as_float(w.x & 0xFFFF0000u);
                gv[r].z = __uint_as_float(w.y << 16);
                gv[r].w = __uint_as_float(w.y & 0xFFFF0000u);
            } else {
                gv[r] = ld<NTL>(reinterpret_cast<const f32x4 *>(g) + i);
            }
        }
    }
    // Store descriptors (mode 4) are set up after the loads have been issued: the scalar work
    // must not stand between a wave's start and its first load (it did, ~50 instructions, when
    // it was written first; the fence keeps the compiler from hoisting it back).
    if constexpr (ROWS == 1)
        __builtin_amdgcn_sched_barrier(0);
    __amdgpu_buffer_rsrc_t rp, rm, rv, ro;
    int64_t packed_first = 0;                        // packed vector index of the tile's first vector
    if constexpr (NT == 4) {
        int64_t vecs = kTileVecs;                    // whole 16-byte vectors this tile may write
        if constexpr (GUARD) {
            vecs = nvec - tile_first;
            vecs = vecs < 0 ? 0 : (vecs > kTileVecs ? kTileVecs : vecs);
        }
        if constexpr (PACKED) {
            packed_first = packed_vec_at(gv0 + tile_first);
            const int64_t span = vecs > 0 ? packed_vec_at(gv0 + tile_first + vecs - 1) - packed_first + 1 : 0;
            rp = stream_out_rsrc(po4 + packed_first, span * 16);
            rm = stream_out_rsrc(po4 + packed_first + kGranuleVecs, span * 16);
            rv = stream_out_rsrc(po4 + packed_first + 2 * kGranuleVecs, span * 16);
        } else {
            rp = stream_out_rsrc(po4 + tile_first, vecs * 16);
            rm = stream_out_rsrc(mo4 + tile_first, vecs * 16);
            rv = stream_out_rsrc(vo4 + tile_first, vecs * 16);
        }
        ro = stream_out_rsrc(out2 ? (void *)(out2 + tile_first) : (void *)po4, out2 ? vecs * 8 : 0);
    }
    if (skip_now != 0)
        return;
    AdamScalars s = s_in;
    if (ctl.gscale) {
        s.gscalef = s_in.gscalef * dev_scale;  // one fp32 product, the same in every variant
        s.gscale = (double)s.gscalef;
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int64_t i = first + (int64_t)r * BLOCK;
        if (!GUARD || i < nvec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float pe = pv[r][k], me = mv[r][k], ve = vv[r][k];
                adam_elem<ARITH>(pe, me, ve, gv[r][k], s);
                pv[r][k] = pe;
                mv[r][k] = me;
                vv[r][k] = ve;
            }
            if constexpr (NT == 4) {
                const int voff = (int)(threadIdx.x + r * BLOCK) * 16;
                const int soff = PACKED ? (int)(packed_vec_at(gv0 + i) - packed_first) * 16 : voff;
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4v, pv[r]), rp, soff, 0, kAuxStreamOut);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4v, mv[r]), rm, soff, 0, kAuxStreamOut);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4v, vv[r]), rv, soff, 0, kAuxStreamOut);
                if (out2) {
                    u32x2v w;
                    w[0] = bf16_rne(pv[r].x) | (bf16_rne(pv[r].y) << 16);
                    w[1] = bf16_rne(pv[r].z) | (bf16_rne(pv[r].w) << 16);
                    __builtin_amdgcn_raw_buffer_store_b64(w, ro, voff >> 1, 0, kAuxStreamOut);
                }
            } else {
                static_assert(!PACKED, "the packed layout is built with streaming stores only");
                st<NTS>(po4 + i, pv[r]);
                st<NTS>(mo4 + i, mv[r]);
                st<NTS>(vo4 + i, vv[r]);
                if (out2) {
                    u32x2 w;
                    w.x = bf16_rne(pv[r].x) | (bf16_rne(pv[r].y) << 16);
                    w.y = bf16_rne(pv[r].z) | (bf16_rne(pv[r].w) << 16);
                    st<NTS>(out2 + i, w);
                }
            }
        }
    }
}

// One tile of ROWS x BLOCK 128-bit vectors per workgroup; workgroups are dispatched in
// tile order, which keeps the set of pages the chip touches at any instant compact.
// Requires p, m, v 16-byte aligned and g, out aligned to 4 elements.  `tile0` is the
// tile index of workgroup 0 (launches are cut so that the grid stays below 2^31).
// The new state goes to po, mo, vo: the same arrays for the in-place step, or other arrays
// of the same alignment (the offloaded step reads staged copies and writes host memory).
// Each element is read before it is written and by the same lane, so p == po needs no care.
// PACKED: p == po is the packed state array, m, v, mo, vo are unused, and e0 is the index in
// the flat partition of the stretch's first element (a multiple of 4).
template <int ROWS, int BLOCK, bool G_BF16, int NT, int ARITH, bool PACKED = false>
__global__ __launch_bounds__(BLOCK) void adam_vec_kernel(const float *p, const float *m, const float *v,
                                                         float *po, float *mo, float *vo,
                                                         const void *__restrict__ g,
                                                         uint16_t *__restrict__ out, int64_t n,
                                                         int64_t tile0, AdamScalars s, DevCtl ctl,
                                                         int64_t e0 = 0)
{
    const int64_t nvec = n >> 2;
    const f32x4 *p4 = reinterpret_cast<const f32x4 *>(p);
    const f32x4 *m4 = reinterpret_cast<const f32x4 *>(m);
    const f32x4 *v4 = reinterpret_cast<const f32x4 *>(v);
    f32x4 *po4 = reinterpret_cast<f32x4 *>(po);
    f32x4 *mo4 = reinterpret_cast<f32x4 *>(mo);
    f32x4 *vo4 = reinterpret_cast<f32x4 *>(vo);
    u32x2 *out2 = reinterpret_cast<u32x2 *>(out);
    constexpr int64_t kTileVecs = (int64_t)BLOCK * ROWS;

    const int64_t tile = tile0 + blockIdx.x;
    const int64_t first = tile * kTileVecs + threadIdx.x;
    if ((tile + 1) * kTileVecs <= nvec)
        adam_tile<ROWS, BLOCK, G_BF16, NT, ARITH, false, PACKED>(p4, m4, v4, po4, mo4, vo4, g, out2, first, nvec,
                                                                 s, ctl, e0 >> 2);
    else
        adam_tile<ROWS, BLOCK, G_BF16, NT, ARITH, true, PACKED>(p4, m4, v4, po4, mo4, vo4, g, out2, first, nvec,
                                                                s, ctl, e0 >> 2);

    // The last n % 4 elements, one lane each, in the very first workgroup.
    const int64_t i = (nvec << 2) + threadIdx.x;
    if (tile == 0 && threadIdx.x < 4 && i < n && !(ctl.skip && *ctl.skip != 0)) {
        if (ctl.gscale) {
            s.gscalef = s.gscalef * *ctl.gscale;
            s.gscale = (double)s.gscalef;
        }
        const int64_t ip = PACKED ? packed_at(e0 + i) : i;
        const int64_t im = PACKED ? ip + kGranule : i, iv = PACKED ? ip + 2 * kGranule : i;
        if constexpr (PACKED) {
            m = p, v = p;
            mo = po, vo = po;
        }
        float pe = p[ip], me = m[im], ve = v[iv];
        float ge;
        if constexpr (G_BF16)
            ge = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(g)[i] << 16);
        else
            ge = reinterpret_cast<const float *>(g)[i];
        adam_elem<ARITH>(pe, me, ve, ge, s);
        po[ip] = pe;
        mo[im] = me;
        vo[iv] = ve;
        if (out)
            out[i] = (uint16_t)bf16_rne(pe);
    }
}

// Any natural alignment: one element per lane, grid-stride.  e0 >= 0: p == po is a packed
// state array and e0 the flat index of the stretch's first element (m, v, mo, vo unused).
template <bool G_BF16, int ARITH>
__global__ __launch_bounds__(256) void adam_scalar_kernel(const float *p, const float *m, const float *v,
                                                          float *po, float *mo, float *vo,
                                                          const void *__restrict__ g,
                                                          uint16_t *__restrict__ out, int64_t n,
                                                          AdamScalars s, DevCtl ctl, int64_t e0)
{
    if (ctl.skip && *ctl.skip != 0)
        return;
    if (ctl.gscale) {
        s.gscalef = s.gscalef * *ctl.gscale;
        s.gscale = (double)s.gscalef;
    }
    const bool packed = e0 >= 0;
    if (packed) {
        m = p, v = p;
        mo = po, vo = po;
    }
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const int64_t ip = packed ? packed_at(e0 + i) : i;
        const int64_t im = packed ? ip + kGranule : i, iv = packed ? ip + 2 * kGranule : i;
        float pe = p[ip], me = m[im], ve = v[iv];
        float ge;
        if constexpr (G_BF16)
            ge = __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(g)[i] << 16);
        else
            ge = reinterpret_cast<const float *>(g)[i];
        adam_elem<ARITH>(pe, me, ve, ge, s);
        po[ip] = pe;
        mo[im] = me;
        vo[iv] = ve;
        if (out)
            out[i] = (uint16_t)bf16_rne(pe);
    }
}

struct VecLaunch {
    dim3 grid;
    size_t lds;
    hipStream_t stream;
    const float *p, *m, *v;
    float *po, *mo, *vo;
    const void *g;
    uint16_t *out;
    int64_t n, tile0;
    AdamScalars s;
    DevCtl ctl;
    int64_t e0 = 0;   // packed launches: flat index of the stretch's first element
};

template <int ROWS, int BLOCK, bool G_BF16, int NT, int ARITH>
static void launch_vec(const VecLaunch &a)
{
    hipLaunchKernelGGL((adam_vec_kernel<ROWS, BLOCK, G_BF16, NT, ARITH>), a.grid, dim3(BLOCK), a.lds,
                       a.stream, a.p, a.m, a.v, a.po, a.mo, a.vo, a.g, a.out, a.n, a.tile0, a.s,
                       a.ctl, (int64_t)0);
}

template <int ROWS, int BLOCK, bool G_BF16, int NT>
static void pick_arith(int arith, const VecLaunch &a)
{
    if (arith == 0)
        launch_vec<ROWS, BLOCK, G_BF16, NT, 0>(a);
    else if (arith == 1)
        launch_vec<ROWS, BLOCK, G_BF16, NT, 1>(a);
    else
        launch_vec<ROWS, BLOCK, G_BF16, NT, 2>(a);
}

template <int ROWS, int BLOCK, bool G_BF16>
static void pick_nt(int nt, int arith, const VecLaunch &a)
{
    if (nt == 0) pick_arith<ROWS, BLOCK, G_BF16, 0>(arith, a);
    else if (nt == 1) pick_arith<ROWS, BLOCK, G_BF16, 1>(arith, a);
    else if (nt == 2) pick_arith<ROWS, BLOCK, G_BF16, 2>(arith, a);
    else if (nt == 3) pick_arith<ROWS, BLOCK, G_BF16, 3>(arith, a);
    else pick_arith<ROWS, BLOCK, G_BF16, 4>(arith, a);
}

template <int ROWS, int BLOCK>
static void pick_flags(bool g_bf16, int nt, int arith, const VecLaunch &a)
{
    if (g_bf16) pick_nt<ROWS, BLOCK, true>(nt, arith, a);
    else pick_nt<ROWS, BLOCK, false>(nt, arith, a);
}

template <int BLOCK>
static void pick_rows(int rows, bool g_bf16, int nt, int arith, const VecLaunch &a)
{
    if (rows == 1) pick_flags<1, BLOCK>(g_bf16, nt, arith, a);
    else if (rows == 2) pick_flags<2, BLOCK>(g_bf16, nt, arith, a);
    else pick_flags<4, BLOCK>(g_bf16, nt, arith, a);
}

static void launch_scalar(const float *p, const float *m, const float *v, float *po, float *mo, float *vo,
                          const void *g, bool g_bf16, int64_t n,
                          uint16_t *bf16_out, const AdamScalars &s, DevCtl ctl, int arith, int cus,
                          hipStream_t stream, int64_t e0 = -1)
{
    int64_t blocks = (n + 255) / 256;
    const int64_t cap = (int64_t)cus * 32;
    if (blocks > cap)
        blocks = cap;
    const dim3 grid((unsigned)blocks);
#define ZC_SCALAR(GB, AR)                                                                             \
    hipLaunchKernelGGL((adam_scalar_kernel<GB, AR>), grid, dim3(256), 0, stream, p, m, v, po, mo, vo, \
                       g, bf16_out, n, s, ctl, e0)
    if (g_bf16) {
        if (arith == 0) ZC_SCALAR(true, 0);
        else if (arith == 1) ZC_SCALAR(true, 1);
        else ZC_SCALAR(true, 2);
    } else {
        if (arith == 0) ZC_SCALAR(false, 0);
        else if (arith == 1) ZC_SCALAR(false, 1);
        else ZC_SCALAR(false, 2);
    }
#undef ZC_SCALAR
}

zc_status launch_adam(float *p, float *m, float *v, const void *g, zc_dtype g_dtype, int64_t n,
                      const zc_adam_hparams *hp, uint16_t *bf16_out, const int32_t *skip_flag,
                      hipStream_t stream, int waves_per_cu, const float *grad_scale_dev,
                      const AdamOut *out_of_place, const AdamShape *shape)
{
    const DevCtl ctl{skip_flag, grad_scale_dev};
    if (n == 0)
        return ZC_OK;
    float *po = out_of_place ? out_of_place->p : p;
    float *mo = out_of_place ? out_of_place->m : m;
    float *vo = out_of_place ? out_of_place->v : v;
    const AdamScalars s = make_scalars(hp);
    const Tune &t = tune();
    const bool g_bf16 = g_dtype == ZC_BF16;
    const int64_t g_size = g_bf16 ? 2 : 4;
    const int arith = (int)t.adam_arith;

    // A stretch that does not start on a 128-byte line of p (a parameter range cut out of a
    // larger partition) still takes the vector kernel: the elements in front of the next
    // line (at most 31) go to the one-element-per-lane kernel, after which every wave's
    // 1 KiB row covers whole lines again (measured: 6.4 instead of 5.4 TB/s).  This needs the
    // other arrays to reach vector alignment after the same number of elements; if only a
    // 16-byte boundary can be reached together, that one is taken.  Elements are
    // independent, so the order of the two launches does not matter.
    const uintptr_t pa = reinterpret_cast<uintptr_t>(p);
    const int64_t to_line = (int64_t)((128 - pa % 128) % 128) / 4;
    const int64_t to_vec = (int64_t)((16 - pa % 16) % 16) / 4;
    auto vec_ok_after = [&](int64_t k) {
        const char *gk = static_cast<const char *>(g) + k * g_size;
        return k < n && aligned_to(p + k, 16) && aligned_to(m + k, 16) && aligned_to(v + k, 16) &&
               aligned_to(po + k, 16) && aligned_to(mo + k, 16) && aligned_to(vo + k, 16) &&
               aligned_to(gk, g_bf16 ? 8 : 16) && (!bf16_out || aligned_to(bf16_out + k, 8));
    };
    int64_t peel = -1;                     // -1: the whole stretch takes the scalar kernel
    if (n >= 4096 && vec_ok_after(to_line))
        peel = to_line;
    else if (vec_ok_after(0))
        peel = 0;
    else if (vec_ok_after(to_vec))
        peel = to_vec;

    int cus = 0;
    if (peel != 0)
        ZC_TRY(num_cus(&cus));
    if (peel < 0) {
        launch_scalar(p, m, v, po, mo, vo, g, g_bf16, n, bf16_out, s, ctl, arith, cus, stream);
    } else {
        if (peel > 0) {
            launch_scalar(p, m, v, po, mo, vo, g, g_bf16, peel, bf16_out, s, ctl, arith, cus, stream);
            p += peel;
            m += peel;
            v += peel;
            po += peel;
            mo += peel;
            vo += peel;
            g = static_cast<const char *>(g) + peel * g_size;
            if (bf16_out)
                bf16_out += peel;
            n -= peel;
        }
        const int rows = shape ? shape->rows : (int)t.adam_rows;
        const int block = shape ? shape->block : (int)t.adam_block;
        const int nt = shape ? shape->nontemporal : (int)t.adam_nontemporal;
        const int64_t tile_vecs = (int64_t)block * rows;
        const int64_t nvec = n >> 2;
        int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;
        if (ntiles == 0)
            ntiles = 1;  // workgroup 0 also owns the n % 4 tail
        size_t lds = 0;
        // Resident-wave cap: the caller's, else the knob's, else (knob at -1) what measured
        // best on N(0, sigma) data with one-wave workgroups of one row at all three model
        // sizes: 13 waves per CU with bf16 gradients, 12 with fp32 gradients (one more
        // 16-byte load per lane in flight).  Below the optimum the kernel is latency-bound,
        // above it the eight read and write streams start to evict each other's open DRAM pages.
        int cap = waves_per_cu >= 0 ? waves_per_cu : (int)t.adam_waves_per_cu;
        if (cap < 0)
            cap = g_bf16 ? 13 : 12;
        ZC_TRY(occupancy_cap_lds(cap, block, &lds));
        VecLaunch a{dim3(1), lds, stream, p, m, v, po, mo, vo, g, bf16_out, n, 0, s, ctl};
        const int64_t kMaxGrid = max_workgroups_per_launch(t.launch_max_grid, block);
        for (int64_t tile0 = 0; tile0 < ntiles; tile0 += kMaxGrid) {
            const int64_t count = (ntiles - tile0) < kMaxGrid ? (ntiles - tile0) : kMaxGrid;
            a.grid = dim3((unsigned)count);
            a.tile0 = tile0;
            if (block == 64) pick_rows<64>(rows, g_bf16, nt, arith, a);
            else if (block == 128) pick_rows<128>(rows, g_bf16, nt, arith, a);
            else pick_rows<256>(rows, g_bf16, nt, arith, a);
        }
    }
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

// The update over elements [e0, e0 + n) of a packed state array; g and bf16_out point at the
// stretch's first element.  One-wave workgroups of one row with streaming stores and the
// default arithmetic: the shape every size ran fastest with; only the resident-wave cap is
// taken from the knobs.  The state array is 128-byte aligned and a granule is a whole number
// of lines, so the alignment of element e inside the array is that of 4*e.
static zc_status launch_adam_packed(float *state, int64_t e0, const void *g, zc_dtype g_dtype, int64_t n,
                                    const zc_adam_hparams *hp, uint16_t *bf16_out, const int32_t *skip_flag,
                                    const float *grad_scale_dev, hipStream_t stream)
{
    const DevCtl ctl{skip_flag, grad_scale_dev};
    if (n == 0)
        return ZC_OK;
    const AdamScalars s = make_scalars(hp);
    const Tune &t = tune();
    const bool g_bf16 = g_dtype == ZC_BF16;
    const int64_t g_size = g_bf16 ? 2 : 4;
    const int arith = (int)t.adam_arith;

    const int64_t to_line = (32 - e0 % 32) % 32, to_vec = (4 - e0 % 4) % 4;
    auto vec_ok_after = [&](int64_t k) {
        const char *gk = static_cast<const char *>(g) + k * g_size;
        return k < n && (e0 + k) % 4 == 0 && aligned_to(gk, g_bf16 ? 8 : 16) &&
               (!bf16_out || aligned_to(bf16_out + k, 8));
    };
    int64_t peel = -1;                     // -1: the whole stretch takes the scalar kernel
    if (n >= 4096 && vec_ok_after(to_line))
        peel = to_line;
    else if (vec_ok_after(to_vec))
        peel = to_vec;
    if (arith != 2)
        peel = -1;                         // the vector kernel is built for the default arithmetic only

    int cus = 0;
    if (peel != 0)
        ZC_TRY(num_cus(&cus));
    if (peel < 0) {
        launch_scalar(state, state, state, state, state, state, g, g_bf16, n, bf16_out, s, ctl, arith, cus,
                      stream, e0);
    } else {
        if (peel > 0) {
            launch_scalar(state, state, state, state, state, state, g, g_bf16, peel, bf16_out, s, ctl, arith,
                          cus, stream, e0);
            e0 += peel;
            g = static_cast<const char *>(g) + peel * g_size;
            if (bf16_out)
                bf16_out += peel;
            n -= peel;
        }
        const int64_t nvec = n >> 2;
        int64_t ntiles = (nvec + 63) / 64;
        if (ntiles == 0)
            ntiles = 1;  // workgroup 0 also owns the n % 4 tail
        int cap = (int)t.adam_waves_per_cu;
        if (cap < 0)
            cap = g_bf16 ? 13 : 12;   // as for three arrays: measured best at every size
        size_t lds = 0;
        ZC_TRY(occupancy_cap_lds(cap, 64, &lds));
        const int64_t kMaxGrid = max_workgroups_per_launch(t.launch_max_grid, 64);
        for (int64_t tile0 = 0; tile0 < ntiles; tile0 += kMaxGrid) {
            const int64_t count = (ntiles - tile0) < kMaxGrid ? (ntiles - tile0) : kMaxGrid;
            if (g_bf16)
                hipLaunchKernelGGL((adam_vec_kernel<1, 64, true, 4, 2, true>), dim3((unsigned)count), dim3(64),
                                   lds, stream, state, state, state, state, state, state, g, bf16_out, n, tile0,
                                   s, ctl, e0);
            else
                hipLaunchKernelGGL((adam_vec_kernel<1, 64, false, 4, 2, true>), dim3((unsigned)count), dim3(64),
                                   lds, stream, state, state, state, state, state, state, g, bf16_out, n, tile0,
                                   s, ctl, e0);
        }
    }
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

}  // namespace zc

namespace zc {

static zc_status check_adam_args(float *p, float *m, float *v, const void *g, zc_dtype g_dtype, int64_t n,
                                 const zc_adam_hparams *hp, uint16_t *bf16_out, const int32_t *skip_flag)
{
    if (n < 0)
        return fail(ZC_ERR_INVALID_ARG, "n is negative (%lld)", (long long)n);
    if (n > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "n exceeds 2^40 elements");
    ZC_TRY(check_dtype(g_dtype));
    ZC_TRY(check_hparams(hp));
    if (n == 0)
        return ZC_OK;
    if (!p || !m || !v || !g)
        return fail(ZC_ERR_INVALID_ARG, "p, m, v and g must not be NULL when n > 0");
    if (!aligned_to(p, 4) || !aligned_to(m, 4) || !aligned_to(v, 4))
        return fail(ZC_ERR_ALIGNMENT, "p, m, v must be 4-byte aligned");
    if (!aligned_to(g, g_dtype == ZC_BF16 ? 2 : 4))
        return fail(ZC_ERR_ALIGNMENT, "g is not aligned to its element size");
    if (bf16_out && !aligned_to(bf16_out, 2))
        return fail(ZC_ERR_ALIGNMENT, "bf16_out must be 2-byte aligned");
    if (skip_flag && !aligned_to(skip_flag, 4))
        return fail(ZC_ERR_ALIGNMENT, "skip_flag must be 4-byte aligned");
    // Every lane reads its own elements and then writes them; an array that shared bytes with
    // another would be read by one lane after another lane has written it.  No two may overlap.
    struct Span { uintptr_t lo, hi; };
    const uintptr_t n4 = (uintptr_t)n * 4, ng = (uintptr_t)n * (g_dtype == ZC_BF16 ? 2 : 4);
    const Span spans[5] = {{(uintptr_t)p, (uintptr_t)p + n4}, {(uintptr_t)m, (uintptr_t)m + n4},
                           {(uintptr_t)v, (uintptr_t)v + n4}, {(uintptr_t)g, (uintptr_t)g + ng},
                           {(uintptr_t)bf16_out, (uintptr_t)bf16_out + (bf16_out ? (uintptr_t)n * 2 : 0)}};
    for (int a = 0; a < 5; ++a)
        for (int b = a + 1; b < 5; ++b)
            if (spans[a].lo < spans[b].hi && spans[b].lo < spans[a].hi)
                return fail(ZC_ERR_INVALID_ARG, "p, m, v, g, bf16_out must not overlap");
    return ZC_OK;
}

static zc_status check_packed_args(float *state, const void *g, zc_dtype g_dtype, int64_t n,
                                   const zc_adam_hparams *hp, uint16_t *bf16_out, const int32_t *skip_flag)
{
    if (n < 0)
        return fail(ZC_ERR_INVALID_ARG, "n is negative (%lld)", (long long)n);
    if (n > kMaxElements)
        return fail(ZC_ERR_UNSUPPORTED, "n exceeds 2^40 elements");
    ZC_TRY(check_dtype(g_dtype));
    ZC_TRY(check_hparams(hp));
    if (n == 0)
        return ZC_OK;
    if (!state || !g)
        return fail(ZC_ERR_INVALID_ARG, "state and g must not be NULL when n > 0");
    if (!aligned_to(state, 128))
        return fail(ZC_ERR_ALIGNMENT, "state must be 128-byte aligned");
    if (!aligned_to(g, g_dtype == ZC_BF16 ? 2 : 4))
        return fail(ZC_ERR_ALIGNMENT, "g is not aligned to its element size");
    if (bf16_out && !aligned_to(bf16_out, 2))
        return fail(ZC_ERR_ALIGNMENT, "bf16_out must be 2-byte aligned");
    if (skip_flag && !aligned_to(skip_flag, 4))
        return fail(ZC_ERR_ALIGNMENT, "skip_flag must be 4-byte aligned");
    struct Span { uintptr_t lo, hi; };
    const uintptr_t ng = (uintptr_t)n * (g_dtype == ZC_BF16 ? 2 : 4);
    const Span spans[3] = {{(uintptr_t)state, (uintptr_t)state + (uintptr_t)zc_packed_state_numel(n) * 4},
                           {(uintptr_t)g, (uintptr_t)g + ng},
                           {(uintptr_t)bf16_out, (uintptr_t)bf16_out + (bf16_out ? (uintptr_t)n * 2 : 0)}};
    for (int a = 0; a < 3; ++a)
        for (int b = a + 1; b < 3; ++b)
            if (spans[a].lo < spans[b].hi && spans[b].lo < spans[a].hi)
                return fail(ZC_ERR_INVALID_ARG, "state, g, bf16_out must not overlap");
    return ZC_OK;
}

// Per-range hyper-parameters: sorted, disjoint, inside [0, n), finite values.
static zc_status check_ranges(const zc_adam_hparams *hp, const zc_param_range *ranges, int64_t nranges,
                              int64_t n, const float *grad_scale_dev)
{
    if (nranges < 0 || (nranges > 0 && !ranges))
        return fail(ZC_ERR_INVALID_ARG, "nranges is negative or ranges is NULL");
    if (grad_scale_dev && !aligned_to(grad_scale_dev, 4))
        return fail(ZC_ERR_ALIGNMENT, "grad_scale_dev must be 4-byte aligned");
    int64_t prev_end = 0;
    for (int64_t r = 0; r < nranges; ++r) {
        const zc_param_range &k = ranges[r];
        if (k.begin < prev_end || k.end < k.begin || k.end > n)
            return fail(ZC_ERR_INVALID_ARG, "range %lld: [%lld, %lld) is out of order or outside [0, n)",
                        (long long)r, (long long)k.begin, (long long)k.end);
        if (!(k.lr_scale == k.lr_scale) || k.lr_scale - k.lr_scale != 0.0f ||
            !(k.weight_decay == k.weight_decay) || k.weight_decay - k.weight_decay != 0.0f)
            return fail(ZC_ERR_INVALID_ARG, "range %lld: lr_scale and weight_decay must be finite", (long long)r);
        const float lr_here = hp->lr * k.lr_scale;
        if (lr_here - lr_here != 0.0f)
            return fail(ZC_ERR_INVALID_ARG, "range %lld: lr * lr_scale is not finite", (long long)r);
        prev_end = k.end;
    }
    return ZC_OK;
}

// One-lane kernel: clipping coefficient and loss-scale removal from the squared norm.
__global__ void clip_scale_kernel(const float *__restrict__ sqnorm, double max_norm, double inv_loss_scale,
                                  float *__restrict__ scale_out)
{
    if (threadIdx.x != 0 || blockIdx.x != 0)
        return;
    const double norm = sqrt((double)*sqnorm) * inv_loss_scale;
    double coef = 1.0;
    if (max_norm > 0.0) {
        coef = max_norm / (norm + 1e-6);
        if (coef > 1.0)
            coef = 1.0;
    }
    *scale_out = (float)(inv_loss_scale * coef);
}

}  // namespace zc

extern "C" zc_status zc_adam_step(float *p, float *m, float *v, const void *g, zc_dtype g_dtype,
                                  int64_t n, const zc_adam_hparams *hp, uint16_t *bf16_out,
                                  const int32_t *skip_flag, void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_adam_args(p, m, v, g, g_dtype, n, hp, bf16_out, skip_flag));
    if (n == 0)
        return ZC_OK;
    return launch_adam(p, m, v, g, g_dtype, n, hp, bf16_out, skip_flag, (hipStream_t)hip_stream);
}

extern "C" zc_status zc_adam_step_groups(float *p, float *m, float *v, const void *g, zc_dtype g_dtype,
                                         int64_t n, const zc_adam_hparams *hp,
                                         const zc_param_range *ranges, int64_t nranges, uint16_t *bf16_out,
                                         const int32_t *skip_flag, const float *grad_scale_dev,
                                         void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_adam_args(p, m, v, g, g_dtype, n, hp, bf16_out, skip_flag));
    ZC_TRY(check_ranges(hp, ranges, nranges, n, grad_scale_dev));
    if (n == 0)
        return ZC_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t g_size = g_dtype == ZC_BF16 ? 2 : 4;
    // One launch per stretch with its own hyper-parameters; uncovered stretches use *hp.
    auto launch = [&](int64_t begin, int64_t end, const zc_adam_hparams &h) -> zc_status {
        if (end <= begin)
            return ZC_OK;
        return launch_adam(p + begin, m + begin, v + begin, static_cast<const char *>(g) + begin * g_size,
                           g_dtype, end - begin, &h, bf16_out ? bf16_out + begin : nullptr, skip_flag, stream,
                           -1, grad_scale_dev);
    };
    int64_t at = 0;
    for (int64_t r = 0; r < nranges; ++r) {
        ZC_TRY(launch(at, ranges[r].begin, *hp));
        zc_adam_hparams h = *hp;
        h.lr = hp->lr * ranges[r].lr_scale;  // one fp32 product
        h.weight_decay = ranges[r].weight_decay;
        ZC_TRY(launch(ranges[r].begin, ranges[r].end, h));
        at = ranges[r].end;
    }
    return launch(at, n, *hp);
}

extern "C" int64_t zc_packed_state_numel(int64_t n)
{
    if (n <= 0)
        return 0;
    return 3 * ((n + zc::kGranule - 1) / zc::kGranule) * zc::kGranule;
}

extern "C" zc_status zc_adam_step_packed(float *state, const void *g, zc_dtype g_dtype, int64_t n,
                                         const zc_adam_hparams *hp, const zc_param_range *ranges,
                                         int64_t nranges, uint16_t *bf16_out, const int32_t *skip_flag,
                                         const float *grad_scale_dev, void *hip_stream)
{
    using namespace zc;
    ZC_TRY(check_packed_args(state, g, g_dtype, n, hp, bf16_out, skip_flag));
    ZC_TRY(check_ranges(hp, ranges, nranges, n, grad_scale_dev));
    if (n == 0)
        return ZC_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t g_size = g_dtype == ZC_BF16 ? 2 : 4;
    auto launch = [&](int64_t begin, int64_t end, const zc_adam_hparams &h) -> zc_status {
        if (end <= begin)
            return ZC_OK;
        return launch_adam_packed(state, begin, static_cast<const char *>(g) + begin * g_size, g_dtype,
                                  end - begin, &h, bf16_out ? bf16_out + begin : nullptr, skip_flag,
                                  grad_scale_dev, stream);
    };
    int64_t at = 0;
    for (int64_t r = 0; r < nranges; ++r) {
        ZC_TRY(launch(at, ranges[r].begin, *hp));
        zc_adam_hparams h = *hp;
        h.lr = hp->lr * ranges[r].lr_scale;  // one fp32 product
        h.weight_decay = ranges[r].weight_decay;
        ZC_TRY(launch(ranges[r].begin, ranges[r].end, h));
        at = ranges[r].end;
    }
    return launch(at, n, *hp);
}

extern "C" zc_status zc_clip_scale(const float *sqnorm, float max_norm, float inv_loss_scale,
                                   float *scale_out, void *hip_stream)
{
    using namespace zc;
    if (!sqnorm || !scale_out)
        return fail(ZC_ERR_INVALID_ARG, "sqnorm and scale_out must not be NULL");
    if (!aligned_to(sqnorm, 4) || !aligned_to(scale_out, 4))
        return fail(ZC_ERR_ALIGNMENT, "sqnorm and scale_out must be 4-byte aligned");
    if (!(max_norm >= 0.0f) || max_norm - max_norm != 0.0f)
        return fail(ZC_ERR_INVALID_ARG, "max_norm must be finite and >= 0 (0 = no clipping)");
    if (!(inv_loss_scale > 0.0f) || inv_loss_scale - inv_loss_scale != 0.0f)
        return fail(ZC_ERR_INVALID_ARG, "inv_loss_scale must be finite and > 0");
    hipLaunchKernelGGL(clip_scale_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, sqnorm,
                       (double)max_norm, (double)inv_loss_scale, scale_out);
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

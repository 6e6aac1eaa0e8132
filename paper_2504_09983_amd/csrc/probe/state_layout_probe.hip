// Stand-alone measurement of the update kernel's memory pattern under different layouts of the
// optimizer state: three separate arrays, one packed array with granules of R rows (R x 256
// elements of p, then of m, then of v), and a packed array with the fp32 gradient as a fourth
// slot.  It shares no code with the library: the point is to time the access pattern alone, with
// the same arithmetic per element, so that the library's granule (8192 elements) can be checked
// or chosen again on another machine.
//
//   state_layout_probe <elements> [bf16|fp32]
//
// One wave per workgroup, one 1 KiB row of each array per wave, non-temporal loads, write-through
// streaming stores, resident waves capped through an unused LDS request: the library's launch
// shape.  Prints the fraction of 8 TB/s (28 bytes per element with bf16 gradients, 30 with fp32).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t su32x4 __attribute__((vector_size(16)));
typedef uint32_t su32x2 __attribute__((vector_size(8)));
constexpr int kFlags = 0x00020000;   // raw buffer, 32-bit format
constexpr int kAux = 2 | 16;         // nt | sc1

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);    \
            exit(1);                                                                 \
        }                                                                            \
    } while (0)

struct Scalars { double b1, omb1, b2, omb2, step_size, inv_sqrt_bc2, eps, decay; };

__device__ __forceinline__ void elem(float &p, float &m, float &v, float g, const Scalars &s)
{
    float mn, vn;
    {
#pragma clang fp contract(off)
        const double gd = (double)g;
        mn = (float)(s.b1 * (double)m + s.omb1 * gd);
        vn = (float)(s.b2 * (double)v + (s.omb2 * gd) * gd);
    }
    const double denom = fma(sqrt((double)vn), s.inv_sqrt_bc2, s.eps);
    p = (float)((double)p * s.decay - s.step_size * (double)mn / denom);
    m = mn;
    v = vn;
}

__device__ __forceinline__ uint32_t rne(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Workgroup b owns row b: row r = b % R of granule T = b / R.  The three (or four) arrays of a
// granule start `slot` vectors apart and granules `stride` vectors apart; separate arrays are
// the case R = 1, stride = 64 with p4, m4, v4 pointing at the arrays.
template <bool G_FP32, bool G_IN_STATE>
__global__ __launch_bounds__(64) void update(f32x4 *p4, f32x4 *m4, f32x4 *v4, const void *g, u32x2 *out2,
                                             int64_t rows, int R, int64_t stride, Scalars s)
{
    const int64_t b = blockIdx.x;
    if (b >= rows)
        return;
    const int64_t at = (b / R) * stride + (b % R) * 64;
    const int lane = threadIdx.x;
    f32x4 pv = __builtin_nontemporal_load(p4 + at + lane);
    f32x4 mv = __builtin_nontemporal_load(m4 + at + lane);
    f32x4 vv = __builtin_nontemporal_load(v4 + at + lane);
    f32x4 gv;
    if constexpr (G_IN_STATE) {
        gv = __builtin_nontemporal_load(v4 + (v4 - m4) + at + lane);    // the slot behind v
    } else if constexpr (G_FP32) {
        gv = __builtin_nontemporal_load(static_cast<const f32x4 *>(g) + b * 64 + lane);
    } else {
        const u32x2 w = __builtin_nontemporal_load(static_cast<const u32x2 *>(g) + b * 64 + lane);
        gv.x = __uint_as_float(w.x << 16);
        gv.y = __uint_as_float(w.x & 0xFFFF0000u);
        gv.z = __uint_as_float(w.y << 16);
        gv.w = __uint_as_float(w.y & 0xFFFF0000u);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float pe = pv[k], me = mv[k], ve = vv[k];
        elem(pe, me, ve, gv[k], s);
        pv[k] = pe;
        mv[k] = me;
        vv[k] = ve;
    }
    const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc((void *)(p4 + at), 0, 1024, kFlags);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc((void *)(m4 + at), 0, 1024, kFlags);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)(v4 + at), 0, 1024, kFlags);
    const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc((void *)(out2 + b * 64), 0, 512, kFlags);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(su32x4, pv), rp, lane * 16, 0, kAux);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(su32x4, mv), rm, lane * 16, 0, kAux);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(su32x4, vv), rv, lane * 16, 0, kAux);
    su32x2 o;
    o[0] = rne(pv.x) | (rne(pv.y) << 16);
    o[1] = rne(pv.z) | (rne(pv.w) << 16);
    __builtin_amdgcn_raw_buffer_store_b64(o, ro, lane * 8, 0, kAux);
}

// Roughly normal values from a counter hash (sum of four uniforms), so that the arrays hold
// ordinary numbers: zero-filled memory runs measurably faster than real data.
__device__ __forceinline__ float noise(uint64_t i, uint32_t salt)
{
    float acc = 0.f;
    uint64_t x = i * 0x9E3779B97F4A7C15ull + salt;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        x ^= x >> 31;
        x *= 0xBF58476D1CE4E5B9ull;
        x ^= x >> 29;
        acc += (float)(uint32_t)(x >> 40) * (1.0f / 16777216.0f) - 0.5f;
    }
    return acc * 1.7320508f;
}

// slot 0: p ~ N(0, 0.02); slot 1: m ~ N(0, 1e-3); slot 2: v = (N(0, 1e-3))^2; slot 3: g ~ N(0, 1e-3).
// `gran` elements per slot; slots == 1 fills one plain array of kind `kind`.
__global__ void fill(float *a, int64_t total, int64_t gran, int slots, int kind)
{
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const int which = slots == 1 ? kind : (int)((i / gran) % slots);
        const float z = noise((uint64_t)i, 7u + which);
        a[i] = which == 0 ? 0.02f * z : which == 2 ? (1e-3f * z) * (1e-3f * z) : 1e-3f * z;
    }
}

__global__ void fill_bf16(uint16_t *a, int64_t n)
{
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step)
        a[i] = (uint16_t)rne(1e-3f * noise((uint64_t)i, 3u));
}

static size_t lds_for_cap(int cap, int lds_per_cu)
{
    size_t per = (size_t)lds_per_cu / (size_t)cap;
    per &= ~(size_t)255;
    return per > 64 * 1024 ? 64 * 1024 : per;
}

int main(int argc, char **argv)
{
    int64_t n = argc > 1 ? atoll(argv[1]) : 1003782656ll;
    const bool g_fp32 = argc > 2 && strcmp(argv[2], "fp32") == 0;
    constexpr int kMaxR = 4096;
    n -= n % ((int64_t)256 * kMaxR);                       // whole granules for every R tried
    const int64_t rows = n / 256;
    if (n <= 0 || rows > 0xFFFFFFFFll / 64) {
        printf("elements must be between %d and 2^34\n", 256 * kMaxR);
        return 1;
    }
    int lds_per_cu = 0;
    CK(hipDeviceGetAttribute(&lds_per_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, 0));
    const double bytes = g_fp32 ? 30.0 : 28.0;
    printf("# %lld elements, %s gradients, %.0f bytes per element; fraction of 8 TB/s by cap on resident waves per CU\n",
           (long long)n, g_fp32 ? "fp32" : "bf16", bytes);
    float *state = nullptr;
    void *g = nullptr;
    uint16_t *out = nullptr;
    CK(hipMalloc(&state, (size_t)n * 16));
    CK(hipMalloc(&g, (size_t)n * (g_fp32 ? 4 : 2)));
    CK(hipMalloc(&out, (size_t)n * 2));
    if (g_fp32)
        fill<<<4096, 256>>>((float *)g, n, n, 1, 3);
    else
        fill_bf16<<<4096, 256>>>((uint16_t *)g, n);
    const Scalars s{0.9, 0.1, 0.999, 0.001, 1e-4, 1.0, 1e-8, 1.0 - 1e-6};
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    struct Layout { const char *name; int R; int slots; };
    const Layout layouts[] = {{"three arrays", 0, 3},        {"granule 256", 1, 3},      {"granule 2048", 8, 3},
                              {"granule 4096", 16, 3},       {"granule 8192", 32, 3},    {"granule 16384", 64, 3},
                              {"granule 32768", 128, 3},     {"granule 262144", 1024, 3}, {"granule 1048576", 4096, 3},
                              {"granule 8192, g inside", 32, 4}, {"three arrays", 0, 3}};
    const int caps[] = {8, 10, 11, 12, 13, 14, 16};
    for (const Layout &L : layouts) {
        if (L.slots == 4 && !g_fp32)
            continue;
        f32x4 *p4 = (f32x4 *)state, *m4, *v4;
        int R;
        int64_t stride;
        if (L.R == 0) {
            for (int a = 0; a < 3; ++a)
                fill<<<4096, 256>>>(state + a * n, n, n, 1, a);
            m4 = (f32x4 *)(state + n);
            v4 = (f32x4 *)(state + 2 * n);
            R = 1;
            stride = 64;
        } else {
            R = L.R;
            fill<<<4096, 256>>>(state, (int64_t)L.slots * n, (int64_t)R * 256, L.slots, 0);
            m4 = p4 + (int64_t)R * 64;
            v4 = p4 + (int64_t)2 * R * 64;
            stride = (int64_t)L.slots * R * 64;
        }
        CK(hipDeviceSynchronize());
        printf("%-24s:", L.name);
        for (int cap : caps) {
            const size_t lds = lds_for_cap(cap, lds_per_cu);
            const int reps = n > (int64_t)2e9 ? 4 : 10;
            auto run = [&]() {
                const dim3 grid((unsigned)rows), block(64);
                if (L.slots == 4)
                    update<true, true><<<grid, block, lds>>>(p4, m4, v4, nullptr, (u32x2 *)out, rows, R, stride, s);
                else if (g_fp32)
                    update<true, false><<<grid, block, lds>>>(p4, m4, v4, g, (u32x2 *)out, rows, R, stride, s);
                else
                    update<false, false><<<grid, block, lds>>>(p4, m4, v4, g, (u32x2 *)out, rows, R, stride, s);
            };
            run();
            run();
            CK(hipEventRecord(e0));
            for (int i = 0; i < reps; ++i)
                run();
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipGetLastError());
            float ms = 0;
            CK(hipEventElapsedTime(&ms, e0, e1));
            printf(" %2d %.3f", cap, (double)n * bytes / (ms / reps * 1e-3) / 8e12);
            fflush(stdout);
        }
        printf("\n");
    }
    CK(hipFree(state));
    CK(hipFree(g));
    CK(hipFree(out));
    return 0;
}

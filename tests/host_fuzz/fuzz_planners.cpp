// Host-only fuzz driver for the layout and planner entry points, built with
// AddressSanitizer and UndefinedBehaviorSanitizer on the host side (no GPU call is made:
// these entry points are pure host functions).  Random, partly invalid arguments; every
// call must either succeed or return a status, and the sanitizers must stay silent.
// Built and run by tests/test_host_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include <hip/hip_runtime.h>

#include "zc.h"

// The planner source also holds the stream executor, which refers to the offload context's
// accessors; the executor is not called here, so inert stand-ins satisfy the linker.
struct zc_offload_ctx;
namespace zc {
hipStream_t offload_h2d_stream(zc_offload_ctx *) { return nullptr; }
hipStream_t offload_d2h_stream(zc_offload_ctx *) { return nullptr; }
int offload_device(zc_offload_ctx *) { return 0; }
zc_status offload_events(zc_offload_ctx *, int64_t, hipEvent_t **) { return ZC_ERR_UNSUPPORTED; }
}  // namespace zc

static void expect_error(zc_status s)
{
    if (s == ZC_OK) {
        std::fprintf(stderr, "sizes near INT64_MAX were accepted\n");
        std::exit(3);
    }
}

static void extreme_sizes()
{
    {
        // an alignment near INT64_MAX must be refused, not rounded up to
        std::vector<int64_t> one = {5};
        std::vector<int64_t> o(2), a(9), b(9), c(9);
        int64_t shard = 0, total = 0, send = 0;
        expect_error(zc_flat_layout(one.data(), 1, 8, INT64_MAX - 3, o.data(), &shard, &total));
        expect_error(zc_per_tensor_layout(one.data(), 1, 8, INT64_MAX - 3, a.data(), b.data(), c.data(), &send));
    }
    int64_t big = INT64_MAX / 2;
    std::vector<int64_t> numels = {big, big, big, 7};
    std::vector<int64_t> offs(5); int64_t shard = 0, total = 0;
    expect_error(zc_flat_layout(numels.data(), 4, 8, 4096, offs.data(), &shard, &total));
    std::vector<int64_t> a(64), b(64), c(64); int64_t send = 0;
    expect_error(zc_per_tensor_layout(numels.data(), 4, 8, 4096, a.data(), b.data(), c.data(), &send));
    std::vector<int64_t> pmem = {INT64_MAX - 5, 10}, fb = {INT64_MAX / 2, INT64_MAX / 2, INT64_MAX / 2};
    std::vector<zc_sched_op> out(64); int64_t nout = 0;
    expect_error(zc_plan_adaptive_offload(pmem.data(), 2, 1, fb.data(), 3, INT64_MAX, out.data(), 64, &nout));
    std::vector<int32_t> isag = {1, 1, 1}; std::vector<int64_t> bag = {INT64_MAX / 2, INT64_MAX / 2, INT64_MAX / 2}, pm = {INT64_MAX / 2, 1, 1};
    std::vector<int64_t> sizes = {1, INT64_MAX}; std::vector<double> times = {1.0, 2.0};
    std::vector<int32_t> order(4), grp(4);
    expect_error(zc_plan_prefetch(isag.data(), bag.data(), pm.data(), 3, INT64_MAX, INT64_MAX, sizes.data(), times.data(), 2, 1.5, order.data(), grp.data()));
    std::vector<int32_t> chosen(4); int64_t nch = 0;
    (void)(zc_select_unsharded(bag.data(), 3, sizes.data(), times.data(), 2, INT64_MAX, chosen.data(), &nch));
}

int main()
{
    extreme_sizes();
    std::mt19937_64 rng(12345);
    auto rnd = [&](int64_t lo, int64_t hi) { return lo + (int64_t)(rng() % (uint64_t)(hi - lo + 1)); };
    long calls = 0, ok = 0;
    for (int it = 0; it < 20000; ++it) {
        int64_t nt = rnd(0, 40);
        std::vector<int64_t> numels(nt);
        for (auto &x : numels) x = rnd(-1, 5000) < 0 ? (rnd(0, 9) ? 0 : -5) : rnd(0, 5000);
        int32_t world = (int32_t)rnd(-1, 9);
        int64_t align = rnd(-1, 5) < 0 ? 0 : (int64_t[]){1, 3, 8, 4096, 7, 1}[rnd(0, 5)];
        std::vector<int64_t> offs(nt + 1);
        int64_t shard = 0, total = 0;
        calls++; if (zc_flat_layout(numels.data(), nt, world, align, offs.data(), &shard, &total) == ZC_OK) ok++;
        if (world > 0) {
            std::vector<int64_t> a((size_t)nt * world + 1), b((size_t)nt * world + 1), c((size_t)nt * world + 1);
            int64_t send = 0;
            calls++; if (zc_per_tensor_layout(numels.data(), nt, world, align, a.data(), b.data(), c.data(), &send) == ZC_OK) ok++;
        }
        // adaptive offload
        int64_t nops = rnd(0, 30), nf = rnd(0, nops + 1), nfr = rnd(0, 12);
        std::vector<int64_t> pmem(nops), fb(nfr);
        for (auto &x : pmem) x = rnd(-2, 100);
        for (auto &x : fb) x = rnd(-1, 20);
        int64_t cap = rnd(0, 3 * (nops + 2 * nfr) + 4);
        std::vector<zc_sched_op> out(cap + 1);
        int64_t nout = 0;
        calls++; if (zc_plan_adaptive_offload(pmem.data(), nops, nf, fb.data(), nfr, rnd(0, 200), out.data(), cap, &nout) == ZC_OK) ok++;
        // prefetch
        int64_t N = rnd(0, 30), ns = rnd(0, 5);
        std::vector<int32_t> isag(N); std::vector<int64_t> bag(N), pm(N), sizes(ns); std::vector<double> times(ns);
        for (int64_t i = 0; i < N; ++i) { isag[i] = (int32_t)rnd(0, 1); bag[i] = rnd(-1, 50); pm[i] = rnd(0, 100); }
        int64_t s = 0; for (int64_t i = 0; i < ns; ++i) { s += rnd(0, 20); sizes[i] = s; times[i] = (double)rnd(-1, 100) / 7.0; }
        std::vector<int32_t> order(N + 1), grp(N + 1);
        calls++; if (zc_plan_prefetch(isag.data(), bag.data(), pm.data(), N, rnd(0, 200), rnd(0, 100), sizes.data(), times.data(), ns, (double)rnd(0, 30) / 10.0, order.data(), grp.data()) == ZC_OK) ok++;
        std::vector<int32_t> chosen(N + 1); int64_t nch = 0;
        calls++; if (zc_select_unsharded(bag.data(), N, sizes.data(), times.data(), ns, rnd(-1, 300), chosen.data(), &nch) == ZC_OK) ok++;
    }
    printf("calls %ld ok %ld\n", calls, ok);
    return 0;
}

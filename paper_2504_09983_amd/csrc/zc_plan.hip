// Adaptive offloading of optimizer-state fragments: the planner (host only) and a
// small executor that replays a plan on HIP streams with stand-in compute kernels.
//
// Planner: forward pass as in the paper's Algorithm 2 (Adaptive offloading) —
// start asynchronous copies of just enough fragments for the profiled peak to
// fit, and insert "wait for the copy and free" right before the first operator
// that would otherwise exceed the limit; backward pass as in the paragraph that
// follows it — start the copy back of a fragment as soon as enough memory stays
// free from that operator to the end of the schedule.  Fragments leave and
// return in list order; every reload is waited for at the end, before the update.
//
// Executor: operators are spin kernels of given durations on the caller's
// stream, copies run on the offload context's two copy streams, and the plan's
// wait operators become cross-stream event waits, so the overlap the plan
// promises can be measured against the "offload everything, synchronously" mode.
#include <algorithm>
#include <vector>

#include "zc_internal.h"

struct zc_offload_ctx;

namespace zc {

// Access to the copy streams of an offload context (defined with the context).
hipStream_t offload_h2d_stream(zc_offload_ctx *ctx);
hipStream_t offload_d2h_stream(zc_offload_ctx *ctx);
int offload_device(zc_offload_ctx *ctx);
zc_status offload_events(zc_offload_ctx *ctx, int64_t count, hipEvent_t **out);

// Bounded busy-wait: leaves after `ticks` of the constant-rate wall clock or after
// `max_iters` rounds, whichever comes first, so the wave always retires.
__global__ __launch_bounds__(64) void spin_kernel(uint64_t ticks, int64_t max_iters)
{
    const uint64_t t0 = wall_clock64();
    for (int64_t it = 0; it < max_iters; ++it) {
        if (wall_clock64() - t0 >= ticks)
            break;
        __builtin_amdgcn_s_sleep(64);
    }
}

__global__ __launch_bounds__(256) void poison_kernel(uint32_t *__restrict__ dst, int64_t nwords)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nwords; i += stride)
        dst[i] = 0xDEADBEEFu;
}

// Overwrite `words` 32-bit words with a pattern no optimizer state holds: stands in for
// handing memory to another owner, so that a missing fence shows up as garbage.
zc_status launch_poison(void *dst, int64_t words, hipStream_t stream)
{
    if (words <= 0)
        return ZC_OK;
    int cus = 0;
    ZC_TRY(num_cus(&cus));
    int64_t blocks = (words + 255) / 256;
    if (blocks > (int64_t)cus * 8)
        blocks = (int64_t)cus * 8;
    hipLaunchKernelGGL(poison_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<uint32_t *>(dst), words);
    ZC_HIP(hipGetLastError());
    return ZC_OK;
}

// Profiled communication time for `bytes`: the table is linear between samples, flat
// below the first one and continued with the last slope above the last one.
static double comm_time(int64_t bytes, const int64_t *sizes, const double *times, int64_t n)
{
    if (bytes <= sizes[0] || n == 1)
        return times[0];
    int64_t k = n - 1;
    for (int64_t i = 1; i < n; ++i) {
        if (bytes <= sizes[i]) {
            k = i;
            break;
        }
    }
    const double s0 = (double)sizes[k - 1], s1 = (double)sizes[k];
    const double t0 = times[k - 1], t1 = times[k];
    return t0 + (t1 - t0) * ((double)bytes - s0) / (s1 - s0);
}

static zc_status check_comm_table(const int64_t *sizes, const double *times, int64_t n)
{
    if (n < 1 || !sizes || !times)
        return fail(ZC_ERR_INVALID_ARG, "the communication-time table needs at least one sample");
    for (int64_t i = 0; i < n; ++i) {
        if (sizes[i] <= 0 || !(times[i] >= 0.0) || (i > 0 && sizes[i] <= sizes[i - 1]))
            return fail(ZC_ERR_INVALID_ARG, "table sizes must be positive and increasing, times >= 0");
    }
    return ZC_OK;
}

enum FragState { kResident, kCopyingOut, kOnHost, kCopyingIn };

// Shared validation: the ordering rules any executable schedule must obey.
static zc_status check_schedule(const zc_sched_op *ops, int64_t nops, int64_t n_ops, int64_t nfrags)
{
    std::vector<int> state((size_t)nfrags, kResident);
    int64_t next_op = 0;
    for (int64_t k = 0; k < nops; ++k) {
        const int32_t kind = ops[k].kind, idx = ops[k].index;
        if (kind == ZC_OP_COMPUTE) {
            if (idx != next_op)
                return fail(ZC_ERR_INVALID_ARG, "schedule entry %lld: operator %d out of order", (long long)k, idx);
            ++next_op;
            continue;
        }
        if (kind < ZC_OP_COMPUTE || kind > ZC_OP_SYNC_RELOAD)
            return fail(ZC_ERR_INVALID_ARG, "schedule entry %lld: unknown kind %d", (long long)k, kind);
        if (idx < 0 || idx >= nfrags)
            return fail(ZC_ERR_INVALID_ARG, "schedule entry %lld: fragment %d out of range", (long long)k, idx);
        int &s = state[(size_t)idx];
        const int want = kind == ZC_OP_OFFLOAD ? kResident
                         : kind == ZC_OP_SYNC_FREE ? kCopyingOut
                         : kind == ZC_OP_RELOAD ? kOnHost : kCopyingIn;
        if (s != want)
            return fail(ZC_ERR_INVALID_ARG, "schedule entry %lld: fragment %d is in the wrong state for kind %d",
                        (long long)k, idx, kind);
        s = kind == ZC_OP_OFFLOAD ? kCopyingOut
            : kind == ZC_OP_SYNC_FREE ? kOnHost
            : kind == ZC_OP_RELOAD ? kCopyingIn : kResident;
    }
    if (next_op != n_ops)
        return fail(ZC_ERR_INVALID_ARG, "schedule runs %lld of %lld operators", (long long)next_op, (long long)n_ops);
    for (int64_t f = 0; f < nfrags; ++f)
        if (state[(size_t)f] == kOnHost || state[(size_t)f] == kCopyingIn)
            return fail(ZC_ERR_INVALID_ARG, "fragment %lld is not back on the device when the schedule ends", (long long)f);
    return ZC_OK;
}

}  // namespace zc

extern "C" {

zc_status zc_plan_adaptive_offload(const int64_t *p_mem, int64_t n_ops, int64_t n_forward,
                                   const int64_t *frag_bytes, int64_t nfrags, int64_t mem_limit,
                                   zc_sched_op *out, int64_t capacity, int64_t *out_len)
{
    using namespace zc;
    if (!out_len)
        return fail(ZC_ERR_INVALID_ARG, "out_len is NULL");
    *out_len = 0;
    if (n_ops < 0 || n_forward < 0 || n_forward > n_ops || nfrags < 0 || mem_limit < 0)
        return fail(ZC_ERR_INVALID_ARG, "need 0 <= n_forward <= n_ops, nfrags >= 0, mem_limit >= 0");
    if ((n_ops > 0 && !p_mem) || (nfrags > 0 && !frag_bytes))
        return fail(ZC_ERR_INVALID_ARG, "p_mem / frag_bytes is NULL");
    if (n_ops > 0x7FFFFFFF || nfrags > 0x7FFFFFFF)
        return fail(ZC_ERR_UNSUPPORTED, "more than 2^31 operators or fragments");
    const int64_t kMax = int64_t(1) << 60;
    int64_t m_opt = 0;
    for (int64_t f = 0; f < nfrags; ++f) {
        if (frag_bytes[f] < 0 || frag_bytes[f] > kMax - m_opt)
            return fail(ZC_ERR_INVALID_ARG, "fragment sizes must be >= 0 and sum below 2^60");
        m_opt += frag_bytes[f];
    }
    int64_t m_peak = 0;
    for (int64_t i = 0; i < n_ops; ++i) {
        if (p_mem[i] < 0 || p_mem[i] > kMax)
            return fail(ZC_ERR_INVALID_ARG, "p_mem[%lld] out of range", (long long)i);
        if (p_mem[i] > m_peak)
            m_peak = p_mem[i];  // over the whole iteration: the spikes may sit in the backward pass
    }

    std::vector<zc_sched_op> s;
    s.reserve((size_t)(n_ops + 4 * nfrags));
    // Which fragments leave: the shortest prefix that lets the peak fit.
    int64_t n_out = 0, out_bytes = 0;
    while (n_out < nfrags && m_peak + m_opt - out_bytes > mem_limit) {
        s.push_back({ZC_OP_OFFLOAD, (int32_t)n_out});
        out_bytes += frag_bytes[n_out];
        ++n_out;
    }
    // tail_max[i] = largest profiled usage from operator i to the end.
    std::vector<int64_t> tail_max((size_t)n_ops + 1, 0);
    for (int64_t i = n_ops - 1; i >= 0; --i)
        tail_max[(size_t)i] = p_mem[i] > tail_max[(size_t)i + 1] ? p_mem[i] : tail_max[(size_t)i + 1];
    // Fragments [0, freed) have been freed, [0, back) of those are on their way back.
    int64_t freed = 0, back = 0, m_minus = 0;
    for (int64_t i = 0; i < n_ops; ++i) {
        // free a fragment (after waiting for its copy) only when an operator needs the room
        while (p_mem[i] + m_opt - m_minus > mem_limit) {
            if (freed == n_out)
                return fail(ZC_ERR_UNSUPPORTED,
                            "operator %lld needs %lld bytes: over the limit even with every fragment offloaded",
                            (long long)i, (long long)p_mem[i]);
            s.push_back({ZC_OP_SYNC_FREE, (int32_t)freed});
            m_minus += frag_bytes[freed];
            ++freed;
        }
        // backward pass: start a copy back as soon as the rest of the schedule leaves room
        if (i >= n_forward) {
            while (back < freed && tail_max[(size_t)i] + m_opt - m_minus + frag_bytes[back] <= mem_limit) {
                s.push_back({ZC_OP_RELOAD, (int32_t)back});
                m_minus -= frag_bytes[back];
                ++back;
            }
        }
        s.push_back({ZC_OP_COMPUTE, (int32_t)i});
    }
    for (; back < freed; ++back)
        s.push_back({ZC_OP_RELOAD, (int32_t)back});
    for (int64_t f = 0; f < freed; ++f)
        s.push_back({ZC_OP_SYNC_RELOAD, (int32_t)f});

    *out_len = (int64_t)s.size();
    if ((int64_t)s.size() > capacity || (!out && !s.empty()))
        return fail(ZC_ERR_INVALID_ARG, "schedule has %lld entries, room for %lld", (long long)s.size(),
                    (long long)capacity);
    for (size_t k = 0; k < s.size(); ++k)
        out[k] = s[k];
    return ZC_OK;
}

zc_status zc_plan_prefetch(const int32_t *is_allgather, const int64_t *bag_bytes, const int64_t *p_mem,
                           int64_t n_ops, int64_t mem_limit, int64_t prefetch_limit,
                           const int64_t *tc_sizes, const double *tc_times, int64_t n_tc, double alpha,
                           int32_t *order_out, int32_t *group_out)
{
    using namespace zc;
    if (n_ops < 0 || mem_limit < 0 || prefetch_limit < 0)
        return fail(ZC_ERR_INVALID_ARG, "n_ops, mem_limit and prefetch_limit must be >= 0");
    if (n_ops > 0 && (!is_allgather || !bag_bytes || !p_mem || !order_out || !group_out))
        return fail(ZC_ERR_INVALID_ARG, "an input or output table is NULL");
    if (n_ops > 0x7FFFFFFF)
        return fail(ZC_ERR_UNSUPPORTED, "more than 2^31 operators");
    if (!(alpha >= 0.0))
        return fail(ZC_ERR_INVALID_ARG, "alpha must be >= 0");
    ZC_TRY(check_comm_table(tc_sizes, tc_times, n_tc));
    const int64_t kMax = int64_t(1) << 60;
    for (int64_t i = 0; i < n_ops; ++i) {
        if (p_mem[i] < 0 || p_mem[i] > kMax || bag_bytes[i] < 0 || bag_bytes[i] > kMax)
            return fail(ZC_ERR_INVALID_ARG, "operator %lld: sizes out of range", (long long)i);
        if (is_allgather[i] && bag_bytes[i] == 0)
            return fail(ZC_ERR_INVALID_ARG, "operator %lld: an all-gather needs a buffer size", (long long)i);
    }

    // The new schedule is assembled back to front: (operator, group id) pairs.
    std::vector<int32_t> rev_op, rev_grp;
    rev_op.reserve((size_t)n_ops);
    rev_grp.reserve((size_t)n_ops);
    std::vector<int32_t> pending;  // unscheduled all-gathers, latest first
    int64_t pending_bytes = 0;
    int32_t next_group = 0;

    // Place the pending all-gathers here, fused where two of them together are cheaper than
    // apart by the factor alpha.  Groups are formed in schedule order (earliest first).
    auto flush = [&]() {
        if (pending.empty())
            return;
        std::vector<int32_t> grp_of(pending.size());
        int64_t cur_bytes = 0;
        int32_t cur = -1;
        for (size_t k = pending.size(); k-- > 0;) {  // earliest first
            const int64_t v2 = bag_bytes[pending[k]];
            bool join = false;
            if (cur >= 0) {
                const double apart = comm_time(cur_bytes, tc_sizes, tc_times, n_tc) +
                                     comm_time(v2, tc_sizes, tc_times, n_tc);
                join = apart > alpha * comm_time(cur_bytes + v2, tc_sizes, tc_times, n_tc);
            }
            if (join) {
                cur_bytes += v2;
            } else {
                cur = next_group++;
                cur_bytes = v2;
            }
            grp_of[k] = cur;
        }
        for (size_t k = 0; k < pending.size(); ++k) {  // latest first, as the list is reversed later
            rev_op.push_back(pending[k]);
            rev_grp.push_back(grp_of[k]);
        }
        pending.clear();
        pending_bytes = 0;
    };

    for (int64_t i = n_ops - 1; i >= 1; --i) {
        if (!is_allgather[i]) {
            rev_op.push_back((int32_t)i);
            rev_grp.push_back(-1);
            continue;
        }
        const int64_t group_bytes = pending_bytes + bag_bytes[i];
        if (p_mem[i - 1] + group_bytes < mem_limit && group_bytes < prefetch_limit) {
            pending.push_back((int32_t)i);  // moves further up together with the others
            pending_bytes = group_bytes;
        } else {
            flush();
            if (p_mem[i - 1] + bag_bytes[i] < mem_limit && bag_bytes[i] < prefetch_limit) {
                pending.push_back((int32_t)i);
                pending_bytes = bag_bytes[i];
            } else {
                rev_op.push_back((int32_t)i);  // stays where it is
                rev_grp.push_back(next_group++);
            }
        }
    }
    if (n_ops > 0) {
        if (is_allgather[0]) {
            if (pending_bytes + bag_bytes[0] >= prefetch_limit)
                flush();
            pending.push_back(0);
            pending_bytes += bag_bytes[0];
        } else {
            flush();
            rev_op.push_back(0);
            rev_grp.push_back(-1);
        }
    }
    flush();
    // Reverse, renumbering the groups in schedule order.
    std::vector<int32_t> renumber((size_t)next_group, -1);
    int32_t seen = 0;
    for (int64_t k = 0; k < n_ops; ++k) {
        const size_t r = (size_t)(n_ops - 1 - k);
        order_out[k] = rev_op[r];
        int32_t g = rev_grp[r];
        if (g >= 0) {
            if (renumber[(size_t)g] < 0)
                renumber[(size_t)g] = seen++;
            g = renumber[(size_t)g];
        }
        group_out[k] = g;
    }
    return ZC_OK;
}

zc_status zc_select_unsharded(const int64_t *bag_bytes, int64_t n, const int64_t *tc_sizes,
                              const double *tc_times, int64_t n_tc, int64_t budget, int32_t *chosen_out,
                              int64_t *n_chosen_out)
{
    using namespace zc;
    if (n < 0 || budget < 0)
        return fail(ZC_ERR_INVALID_ARG, "n and budget must be >= 0");
    if (!n_chosen_out || (n > 0 && (!bag_bytes || !chosen_out)))
        return fail(ZC_ERR_INVALID_ARG, "an input or output table is NULL");
    if (n > 0x7FFFFFFF)
        return fail(ZC_ERR_UNSUPPORTED, "more than 2^31 parameters");
    ZC_TRY(check_comm_table(tc_sizes, tc_times, n_tc));
    for (int64_t i = 0; i < n; ++i)
        if (bag_bytes[i] <= 0)
            return fail(ZC_ERR_INVALID_ARG, "bag_bytes[%lld] must be positive", (long long)i);
    std::vector<int32_t> order((size_t)n);
    std::vector<double> ratio((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        order[(size_t)i] = (int32_t)i;
        ratio[(size_t)i] = comm_time(bag_bytes[i], tc_sizes, tc_times, n_tc) / (double)bag_bytes[i];
    }
    // most communication time saved per byte first; smaller buffers, then earlier ones, among equals
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (ratio[(size_t)a] != ratio[(size_t)b])
            return ratio[(size_t)a] > ratio[(size_t)b];
        if (bag_bytes[a] != bag_bytes[b])
            return bag_bytes[a] < bag_bytes[b];
        return a < b;
    });
    int64_t used = 0, count = 0;
    for (int64_t k = 0; k < n; ++k) {
        const int32_t o = order[(size_t)k];
        if (bag_bytes[o] <= budget - used) {
            chosen_out[count++] = o;
            used += bag_bytes[o];
        }
    }
    *n_chosen_out = count;
    return ZC_OK;
}

zc_status zc_schedule_run(zc_offload_ctx *ctx, const zc_sched_op *ops, int64_t nops, const float *op_ms,
                          int64_t n_ops, const zc_fragment *frags, int64_t nfrags, int32_t poison_freed,
                          void *hip_stream)
{
    using namespace zc;
    if (!ctx)
        return fail(ZC_ERR_INVALID_ARG, "ctx is NULL");
    if (nops < 0 || n_ops < 0 || nfrags < 0)
        return fail(ZC_ERR_INVALID_ARG, "negative count");
    if ((nops > 0 && !ops) || (nfrags > 0 && !frags))
        return fail(ZC_ERR_INVALID_ARG, "ops / frags is NULL");
    ZC_TRY(check_schedule(ops, nops, n_ops, nfrags));
    for (int64_t i = 0; op_ms && i < n_ops; ++i)
        if (!(op_ms[i] >= 0.0f && op_ms[i] <= 10000.0f))
            return fail(ZC_ERR_INVALID_ARG, "op_ms[%lld] must be in [0, 10000]", (long long)i);
    for (int64_t f = 0; f < nfrags; ++f) {
        if (frags[f].bytes < 0 || (frags[f].bytes > 0 && (!frags[f].dev || !frags[f].host)))
            return fail(ZC_ERR_INVALID_ARG, "fragment %lld: bad size or NULL pointer", (long long)f);
        if (frags[f].bytes % 4 != 0 || !aligned_to(frags[f].dev, 4))
            return fail(ZC_ERR_ALIGNMENT, "fragment %lld: size and device pointer must be multiples of 4",
                        (long long)f);
    }
    int dev = 0;
    ZC_HIP(hipGetDevice(&dev));
    if (dev != offload_device(ctx))
        return fail(ZC_ERR_INVALID_ARG, "context belongs to another device");
    int clock_khz = 0;
    ZC_HIP(hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, dev));
    if (clock_khz <= 0)
        clock_khz = 100000;

    hipStream_t stream = (hipStream_t)hip_stream;
    hipStream_t h2d = offload_h2d_stream(ctx), d2h = offload_d2h_stream(ctx);
    // events: [0, nfrags) copy-out done, [nfrags, 2 nfrags) copy-in done, then one marker per copy start
    hipEvent_t *ev = nullptr;
    ZC_TRY(offload_events(ctx, 4 * nfrags, &ev));

    for (int64_t k = 0; k < nops; ++k) {
        const int32_t kind = ops[k].kind, idx = ops[k].index;
        switch (kind) {
        case ZC_OP_COMPUTE: {
            const double ms = op_ms ? (double)op_ms[idx] : 0.0;
            if (ms > 0.0) {
                const uint64_t ticks = (uint64_t)(ms * (double)clock_khz);
                const int64_t max_iters = (int64_t)(ms * 20000.0) + 1000;
                hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, stream, ticks, max_iters);
                ZC_HIP(hipGetLastError());
            }
            break;
        }
        case ZC_OP_OFFLOAD:
            // the copy may start once the caller's stream has reached this point of the schedule
            ZC_HIP(hipEventRecord(ev[2 * nfrags + idx], stream));
            ZC_HIP(hipStreamWaitEvent(d2h, ev[2 * nfrags + idx], 0));
            if (frags[idx].bytes > 0)
                ZC_HIP(hipMemcpyAsync(frags[idx].host, frags[idx].dev, (size_t)frags[idx].bytes,
                                      hipMemcpyDeviceToHost, d2h));
            ZC_HIP(hipEventRecord(ev[idx], d2h));
            break;
        case ZC_OP_SYNC_FREE:
            ZC_HIP(hipStreamWaitEvent(stream, ev[idx], 0));
            if (poison_freed)
                ZC_TRY(launch_poison(frags[idx].dev, frags[idx].bytes / 4, stream));
            break;
        case ZC_OP_RELOAD:
            ZC_HIP(hipEventRecord(ev[3 * nfrags + idx], stream));
            ZC_HIP(hipStreamWaitEvent(h2d, ev[3 * nfrags + idx], 0));
            if (frags[idx].bytes > 0)
                ZC_HIP(hipMemcpyAsync(frags[idx].dev, frags[idx].host, (size_t)frags[idx].bytes,
                                      hipMemcpyHostToDevice, h2d));
            ZC_HIP(hipEventRecord(ev[nfrags + idx], h2d));
            break;
        case ZC_OP_SYNC_RELOAD:
            ZC_HIP(hipStreamWaitEvent(stream, ev[nfrags + idx], 0));
            break;
        default:
            break;
        }
    }
    return ZC_OK;
}

}  // extern "C"

// lagom_overlap_run, lagom_contention_sweep, lagom_overlap_profile: execute one overlap
// group -- communications serialized on one stream, computations on another (Sec. 3.1,
// Eq. 1) -- and time it with HIP events.  This is Alg. 2's ProfileTime and the experiment
// behind Fig. 3.
//
// Both streams are released together: each starts with a short, bounded delay kernel that holds it
// while the host enqueues every launch of both streams.  The kernel on the communication stream picks
// the tick of the constant-rate wall clock at which the hold ends and publishes it through a word of
// pinned host memory; the kernel on the computation stream reads it and holds until the same tick.
// (An event wait across streams instead of the second kernel released the computation stream 6 - 7 us
// after the communication stream, which showed in Z of every computation-bound group.)  The kernels
// therefore run back to back, unaffected by host launch latency, and start at a common instant.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <atomic>
#include <cmath>
#include <mutex>
#include <vector>
#include "common.h"

namespace {

#define HIP_TRY(expr)                                                                               \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess) return lagom::fail(LAGOM_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// Holds a stream for about `ticks` of the constant-rate wall clock.  Every exit condition is
// bounded: the loop ends after `max_iter` sleeps whatever the clock says.
__global__ void gate_delay_kernel(long long ticks, int max_iter) {
    if (threadIdx.x == 0) {
        const long long t0 = wall_clock64();
        for (int i = 0; i < max_iter; ++i) {
            if (wall_clock64() - t0 >= ticks) break;
            __builtin_amdgcn_s_sleep(64);
        }
    }
}

// The start gate of a co-run.  The leader publishes the tick at which both streams go on, then the
// sequence number of this repetition (release); the follower waits for its sequence number (acquire),
// reads the tick and holds until then.  Every loop is bounded by `max_iter` whatever memory or the
// clock say; a follower that never sees its number just ends late.
struct GateWord { unsigned long long deadline; unsigned long long seq; };

__global__ void gate_leader_kernel(GateWord* g, unsigned long long seq, long long ticks, int max_iter) {
    if (threadIdx.x == 0) {
        const long long t0 = wall_clock64();
        __hip_atomic_store(&g->deadline, (unsigned long long)(t0 + ticks), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __hip_atomic_store(&g->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        for (int i = 0; i < max_iter; ++i) {
            if (wall_clock64() - t0 >= ticks) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
}

__global__ void gate_follower_kernel(GateWord* g, unsigned long long seq, int max_iter) {
    if (threadIdx.x == 0) {
        long long deadline = 0;
        bool known = false;
        for (int i = 0; i < max_iter; ++i) {
            if (!known && __hip_atomic_load(&g->seq, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM) == seq) {
                deadline = (long long)__hip_atomic_load(&g->deadline, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                known = true;
            }
            if (known && wall_clock64() - deadline >= 0) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
}

// One gate word of pinned host memory per device, allocated at the first co-run on that device and
// kept until the process ends (16 bytes; pinned host memory, not device memory).
int gate_word(int dev, GateWord** out) {
    static std::mutex mu;
    static std::vector<GateWord*> words;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < 0) return lagom::fail(LAGOM_EINVAL, "bad device %d", dev);
    if ((size_t)dev >= words.size()) words.resize((size_t)dev + 1, nullptr);
    if (!words[dev]) {
        void* p = nullptr;
        HIP_TRY(hipHostMalloc(&p, sizeof(GateWord), hipHostMallocDefault));
        GateWord* w = static_cast<GateWord*>(p);
        w->deadline = 0; w->seq = 0;
        words[dev] = w;
    }
    *out = words[dev];
    return LAGOM_OK;
}

unsigned long long next_gate_seq() {
    static std::atomic<unsigned long long> counter{0};
    return counter.fetch_add(1) + 1;
}

struct Events {
    std::vector<hipEvent_t> ev;
    ~Events() { for (hipEvent_t e : ev) (void)hipEventDestroy(e); }
    int make(int n) {
        for (int i = 0; i < n; ++i) {
            hipEvent_t e;
            HIP_TRY(hipEventCreate(&e));
            ev.push_back(e);
        }
        return LAGOM_OK;
    }
};

double median(std::vector<double>& v) {
    if (v.empty()) return 0.0;
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n & 1 ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
}

// median absolute deviation around `med`
double mad(const std::vector<double>& v, double med) {
    std::vector<double> d(v.size());
    for (size_t i = 0; i < v.size(); ++i) d[i] = std::fabs(v[i] - med);
    return median(d);
}

// After a failure between the first enqueue of a repetition and its end nothing may stay queued on the
// caller's streams (events the streams still wait on are about to be destroyed): drain both, keep the code.
int drained(int rc, hipStream_t sa, hipStream_t sb) {
    if (rc != LAGOM_OK) {
        (void)hipStreamSynchronize(sa);
        (void)hipStreamSynchronize(sb);
    }
    return rc;
}

int validate(const lagom_comm_desc* L, int nlaunch, const lagom_cfg* cfgs, int ncfg,
             const lagom_gemm_desc* G, int ncomp, int mode) {
    if (mode != LAGOM_ALONE_COMM && mode != LAGOM_ALONE_COMP && mode != LAGOM_CORUN)
        return lagom::fail(LAGOM_EINVAL, "unknown mode %d", mode);
    if (nlaunch < 0 || nlaunch > LAGOM_MAX_LAUNCHES || ncomp < 0 || ncomp > LAGOM_MAX_LAUNCHES)
        return lagom::fail(LAGOM_EINVAL, "launch counts outside 0..%d", LAGOM_MAX_LAUNCHES);
    if (ncfg < 0 || ncfg > LAGOM_MAX_COMMS) return lagom::fail(LAGOM_EINVAL, "ncfg outside 0..%d", LAGOM_MAX_COMMS);
    if ((nlaunch > 0 && (!L || !cfgs)) || (ncomp > 0 && !G)) return lagom::fail(LAGOM_EINVAL, "null descriptor array");
    if (mode != LAGOM_ALONE_COMP && nlaunch == 0) return lagom::fail(LAGOM_EINVAL, "no communication to run");
    if (mode != LAGOM_ALONE_COMM && ncomp == 0) return lagom::fail(LAGOM_EINVAL, "no computation to run");
    int prev = -1;
    std::vector<char> seen(ncfg > 0 ? ncfg : 1, 0);
    for (int i = 0; i < nlaunch; ++i) {
        const lagom_comm_desc& d = L[i];
        if (d.comm_id < 0 || d.comm_id >= ncfg) return lagom::fail(LAGOM_EINVAL, "launch %d: comm_id %d outside 0..%d", i, d.comm_id, ncfg - 1);
        if (d.comm_id != prev) {
            if (seen[d.comm_id]) return lagom::fail(LAGOM_EINVAL, "launch %d: launches of communication %d are not contiguous", i, d.comm_id);
            seen[d.comm_id] = 1;
            prev = d.comm_id;
        }
        if (d.after_comp < -1 || d.after_comp >= ncomp) return lagom::fail(LAGOM_EINVAL, "launch %d: after_comp %d outside -1..%d", i, d.after_comp, ncomp - 1);
        if (int rc = lagom::check_comm_args(d.op, d.dtype, d.srcs, d.nsrc, d.dsts, d.ndst, d.count)) return rc;
        if (d.lds_staged && (d.fuse_with_prev || (i + 1 < nlaunch && L[i + 1].fuse_with_prev)))
            return lagom::fail(LAGOM_EINVAL, "launch %d: a launch staged through LDS cannot be part of a fused run", i);
        if (d.fuse_with_prev) {
            if (i == 0 || L[i - 1].comm_id != d.comm_id || L[i - 1].dtype != d.dtype || L[i - 1].count != d.count || d.after_comp != -1)
                return lagom::fail(LAGOM_EINVAL, "launch %d: fuse_with_prev needs a previous launch of the same communication, dtype and count, and no dependency of its own", i);
        }
    }
    // every run of fused launches must be a valid lagom_comm_steps call
    for (int i = 0; i < nlaunch;) {
        int k = i + 1;
        while (k < nlaunch && L[k].fuse_with_prev) ++k;
        if (k - i > 1) {
            std::vector<lagom_comm_step> steps;
            for (int q = i; q < k; ++q) steps.push_back(lagom_comm_step{L[q].op, L[q].srcs, L[q].nsrc, L[q].dsts, L[q].ndst});
            if (int rc = lagom::check_comm_steps(L[i].dtype, steps.data(), k - i, L[i].count)) return rc;
        }
        i = k;
    }
    for (int j = 0; j < ncfg; ++j)
        if (int rc = lagom::check_cfg(&cfgs[j])) return rc;
    for (int i = 0; i < ncomp; ++i) {
        const lagom_gemm_desc& g = G[i];
        if (g.after_comm_id < -1 || g.after_comm_id >= ncfg || (g.after_comm_id >= 0 && !seen[g.after_comm_id]))
            return lagom::fail(LAGOM_EINVAL, "computation %d: after_comm_id %d names no communication of the group", i, g.after_comm_id);
        if (int rc = lagom::check_gemm_args(g.A, g.B, g.C, g.M, g.N, g.K, g.out_dtype)) return rc;
    }
    return LAGOM_OK;
}

// Launches of one communication form a group; groups and computations are what dependencies name.
struct GroupPlan {
    std::vector<int> first, last, id, of;   // per group: first / last launch, comm_id; per comm_id: its group
    int n = 0;
    void build(const lagom_comm_desc* launches, int nlaunch, int ncfg) {
        of.assign(ncfg > 0 ? ncfg : 1, -1);
        for (int i = 0; i < nlaunch; ++i) {
            if (i == 0 || launches[i].comm_id != launches[i - 1].comm_id) {
                of[launches[i].comm_id] = (int)first.size();
                first.push_back(i); last.push_back(i); id.push_back(launches[i].comm_id);
            } else {
                last.back() = i;
            }
        }
        n = (int)first.size();
    }
};

// Enqueues one repetition of the group: nl launches on sa, nc computations on sb.  The two enqueue
// orders are merged so that an awaited event has always been recorded first; a dependency cycle
// drains both streams and is LAGOM_EINVAL.  ga_start / gb_start may be null (no per-operator timing).
int enqueue_group(const GroupPlan& plan, const lagom_comm_desc* launches, int nl, const lagom_cfg* cfgs,
                  const lagom_gemm_desc* comps, int nc, bool deps, hipStream_t sa, hipStream_t sb,
                  hipEvent_t* ga_start, hipEvent_t* ga_end, hipEvent_t* gb_start, hipEvent_t* gb_end) {
    std::vector<char> group_done(plan.n > 0 ? plan.n : 1, 0), comp_done(nc > 0 ? nc : 1, 0);
    int li = 0, ci = 0;
    while (li < nl || ci < nc) {
        bool progressed = false;
        if (li < nl) {
            const lagom_comm_desc& d = launches[li];
            const int dep = deps ? d.after_comp : -1;
            if (dep < 0 || comp_done[dep]) {
                const int g = plan.of[d.comm_id];
                if (dep >= 0) HIP_TRY(hipStreamWaitEvent(sa, gb_end[dep], 0));
                if (ga_start && li == plan.first[g]) HIP_TRY(hipEventRecord(ga_start[g], sa));
                int run = 1;                                   // this launch and the ones fused to it
                while (li + run < nl && launches[li + run].fuse_with_prev) ++run;
                if (run == 1 && d.lds_staged) {
                    if (int rc = lagom_comm_kernel_lds((lagom_op)d.op, (lagom_dtype)d.dtype, d.srcs, d.nsrc, d.dsts, d.ndst,
                                                       d.count, &cfgs[d.comm_id], sa)) return rc;
                } else if (run == 1) {
                    if (int rc = lagom_comm_kernel((lagom_op)d.op, (lagom_dtype)d.dtype, d.srcs, d.nsrc, d.dsts, d.ndst,
                                                   d.count, &cfgs[d.comm_id], sa)) return rc;
                } else {
                    lagom_comm_step steps[LAGOM_MAX_STEPS];
                    for (int q = 0; q < run; ++q) {
                        const lagom_comm_desc& e = launches[li + q];
                        steps[q] = lagom_comm_step{e.op, e.srcs, e.nsrc, e.dsts, e.ndst};
                    }
                    if (int rc = lagom_comm_steps((lagom_dtype)d.dtype, steps, run, d.count, &cfgs[d.comm_id], sa)) return rc;
                }
                li += run;
                if (li - 1 == plan.last[g]) { HIP_TRY(hipEventRecord(ga_end[g], sa)); group_done[g] = 1; }
                progressed = true;
            }
        }
        if (ci < nc) {
            const lagom_gemm_desc& c = comps[ci];
            const int dep = deps ? c.after_comm_id : -1;
            if (dep < 0 || group_done[plan.of[dep]]) {
                if (dep >= 0) HIP_TRY(hipStreamWaitEvent(sb, ga_end[plan.of[dep]], 0));
                if (gb_start) HIP_TRY(hipEventRecord(gb_start[ci], sb));
                if (int rc = lagom_gemm(c.A, c.B, c.C, c.M, c.N, c.K, c.b_is_nk, (lagom_dtype)c.out_dtype, sb)) return rc;
                HIP_TRY(hipEventRecord(gb_end[ci], sb));
                comp_done[ci] = 1;
                ++ci;
                progressed = true;
            }
        }
        if (!progressed) {
            // nothing of this repetition may stay queued: drain, then report
            (void)hipStreamSynchronize(sa);
            (void)hipStreamSynchronize(sb);
            return lagom::fail(LAGOM_EINVAL, "the cross-stream dependencies form a cycle (launch %d, computation %d)", li, ci);
        }
    }
    return LAGOM_OK;
}

int require_overlap(hipStream_t sa, hipStream_t sb) {
    if (sa == sb) return lagom::fail(LAGOM_EINVAL, "co-run needs two distinct streams");
    int overlap = 0;
    if (int rc = lagom_streams_overlap(sa, sb, &overlap)) return rc;
    if (!overlap)
        return lagom::fail(LAGOM_EINVAL, "kernels on the two streams do not run at the same time (HIP maps streams onto a few "
                                         "hardware queues and these two share one): pick another pair, see lagom_streams_overlap");
    return LAGOM_OK;
}

}  // namespace

// Two bounded delay kernels, a long one on stream a and, behind a common event, a short one on
// stream b: on separate hardware queues the short one ends before the long one does, on a shared
// queue it cannot start until the long one has ended.  The long kernel has to outlast the host's
// submission of the short one; a verdict of "shared" is therefore confirmed with a ten times longer one.
extern "C" int lagom_streams_overlap(void* stream_a, void* stream_b, int* overlap) {
    if (!overlap) return lagom::fail(LAGOM_EINVAL, "null output");
    hipStream_t sa = static_cast<hipStream_t>(stream_a), sb = static_cast<hipStream_t>(stream_b);
    *overlap = 0;
    if (sa == sb) return LAGOM_OK;
    int dev = 0, clock_khz = 100000;
    HIP_TRY(hipGetDevice(&dev));
    if (hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || clock_khz <= 0) clock_khz = 100000;
    Events E;
    if (int rc = E.make(3)) return rc;
    for (const double long_us : {300.0, 3000.0}) {
        HIP_TRY(hipEventRecord(E.ev[0], sa));
        HIP_TRY(hipStreamWaitEvent(sb, E.ev[0], 0));
        hipLaunchKernelGGL(gate_delay_kernel, dim3(1), dim3(64), 0, sa, (long long)(long_us * clock_khz / 1000.0), 1 << 14);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(E.ev[1], sa));
        hipLaunchKernelGGL(gate_delay_kernel, dim3(1), dim3(64), 0, sb, (long long)(1.0 * clock_khz / 1000.0), 1 << 14);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipEventRecord(E.ev[2], sb));
        HIP_TRY(hipStreamSynchronize(sa));
        HIP_TRY(hipStreamSynchronize(sb));
        float ta = 0.f, tb = 0.f;
        HIP_TRY(hipEventElapsedTime(&ta, E.ev[0], E.ev[1]));
        HIP_TRY(hipEventElapsedTime(&tb, E.ev[0], E.ev[2]));
        if (tb < ta) { *overlap = 1; break; }
    }
    return LAGOM_OK;
}

extern "C" int lagom_overlap_run(const lagom_comm_desc* launches, int nlaunch, const lagom_cfg* cfgs, int ncfg,
                                 const lagom_gemm_desc* comps, int ncomp, void* comm_stream, void* comp_stream,
                                 int warmup, int iters, int mode, lagom_timing* out) {
    if (!out) return lagom::fail(LAGOM_EINVAL, "null output");
    if (warmup < 0 || iters < 1 || iters > 100000) return lagom::fail(LAGOM_EINVAL, "warmup >= 0 and 1 <= iters <= 100000 required");
    if (int rc = validate(launches, nlaunch, cfgs, ncfg, comps, ncomp, mode)) return rc;
    const bool run_comm = mode != LAGOM_ALONE_COMP, run_comp = mode != LAGOM_ALONE_COMM;
    hipStream_t sa = static_cast<hipStream_t>(comm_stream), sb = static_cast<hipStream_t>(comp_stream);
    if (run_comm && run_comp)
        if (int rc = require_overlap(sa, sb)) return rc;

    // every group of launches and every GEMM gets a start and an end event
    GroupPlan plan;
    if (run_comm) plan.build(launches, nlaunch, ncfg);
    const int ngroups = plan.n;
    const std::vector<int>& group_id = plan.id;
    const int ncomp_run = run_comp ? ncomp : 0;
    const bool deps = run_comm && run_comp;        // dependencies only matter when both streams run
    Events E;
    if (int rc = E.make(2 * ngroups + 2 * ncomp_run)) return rc;
    hipEvent_t* ga_start = E.ev.data();
    hipEvent_t* ga_end = ga_start + ngroups;
    hipEvent_t* gb_start = ga_end + ngroups;
    hipEvent_t* gb_end = gb_start + ncomp_run;

    int dev = 0, clock_khz = 100000;
    HIP_TRY(hipGetDevice(&dev));
    if (hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || clock_khz <= 0) clock_khz = 100000;
    // long enough for the host to enqueue everything: ~12 us per queued item plus a floor
    const int items = (run_comm ? nlaunch + 2 * ngroups : 0) + 3 * ncomp_run + 4;
    const double delay_us = 60.0 + 12.0 * items;
    const long long ticks = (long long)(delay_us * clock_khz / 1000.0);
    // a pass of the gates' loops takes 0.3 - 0.4 us: several times the passes the delay needs, and no more
    const int max_iter = (int)std::min(8.0 * delay_us + 4096.0, 4.0e6);
    GateWord* word = nullptr;
    if (run_comm && run_comp)
        if (int rc = gate_word(dev, &word)) return rc;

    std::vector<std::vector<double>> xs(ncfg), ys(ncomp);
    std::vector<double> Xs, Ys, Zs, startsA, startsB;
    hipStream_t gate_stream = run_comm ? sa : sb;

    std::vector<double> Ysums;
    // one repetition: gate, both streams enqueued, both drained
    auto repetition = [&]() -> int {
        if (word) {
            const unsigned long long seq = next_gate_seq();
            hipLaunchKernelGGL(gate_leader_kernel, dim3(1), dim3(64), 0, sa, word, seq, ticks, max_iter);
            HIP_TRY(hipGetLastError());
            hipLaunchKernelGGL(gate_follower_kernel, dim3(1), dim3(64), 0, sb, word, seq, max_iter);
            HIP_TRY(hipGetLastError());
        } else {
            hipLaunchKernelGGL(gate_delay_kernel, dim3(1), dim3(64), 0, gate_stream, ticks, max_iter);
            HIP_TRY(hipGetLastError());
        }
        if (int rc = enqueue_group(plan, launches, run_comm ? nlaunch : 0, cfgs, comps, ncomp_run, deps, sa, sb,
                                   ga_start, ga_end, gb_start, gb_end)) return rc;
        if (run_comm) HIP_TRY(hipStreamSynchronize(sa));
        if (run_comp) HIP_TRY(hipStreamSynchronize(sb));
        return LAGOM_OK;
    };
    for (int it = 0; it < warmup + iters; ++it) {
        if (int rc = drained(repetition(), sa, sb)) return rc;
        if (it < warmup) continue;

        // The common start: the start event of the stream whose first kernel follows its gate kernel directly.  With
        // cross-stream dependencies the other stream's first start event is recorded behind a wait; without them the
        // two are the instants at which the two gates opened, and the earlier one is taken.  (No event of its own
        // behind the gate kernel: two event records in a row on one stream lie 5 us apart.)
        float ms = 0.f;
        double X = 0.0, Y = 0.0, endA = 0.0, endB = 0.0, ysum = 0.0;
        hipEvent_t origin = run_comm ? ga_start[0] : gb_start[0];
        if (run_comm && run_comp) {
            HIP_TRY(hipEventElapsedTime(&ms, ga_start[0], gb_start[0]));
            if (ms < 0.f) origin = gb_start[0];
        }
        if (run_comm) {
            for (int g = 0; g < ngroups; ++g) {
                HIP_TRY(hipEventElapsedTime(&ms, ga_start[g], ga_end[g]));
                xs[group_id[g]].push_back((double)ms * 1000.0);
            }
            HIP_TRY(hipEventElapsedTime(&ms, ga_start[0], ga_end[ngroups - 1])); X = (double)ms * 1000.0;
            HIP_TRY(hipEventElapsedTime(&ms, origin, ga_end[ngroups - 1])); endA = (double)ms * 1000.0;
            HIP_TRY(hipEventElapsedTime(&ms, origin, ga_start[0])); startsA.push_back((double)ms * 1000.0);
        }
        if (run_comp) {
            for (int i = 0; i < ncomp; ++i) {
                HIP_TRY(hipEventElapsedTime(&ms, gb_start[i], gb_end[i]));
                ys[i].push_back((double)ms * 1000.0);
                ysum = ysum + (double)ms * 1000.0;
            }
            HIP_TRY(hipEventElapsedTime(&ms, gb_start[0], gb_end[ncomp - 1])); Y = (double)ms * 1000.0;
            HIP_TRY(hipEventElapsedTime(&ms, origin, gb_end[ncomp - 1])); endB = (double)ms * 1000.0;
            HIP_TRY(hipEventElapsedTime(&ms, origin, gb_start[0])); startsB.push_back((double)ms * 1000.0);
        }
        Xs.push_back(X); Ys.push_back(Y); Zs.push_back(endA > endB ? endA : endB); Ysums.push_back(ysum);
    }
    out->X_us = median(Xs);
    out->Y_us = median(Ys);
    out->Z_us = median(Zs);
    out->Z_mad_us = mad(Zs, out->Z_us);
    out->Ysum_us = median(Ysums);
    out->Ysum_mad_us = mad(Ysums, out->Ysum_us);
    out->comm_start_us = startsA.empty() ? 0.0 : median(startsA);
    out->comp_start_us = startsB.empty() ? 0.0 : median(startsB);
    for (int j = 0; j < ncfg; ++j) {
        const double m = median(xs[j]);
        if (out->x_us) out->x_us[j] = m;
        if (out->x_mad_us) out->x_mad_us[j] = mad(xs[j], m);
    }
    if (out->y_us) for (int i = 0; i < ncomp; ++i) out->y_us[i] = median(ys[i]);
    return LAGOM_OK;
}

// Sustained rate of the group: repetitions enqueued back to back, joined through events only.
extern "C" int lagom_overlap_steps(const lagom_comm_desc* launches, int nlaunch, const lagom_cfg* cfgs, int ncfg,
                                   const lagom_gemm_desc* comps, int ncomp, void* comm_stream, void* comp_stream,
                                   int steps, double* us_per_step) {
    if (!us_per_step) return lagom::fail(LAGOM_EINVAL, "null output");
    if (steps < 1 || steps > 100000) return lagom::fail(LAGOM_EINVAL, "1 <= steps <= 100000 required");
    if (int rc = validate(launches, nlaunch, cfgs, ncfg, comps, ncomp, LAGOM_CORUN)) return rc;
    hipStream_t sa = static_cast<hipStream_t>(comm_stream), sb = static_cast<hipStream_t>(comp_stream);
    if (int rc = require_overlap(sa, sb)) return rc;
    GroupPlan plan;
    plan.build(launches, nlaunch, ncfg);
    Events E;
    if (int rc = E.make(4 + plan.n + ncomp)) return rc;
    hipEvent_t t_start = E.ev[0], t_end = E.ev[1], end_a = E.ev[2], end_b = E.ev[3];
    hipEvent_t* ga_end = E.ev.data() + 4;
    hipEvent_t* gb_end = ga_end + plan.n;

    int dev = 0, clock_khz = 100000;
    HIP_TRY(hipGetDevice(&dev));
    if (hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || clock_khz <= 0) clock_khz = 100000;
    // a head start for the host: the device begins the first repetition while later ones are still being enqueued
    hipLaunchKernelGGL(gate_delay_kernel, dim3(1), dim3(64), 0, sa, (long long)(200.0 * clock_khz / 1000.0), 1 << 14);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(t_start, sa));
    HIP_TRY(hipStreamWaitEvent(sb, t_start, 0));
    for (int it = 0; it < steps; ++it) {
        // the events are re-recorded every repetition: a wait refers to the record that preceded it
        auto repetition = [&]() -> int {
            if (int rc = enqueue_group(plan, launches, nlaunch, cfgs, comps, ncomp, true, sa, sb, nullptr, ga_end, nullptr, gb_end)) return rc;
            HIP_TRY(hipEventRecord(end_a, sa));
            HIP_TRY(hipEventRecord(end_b, sb));
            HIP_TRY(hipStreamWaitEvent(sa, end_b, 0));   // the next repetition starts when this one has ended on both streams
            HIP_TRY(hipStreamWaitEvent(sb, end_a, 0));
            return LAGOM_OK;
        };
        if (int rc = drained(repetition(), sa, sb)) return rc;
    }
    if (int rc = drained([&]() -> int { HIP_TRY(hipEventRecord(t_end, sa)); return LAGOM_OK; }(), sa, sb)) return rc;
    HIP_TRY(hipStreamSynchronize(sa));
    HIP_TRY(hipStreamSynchronize(sb));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, t_start, t_end));
    *us_per_step = (double)ms * 1000.0 / (double)steps;
    return LAGOM_OK;
}

// The same repetitions replayed from a HIP graph: one repetition is captured from both streams (fork and
// join through events) and launched `steps` times on the communication stream.
extern "C" int lagom_overlap_steps_graph(const lagom_comm_desc* launches, int nlaunch, const lagom_cfg* cfgs, int ncfg,
                                         const lagom_gemm_desc* comps, int ncomp, void* comm_stream, void* comp_stream,
                                         int steps, double* us_per_step) {
    if (!us_per_step) return lagom::fail(LAGOM_EINVAL, "null output");
    if (steps < 1 || steps > 100000) return lagom::fail(LAGOM_EINVAL, "1 <= steps <= 100000 required");
    if (int rc = validate(launches, nlaunch, cfgs, ncfg, comps, ncomp, LAGOM_CORUN)) return rc;
    hipStream_t sa = static_cast<hipStream_t>(comm_stream), sb = static_cast<hipStream_t>(comp_stream);
    if (int rc = require_overlap(sa, sb)) return rc;
    GroupPlan plan;
    plan.build(launches, nlaunch, ncfg);
    Events E;
    if (int rc = E.make(4 + plan.n + ncomp)) return rc;
    hipEvent_t t_start = E.ev[0], t_end = E.ev[1], fork = E.ev[2], join = E.ev[3];
    hipEvent_t* ga_end = E.ev.data() + 4;
    hipEvent_t* gb_end = ga_end + plan.n;

    // One eager repetition first: kernel attributes are set and code objects loaded outside the capture,
    // and a dependency cycle is reported here, where the streams may still be synchronised.
    HIP_TRY(hipEventRecord(fork, sa));
    HIP_TRY(hipStreamWaitEvent(sb, fork, 0));
    if (int rc = drained(enqueue_group(plan, launches, nlaunch, cfgs, comps, ncomp, true, sa, sb, nullptr, ga_end, nullptr, gb_end), sa, sb)) return rc;
    HIP_TRY(hipStreamSynchronize(sa));
    HIP_TRY(hipStreamSynchronize(sb));

    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    HIP_TRY(hipStreamBeginCapture(sa, hipStreamCaptureModeThreadLocal));
    int rc = LAGOM_OK;
    hipError_t he = hipEventRecord(fork, sa);
    if (he == hipSuccess) he = hipStreamWaitEvent(sb, fork, 0);
    if (he == hipSuccess) rc = enqueue_group(plan, launches, nlaunch, cfgs, comps, ncomp, true, sa, sb, nullptr, ga_end, nullptr, gb_end);
    if (he == hipSuccess && rc == LAGOM_OK) he = hipEventRecord(join, sb);
    if (he == hipSuccess && rc == LAGOM_OK) he = hipStreamWaitEvent(sa, join, 0);
    const hipError_t he_end = hipStreamEndCapture(sa, &graph);      // always: the streams must leave capture mode
    if (rc != LAGOM_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (he != hipSuccess || he_end != hipSuccess || !graph) {
        if (graph) (void)hipGraphDestroy(graph);
        return lagom::fail(LAGOM_EHIP, "graph capture of the overlap group: %s", hipGetErrorString(he != hipSuccess ? he : he_end));
    }
    he = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (he != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return lagom::fail(LAGOM_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(he));
    }
    he = hipEventRecord(t_start, sa);
    for (int it = 0; it < steps && he == hipSuccess; ++it) he = hipGraphLaunch(exec, sa);
    if (he == hipSuccess) he = hipEventRecord(t_end, sa);
    const hipError_t hs = hipStreamSynchronize(sa);
    float ms = 0.f;
    if (he == hipSuccess && hs == hipSuccess) he = hipEventElapsedTime(&ms, t_start, t_end);
    (void)hipGraphExecDestroy(exec);
    (void)hipGraphDestroy(graph);
    if (he != hipSuccess || hs != hipSuccess)
        return lagom::fail(LAGOM_EHIP, "graph replay of the overlap group: %s", hipGetErrorString(he != hipSuccess ? he : hs));
    *us_per_step = (double)ms * 1000.0 / (double)steps;
    return LAGOM_OK;
}

extern "C" int lagom_contention_sweep(const lagom_comm_desc* launches, int nlaunch, int ncfg,
                                      const lagom_gemm_desc* comps, int ncomp, const lagom_cfg* points, int npoints,
                                      void* comm_stream, void* comp_stream, int warmup, int iters, lagom_sweep_point* out) {
    if (!points || !out || npoints < 1) return lagom::fail(LAGOM_EINVAL, "need at least one sweep point and an output array");
    if (ncfg < 1 || ncfg > LAGOM_MAX_COMMS || nlaunch < 1 || ncomp < 1) return lagom::fail(LAGOM_EINVAL, "need communications and computations");
    double bytes = 0.0;
    for (int i = 0; i < nlaunch; ++i) {
        const int64_t b = lagom_comm_bytes(launches[i].op, launches[i].dtype, launches[i].nsrc, launches[i].ndst, launches[i].count);
        if (b < 0) return lagom::fail(LAGOM_EINVAL, "launch %d: bad descriptor", i);
        bytes += (double)b;
    }
    std::vector<lagom_cfg> cfgs(ncfg, points[0]);
    // X and Y of a sweep point are the sums of the per-operator times (Eq. 1), so that a wait for the
    // other stream is not counted as communication or computation time
    std::vector<double> xj(ncfg), yi(ncomp);
    lagom_timing t{};
    t.x_us = xj.data();
    t.y_us = yi.data();
    auto sum = [](const std::vector<double>& v) { double s = 0.0; for (double e : v) s = s + e; return s; };
    if (int rc = lagom_overlap_run(launches, nlaunch, cfgs.data(), ncfg, comps, ncomp, comm_stream, comp_stream,
                                   warmup, iters, LAGOM_ALONE_COMP, &t)) return rc;
    double comp_alone = sum(yi);
    for (int p = 0; p < npoints; ++p) {
        std::fill(cfgs.begin(), cfgs.end(), points[p]);
        lagom_sweep_point& o = out[p];
        o.cfg = points[p];
        if (p > 0 && p % 8 == 0) {   // the clock the chip holds drifts over a long sweep: refresh the reference
            if (int rc = lagom_overlap_run(launches, nlaunch, cfgs.data(), ncfg, comps, ncomp, comm_stream, comp_stream,
                                           warmup, iters, LAGOM_ALONE_COMP, &t)) return rc;
            comp_alone = sum(yi);
        }
        o.comp_alone_us = comp_alone;
        if (int rc = lagom_overlap_run(launches, nlaunch, cfgs.data(), ncfg, comps, ncomp, comm_stream, comp_stream,
                                       warmup, iters, LAGOM_ALONE_COMM, &t)) return rc;
        o.comm_alone_us = sum(xj);
        if (int rc = lagom_overlap_run(launches, nlaunch, cfgs.data(), ncfg, comps, ncomp, comm_stream, comp_stream,
                                       warmup, iters, LAGOM_CORUN, &t)) return rc;
        o.comm_corun_us = sum(xj);
        o.comp_corun_us = sum(yi);
        o.z_corun_us = t.Z_us;
        o.v_alone = o.comm_alone_us > 0.0 ? bytes / o.comm_alone_us : 0.0;
        o.v_corun = o.comm_corun_us > 0.0 ? bytes / o.comm_corun_us : 0.0;
    }
    return LAGOM_OK;
}

extern "C" int lagom_overlap_profile(void* user, const lagom_cfg* cfgs, int ncomm, double* x_us, double* Y_us) {
    if (!user || !cfgs || !x_us || !Y_us) return lagom::fail(LAGOM_EINVAL, "null argument");
    const lagom_overlap_ctx* c = static_cast<const lagom_overlap_ctx*>(user);
    if (c->ncomp < 0 || c->ncomp > LAGOM_MAX_LAUNCHES) return lagom::fail(LAGOM_EINVAL, "ncomp=%d out of range", c->ncomp);
    if (ncomm < 1 || ncomm > LAGOM_MAX_COMMS) return lagom::fail(LAGOM_EINVAL, "ncomm=%d out of range", ncomm);
    std::vector<double> yi((size_t)c->ncomp), xmad((size_t)ncomm);
    lagom_timing t{};
    t.x_us = x_us;
    t.y_us = yi.data();
    t.x_mad_us = xmad.data();
    int iters = c->iters;
    int rc = lagom_overlap_run(c->launches, c->nlaunch, cfgs, ncomm, c->comps, c->ncomp, c->comm_stream, c->comp_stream,
                               c->warmup, iters, LAGOM_CORUN, &t);
    if (rc) return rc;
    if (c->min_total_us > 0.0 && t.Z_us > 0.0 && (double)iters * t.Z_us < c->min_total_us) {
        // a short group: the repetitions asked for do not average enough out; measure again, longer
        const double want = std::ceil(c->min_total_us / t.Z_us);
        const int cap = c->max_iters > iters ? c->max_iters : iters;
        iters = want < (double)cap ? (int)want : cap;
        rc = lagom_overlap_run(c->launches, c->nlaunch, cfgs, ncomm, c->comps, c->ncomp, c->comm_stream, c->comp_stream,
                               0, iters, LAGOM_CORUN, &t);
        if (rc) return rc;
    }
    double Y = 0.0;   // Eq. 1: Y is the sum of the y_i (a GEMM's wait for a communication is not computation time)
    for (double y : yi) Y = Y + y;
    *Y_us = Y;
    if (lagom_profile_log* g = c->log) {
        if (g->n < g->capacity && g->ncomm == ncomm) {
            const int64_t row = (int64_t)g->n * ncomm;
            for (int j = 0; j < ncomm; ++j) {
                if (g->cfgs) g->cfgs[row + j] = cfgs[j];
                if (g->x_us) g->x_us[row + j] = x_us[j];
                if (g->x_mad_us) g->x_mad_us[row + j] = xmad[j];
            }
            if (g->Y_us) g->Y_us[g->n] = Y;
            if (g->Y_mad_us) g->Y_mad_us[g->n] = t.Ysum_mad_us;
            if (g->Z_us) g->Z_us[g->n] = t.Z_us;
            if (g->Z_mad_us) g->Z_mad_us[g->n] = t.Z_mad_us;
            if (g->iters) g->iters[g->n] = iters;
        }
        g->n += 1;
    }
    return LAGOM_OK;
}

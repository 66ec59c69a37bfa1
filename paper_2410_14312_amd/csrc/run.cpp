// One-GPU pipeline emulator: K stages on K HIP streams, tasks issued in nF1B order, cross-stage
// dependencies as events (sections "Work Scheduling" and "Overlapping of Computation and
// Communication": what would be a message between workers is an event between streams here).
//
// Each stage has its own host thread that issues that stage's tasks in schedule order on the stage's
// stream, like a worker process would; a thread that needs another stage's result first waits until
// the producing thread has recorded the event, then makes its stream wait for it.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <shared_mutex>
#include <thread>
#include <vector>

#include "profile.h"
#include "schedule.h"
#include "stage.h"

using namespace tmps;

namespace {

// The events that stand for messages between workers are kept by the stage that records them (tmps_stage::events,
// destroyed with the stage): a second run on the same stages creates none.
int grow_events(tmps_stage* st, size_t n) {
    while (st->events.size() < n) {
        hipEvent_t e;
        TMPS_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        st->events.push_back(e);
    }
    return TMPS_OK;
}

struct RunCtx {
    bool vsync = false;              // forward passes read the weight version they are tagged with
    bool one_f1b = false;            // the comparison system: a backward pass per batch, on the weights of its forward pass
    std::vector<long> base_version;  // every stage's version when the run started
    tmps_stage** stages;
    int K, N, M, mb, n_minibatches;
    const void* inputs;
    const int32_t* labels;
    void** streams;
    float* losses_out;
    int32_t* log;
    size_t asz, total_micro, n_fwd_ev;
    std::vector<int> groups;
    std::vector<std::atomic<unsigned char>> recorded;
    std::atomic<int> err{TMPS_OK};
    char err_text[512];
    std::atomic_flag err_lock = ATOMIC_FLAG_INIT;

    size_t fwd_ev(int s, size_t q) const { return (size_t)s * total_micro + q; }
    size_t bwd_ev(int s, int b0) const { return n_fwd_ev + (size_t)s * n_minibatches + b0; }
    // the event behind an index: stage s keeps its forward events first, then its backward events
    hipEvent_t event(size_t e) const {
        if (e < n_fwd_ev) return stages[e / total_micro]->events[e % total_micro];
        const size_t r = e - n_fwd_ev;
        return stages[r / n_minibatches]->events[total_micro + r % n_minibatches];
    }

    // Block until the producer thread has recorded event e (or a thread failed), then make stream s wait for it.
    int wait_for(size_t e, hipStream_t s) {
        while (!recorded[e].load(std::memory_order_acquire)) {
            if (err.load(std::memory_order_relaxed) != TMPS_OK) return TMPS_EINVAL;
            std::this_thread::yield();
        }
        std::shared_lock<std::shared_mutex> no_capture(capture_lock());   // (see capture_lock)
        TMPS_HIP(hipStreamWaitEvent(s, event(e), 0));
        return TMPS_OK;
    }
    int record(size_t e, hipStream_t s) {
        TMPS_HIP(hipEventRecord(event(e), s));
        recorded[e].store(1, std::memory_order_release);
        return TMPS_OK;
    }
    void set_error(int rc) {
        while (err_lock.test_and_set(std::memory_order_acquire)) {}
        if (err.load() == TMPS_OK) {
            strncpy(err_text, tmps_last_error(), sizeof(err_text) - 1);
            err_text[sizeof(err_text) - 1] = 0;
            err.store(rc);
        }
        err_lock.clear(std::memory_order_release);
    }
};

// Issue one task on its stage's stream.
int issue(RunCtx& c, const Task& k, size_t ti) {
    tmps_stage* st = c.stages[k.stage];
    hipStream_t s = (hipStream_t)c.streams[k.stage];
    const int b0 = k.b - 1, N = c.N, K = c.K;
    if (c.log) {
        int32_t* o = c.log + 7 * ti;
        o[0] = k.t; o[1] = k.stage; o[2] = k.kind; o[3] = k.b; o[4] = k.j;
        const int32_t live = (int32_t)(st->version - c.base_version[k.stage]);
        if (c.one_f1b) {   // version the task reads (a backward pass: the one its forward pass read), version the worker is at
            o[5] = k.kind == kFwd ? live : k.stage_version;
            o[6] = live;
        } else {
            o[5] = live;
            o[6] = k.net_version;
        }
    }
    const int group = b0 % c.groups[k.stage];
    int rc;
    if (k.kind == kFwd) {
        const int j = k.j < 0 ? 0 : k.j;   // (the comparison system has no micro-batches: N = 1)
        const size_t q = (size_t)b0 * N + j;
        const int slot = group * N + j;
        const void* x;
        if (k.stage == 0) {
            x = (const char*)c.inputs + ((size_t)b0 * c.M + (size_t)j * c.mb) * st->in_elems * st->in_esize;
        } else {
            x = tmps_stage_output_ptr(c.stages[k.stage - 1], (b0 % c.groups[k.stage - 1]) * N + j);
            if ((rc = c.wait_for(c.fwd_ev(k.stage - 1, q), s)) != TMPS_OK) return rc;
        }
        const int32_t* lab = st->cfg.is_last ? c.labels + ((size_t)b0 * c.M + (size_t)j * c.mb) * st->label_rps : nullptr;
        if (c.vsync)
            rc = tmps_forward_micro_at(st, c.base_version[k.stage] + k.net_version, slot, x, nullptr, lab, nullptr, s);
        else
            rc = tmps_forward_micro(st, slot, x, nullptr, lab, nullptr, s);
        if (rc != TMPS_OK) return rc;
        if (k.stage < K - 1 && (rc = c.record(c.fwd_ev(k.stage, q), s)) != TMPS_OK) return rc;
        if (st->cfg.is_last && j == N - 1 && c.losses_out) {
            ProfileScope scope(kcReduce, s);
            const int rows = c.M * st->label_rps;
            TMPS_HIP(reduce_scaled_sum(stage_row_loss(st, group * N), rows, 1.0f / (float)rows, c.losses_out + b0, s));
        }
    } else {
        const void* dy = nullptr;
        if (k.stage < K - 1) {
            dy = stage_dxout(c.stages[k.stage + 1], b0 & 1);
            if ((rc = c.wait_for(c.bwd_ev(k.stage + 1, b0), s)) != TMPS_OK) return rc;
        }
        void* dx = nullptr;
        if (k.stage > 0) {
            dx = stage_dxout(st, b0 & 1);
            // the worker below must have consumed what this buffer held two mini-batches ago
            if (b0 >= 2 && (rc = c.wait_for(c.bwd_ev(k.stage - 1, b0 - 2), s)) != TMPS_OK) return rc;
        }
        int slots[64];
        for (int j = 0; j < N; ++j) slots[j] = group * N + j;
        if (c.one_f1b)   // horizontal weight stashing: differentiate at the weights the forward pass read
            rc = tmps_backward_at(st, c.base_version[k.stage] + k.stage_version, slots, N, dy, dx, s);
        else
            rc = tmps_backward(st, slots, N, dy, dx, s);
        if (rc != TMPS_OK) return rc;
        if ((rc = c.record(c.bwd_ev(k.stage, b0), s)) != TMPS_OK) return rc;
        if ((rc = tmps_update(st, s)) != TMPS_OK) return rc;
    }
    return TMPS_OK;
}

}  // namespace

enum { kModeInPlace = 0, kModeVsync = 1, kMode1F1B = 2 };

static int schedule_run(tmps_stage** stages, int K, int N, int n_minibatches, const void* inputs, const int32_t* labels,
                        void** hip_streams, float* losses_out, int32_t* version_log_out, int mode) {
    const bool vsync = mode == kModeVsync, one_f1b = mode == kMode1F1B;
    if (!stages || !hip_streams || !inputs || !labels) return fail(TMPS_EINVAL, "null argument");
    if (K < 1 || N < 1 || n_minibatches < 1) return fail(TMPS_EINVAL, "K, N and n_minibatches must be positive");
    const int mb = stages[0] ? stages[0]->cfg.micro_batch : 0;
    for (int s = 0; s < K; ++s) {
        tmps_stage* st = stages[s];
        if (!st) return fail(TMPS_EINVAL, "stage %d is null", s);
        if (st->cfg.n_micro != N || st->cfg.micro_batch != mb)
            return fail(TMPS_EMICRO, "stage %d was created for %d micro-batches of %d, the run uses %d of %d", s,
                        st->cfg.n_micro, st->cfg.micro_batch, N, mb);
        if ((st->cfg.is_last != 0) != (s == K - 1)) return fail(TMPS_ESHAPE, "only the last stage may end in the loss");
        if (s > 0 && stages[s - 1]->out_elems != st->in_elems)
            return fail(TMPS_ESHAPE, "stage %d output (%lld) does not match stage %d input (%lld)", s - 1,
                        (long long)stages[s - 1]->out_elems, s, (long long)st->in_elems);
        if (s > 0 && stages[s - 1]->cfg.dtype != st->cfg.dtype) return fail(TMPS_ESHAPE, "stages differ in dtype");
        int need = one_f1b ? K - s : stash_groups(K, N, s);
        if (st->cfg.max_stash / N < need)
            return fail(TMPS_ESTASH, "stage %d can stash %d mini-batches, the schedule needs %d", s, st->cfg.max_stash / N, need);
        for (char u : st->slot_used)
            if (u) return fail(TMPS_ESLOT, "stage %d has a stash slot in use", s);
        if (vsync && st->shadow_n < shadow_versions(K, N, s))
            return fail(TMPS_ESTASH, "stage %d keeps %d older weight versions, vertical weight stashing needs %d", s,
                        st->shadow_n, shadow_versions(K, N, s));
        if (one_f1b && st->shadow_n < K - s - 1)
            return fail(TMPS_ESTASH, "stage %d keeps %d older weight versions, horizontal weight stashing needs %d", s,
                        st->shadow_n, K - s - 1);
    }
    const std::vector<Task> tasks = one_f1b ? plan_1f1b(K, n_minibatches) : plan_nf1b(K, N, n_minibatches);

    RunCtx c;
    c.stages = stages; c.K = K; c.N = N; c.mb = mb; c.M = mb * N; c.n_minibatches = n_minibatches;
    c.inputs = inputs; c.labels = labels; c.streams = hip_streams; c.losses_out = losses_out;
    c.log = version_log_out;
    c.vsync = vsync;
    c.one_f1b = one_f1b;
    for (int s = 0; s < K; ++s) c.base_version.push_back(stages[s]->version);
    c.asz = stages[0]->asz;
    c.total_micro = (size_t)n_minibatches * N;
    c.n_fwd_ev = (size_t)(K - 1) * c.total_micro;
    c.groups.resize(K);
    for (int s = 0; s < K; ++s) c.groups[s] = stages[s]->cfg.max_stash / N;
    const size_t n_events = c.n_fwd_ev + (size_t)K * n_minibatches;
    for (int s = 0; s < K; ++s) {
        int rc = grow_events(stages[s], c.total_micro + (size_t)n_minibatches);
        if (rc != TMPS_OK) return rc;
    }
    c.recorded = std::vector<std::atomic<unsigned char>>(n_events);
    for (auto& f : c.recorded) f.store(0, std::memory_order_relaxed);

    // per-stage task lists (indices into `tasks`, which is also the order of the version log)
    std::vector<std::vector<size_t>> mine(K);
    for (size_t i = 0; i < tasks.size(); ++i) mine[tasks[i].stage].push_back(i);

    const char* env = getenv("TMPS_ISSUE_THREADS");
    const bool threaded = K > 1 && !(env && env[0] == '0');
    const bool report = getenv("TMPS_REPORT_ISSUE_TIME") != nullptr;
    const auto t0 = std::chrono::steady_clock::now();
    if (threaded) {
        int dev = 0;
        TMPS_HIP(hipGetDevice(&dev));
        std::vector<std::thread> workers;
        for (int s = 0; s < K; ++s)
            workers.emplace_back([&, s]() {
                if (hipSetDevice(dev) != hipSuccess) {
                    fail(TMPS_EHIP, "hipSetDevice failed in an issue thread");
                    c.set_error(TMPS_EHIP);
                    return;
                }
                for (size_t i : mine[s]) {
                    if (c.err.load(std::memory_order_relaxed) != TMPS_OK) return;
                    int r = issue(c, tasks[i], i);
                    if (r != TMPS_OK) {
                        if (c.err.load() == TMPS_OK) c.set_error(r);
                        return;
                    }
                }
            });
        for (std::thread& t : workers) t.join();
    } else {
        for (size_t i = 0; i < tasks.size(); ++i) {
            int r = issue(c, tasks[i], i);
            if (r != TMPS_OK) {
                c.set_error(r);
                break;
            }
        }
    }
    const auto t1 = std::chrono::steady_clock::now();
    for (int s = 0; s < K; ++s) TMPS_HIP(hipStreamSynchronize((hipStream_t)hip_streams[s]));
    if (c.err.load() != TMPS_OK) {
        // the mini-batches in flight are lost: free their stash slots, so that the stages can run again
        for (int s = 0; s < K; ++s) {
            std::fill(stages[s]->slot_used.begin(), stages[s]->slot_used.end(), 0);
            std::fill(stages[s]->slot_x.begin(), stages[s]->slot_x.end(), nullptr);
        }
        return fail(c.err.load(), "%s", c.err_text);
    }
    if (report) {
        const auto t2 = std::chrono::steady_clock::now();
        fprintf(stderr, "tmps_schedule_run: %d mini-batches, host issue %.3f ms, until idle %.3f ms\n", n_minibatches,
                std::chrono::duration<double, std::milli>(t1 - t0).count(),
                std::chrono::duration<double, std::milli>(t2 - t0).count());
    }
    return TMPS_OK;
}

extern "C" int tmps_schedule_run(tmps_stage** stages, int K, int N, int n_minibatches, const void* inputs,
                                 const int32_t* labels, void** hip_streams, float* losses_out,
                                 int32_t* version_log_out) {
    return schedule_run(stages, K, N, n_minibatches, inputs, labels, hip_streams, losses_out, version_log_out, kModeInPlace);
}

extern "C" int tmps_schedule_run_vsync(tmps_stage** stages, int K, int N, int n_minibatches, const void* inputs,
                                       const int32_t* labels, void** hip_streams, float* losses_out,
                                       int32_t* version_log_out) {
    return schedule_run(stages, K, N, n_minibatches, inputs, labels, hip_streams, losses_out, version_log_out, kModeVsync);
}

extern "C" int tmps_schedule_run_1f1b(tmps_stage** stages, int K, int n_batches, const void* inputs, const int32_t* labels,
                                      void** hip_streams, float* losses_out, int32_t* version_log_out) {
    return schedule_run(stages, K, 1, n_batches, inputs, labels, hip_streams, losses_out, version_log_out, kMode1F1B);
}

extern "C" int tmps_streams_create(void** out, int n) {
    if (!out || n < 1) return fail(TMPS_EINVAL, "tmps_streams_create needs an array and a positive count");
    for (int i = 0; i < n; ++i) out[i] = nullptr;
    for (int i = 0; i < n; ++i) {
        hipStream_t s = nullptr;
        hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
        if (e != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipStreamDestroy((hipStream_t)out[j]);
            return fail(TMPS_EHIP, "hipStreamCreateWithFlags failed: %s", hipGetErrorString(e));
        }
        out[i] = s;
    }
    return TMPS_OK;
}

extern "C" int tmps_streams_destroy(void** streams, int n) {
    if (!streams) return fail(TMPS_EINVAL, "streams is null");
    for (int i = 0; i < n; ++i)
        if (streams[i]) {
            TMPS_HIP(hipStreamDestroy((hipStream_t)streams[i]));
            streams[i] = nullptr;
        }
    return TMPS_OK;
}

// One-GPU pipeline emulator: K stages on K HIP streams, tasks issued in nF1B order, cross-stage
// dependencies as events (sections "Work Scheduling" and "Overlapping of Computation and
// Communication": what would be a message between workers is an event between streams here).
#include <vector>

#include "schedule.h"
#include "stage.h"
#include "profile.h"

using namespace tmps;

namespace {

struct EventPool {
    std::vector<hipEvent_t> ev;
    ~EventPool() {
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    }
    int grow(size_t n) {
        while (ev.size() < n) {
            hipEvent_t e;
            TMPS_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            ev.push_back(e);
        }
        return TMPS_OK;
    }
};

}  // namespace

extern "C" int tmps_schedule_run(tmps_stage** stages, int K, int N, int n_minibatches, const void* inputs,
                                 const int32_t* labels, void** hip_streams, float* losses_out,
                                 int32_t* version_log_out) {
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
        int need = stash_groups(K, N, s);
        if (st->cfg.max_stash / N < need)
            return fail(TMPS_ESTASH, "stage %d can stash %d mini-batches, the schedule needs %d", s, st->cfg.max_stash / N, need);
        for (char u : st->slot_used)
            if (u) return fail(TMPS_ESLOT, "stage %d has a stash slot in use", s);
    }
    const int M = mb * N;
    const std::vector<Task> tasks = plan_nf1b(K, N, n_minibatches);
    const size_t total_micro = (size_t)n_minibatches * N;

    // events: forward (stage, micro-batch) for s < K-1, backward (stage, mini-batch) for every stage
    EventPool pool;
    const size_t n_fwd_ev = (size_t)(K - 1) * total_micro;
    int rc = pool.grow(n_fwd_ev + (size_t)K * n_minibatches);
    if (rc != TMPS_OK) return rc;
    auto fwd_ev = [&](int s, size_t q) { return pool.ev[(size_t)s * total_micro + q]; };
    auto bwd_ev = [&](int s, int b0) { return pool.ev[n_fwd_ev + (size_t)s * n_minibatches + b0]; };

    std::vector<int> groups(K);
    for (int s = 0; s < K; ++s) groups[s] = stages[s]->cfg.max_stash / N;
    const size_t asz = stages[0]->asz;
    std::vector<int> slots(N);

    size_t ti = 0;
    for (const Task& k : tasks) {
        tmps_stage* st = stages[k.stage];
        hipStream_t s = (hipStream_t)hip_streams[k.stage];
        const int b0 = k.b - 1;
        if (version_log_out) {
            int32_t* o = version_log_out + 7 * ti;
            o[0] = k.t; o[1] = k.stage; o[2] = k.kind; o[3] = k.b; o[4] = k.j;
            o[5] = (int32_t)st->version; o[6] = k.net_version;
        }
        ++ti;
        const int group = b0 % groups[k.stage];
        if (k.kind == kFwd) {
            const size_t q = (size_t)b0 * N + k.j;
            const int slot = group * N + k.j;
            const void* x;
            if (k.stage == 0) {
                x = (const char*)inputs + ((size_t)b0 * M + (size_t)k.j * mb) * st->in_elems * asz;
            } else {
                tmps_stage* prev = stages[k.stage - 1];
                x = tmps_stage_output_ptr(prev, (b0 % groups[k.stage - 1]) * N + k.j);
                TMPS_HIP(hipStreamWaitEvent(s, fwd_ev(k.stage - 1, q), 0));
            }
            const int32_t* lab = st->cfg.is_last ? labels + (size_t)b0 * M + (size_t)k.j * mb : nullptr;
            rc = tmps_forward_micro(st, slot, x, nullptr, lab, nullptr, s);
            if (rc != TMPS_OK) return rc;
            if (k.stage < K - 1) TMPS_HIP(hipEventRecord(fwd_ev(k.stage, q), s));
            if (st->cfg.is_last && k.j == N - 1 && losses_out)
            {
                ProfileScope scope(kcReduce, s);
                TMPS_HIP(reduce_scaled_sum(stage_row_loss(st, group * N), M, 1.0f / (float)M, losses_out + b0, s));
            }
        } else {
            const void* dy = nullptr;
            if (k.stage < K - 1) {
                dy = stage_dxout(stages[k.stage + 1], b0 & 1);
                TMPS_HIP(hipStreamWaitEvent(s, bwd_ev(k.stage + 1, b0), 0));
            }
            void* dx = nullptr;
            if (k.stage > 0) {
                dx = stage_dxout(st, b0 & 1);
                // the worker below must have consumed what this buffer held two mini-batches ago
                if (b0 >= 2) TMPS_HIP(hipStreamWaitEvent(s, bwd_ev(k.stage - 1, b0 - 2), 0));
            }
            for (int j = 0; j < N; ++j) slots[j] = group * N + j;
            rc = tmps_backward(st, slots.data(), N, dy, dx, s);
            if (rc != TMPS_OK) return rc;
            TMPS_HIP(hipEventRecord(bwd_ev(k.stage, b0), s));
            rc = tmps_update(st, s);
            if (rc != TMPS_OK) return rc;
        }
    }
    for (int s = 0; s < K; ++s) TMPS_HIP(hipStreamSynchronize((hipStream_t)hip_streams[s]));
    return TMPS_OK;
}

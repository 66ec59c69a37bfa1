// nF1B schedule of TiMePReSt by time-point simulation (section "Work Scheduling") and the version
// bookkeeping of section "Multiple Sequence Problem".  Host only.
//
// State per worker: the time-point at which each micro-batch / each backward pass becomes available
// to it.  A worker does one task per time-point; what it finishes at t is available to its
// neighbour at t+1; a backward pass that is available is taken before any forward; worker 0 always
// has the next micro-batch available; the backward pass of a mini-batch becomes available on the last
// worker right after that worker forwarded the mini-batch's last micro-batch; a worker's update
// follows its backward pass within the same time-point.
#include "schedule.h"

#include <algorithm>

#include "common.h"

namespace tmps {

std::vector<Task> plan_nf1b(int W, int N, int n_minibatches) {
    const int total_micro = n_minibatches * N;
    // fwd_ready[s][q]: time-point from which micro-batch number q (0-based, over the whole run) can be
    // forwarded by worker s; bwd_ready[s][b]: same for the backward pass of mini-batch b (0-based).
    const int32_t never = INT32_MAX;
    std::vector<std::vector<int32_t>> fwd_ready(W, std::vector<int32_t>(total_micro, never));
    std::vector<std::vector<int32_t>> bwd_ready(W, std::vector<int32_t>(n_minibatches, never));
    std::fill(fwd_ready[0].begin(), fwd_ready[0].end(), 1);
    std::vector<int> next_fwd(W, 0), next_bwd(W, 0), updates(W, 0);
    std::vector<int32_t> left_worker0_at;         // time-points at which backward passes left worker 0
    std::vector<int32_t> inject_version(total_micro, 0), bwd_version(n_minibatches, 0);
    std::vector<Task> tasks;
    tasks.reserve((size_t)W * (total_micro + n_minibatches));

    int done = 0;
    for (int32_t t = 1; done < n_minibatches; ++t) {
        int32_t net_version = 0;
        for (int32_t tt : left_worker0_at) net_version += (tt < t);
        for (int s = 0; s < W; ++s) {
            int b = next_bwd[s];
            if (b < n_minibatches && bwd_ready[s][b] <= t) {
                if (s == W - 1) bwd_version[b] = net_version;
                tasks.push_back(Task{t, s, kBwd, b + 1, -1, updates[s], bwd_version[b]});
                ++updates[s];
                ++next_bwd[s];
                if (s > 0) bwd_ready[s - 1][b] = t + 1;
                else {
                    left_worker0_at.push_back(t);
                    ++done;
                }
                continue;
            }
            int q = next_fwd[s];
            if (q < total_micro && fwd_ready[s][q] <= t) {
                if (s == 0) inject_version[q] = net_version;
                tasks.push_back(Task{t, s, kFwd, q / N + 1, q % N, updates[s], inject_version[q]});
                ++next_fwd[s];
                if (s < W - 1) fwd_ready[s + 1][q] = t + 1;
                else if (q % N == N - 1) bwd_ready[s][q / N] = t + 1;
            }
        }
    }
    return tasks;
}

// 1F1B by the same time-point rules (one task per worker and time-point, results reach the neighbour at t+1, a
// backward pass that has arrived goes first), plus the start-up depth of the related-work system: worker s takes a
// forward pass only while fewer than W - s batches are between their forward and backward pass on it.
std::vector<Task> plan_1f1b(int W, int n_batches) {
    const int32_t never = INT32_MAX;
    std::vector<std::vector<int32_t>> fwd_ready(W, std::vector<int32_t>(n_batches, never));
    std::vector<std::vector<int32_t>> bwd_ready(W, std::vector<int32_t>(n_batches, never));
    std::vector<std::vector<int32_t>> read_by_fwd(W, std::vector<int32_t>(n_batches, 0));
    std::fill(fwd_ready[0].begin(), fwd_ready[0].end(), 1);
    std::vector<int> next_fwd(W, 0), next_bwd(W, 0), updates(W, 0);
    std::vector<Task> tasks;
    tasks.reserve((size_t)W * 2 * n_batches);
    int done = 0;
    for (int32_t t = 1; done < n_batches; ++t) {
        for (int s = 0; s < W; ++s) {
            const int b = next_bwd[s];
            if (b < n_batches && bwd_ready[s][b] <= t) {
                tasks.push_back(Task{t, s, kBwd, b + 1, -1, read_by_fwd[s][b], updates[s]});
                ++updates[s];
                ++next_bwd[s];
                if (s > 0) bwd_ready[s - 1][b] = t + 1;
                else ++done;
                continue;
            }
            const int q = next_fwd[s];
            if (q < n_batches && fwd_ready[s][q] <= t && next_fwd[s] - next_bwd[s] < W - s) {
                read_by_fwd[s][q] = updates[s];
                tasks.push_back(Task{t, s, kFwd, q + 1, -1, updates[s], updates[s]});
                ++next_fwd[s];
                if (s < W - 1) fwd_ready[s + 1][q] = t + 1;
                else bwd_ready[s][q] = t + 1;
            }
        }
    }
    return tasks;
}

int stash_groups(int W, int N, int stage) {
    const int n = 3 * W + 4;
    std::vector<Task> tasks = plan_nf1b(W, N, n);
    std::vector<char> live(n + 1, 0);
    int cur = 0, need = 0;
    for (const Task& k : tasks) {
        if (k.stage != stage) continue;
        if (k.kind == kFwd) {
            if (!live[k.b]) { live[k.b] = 1; ++cur; need = std::max(need, cur); }
        } else if (live[k.b]) {
            live[k.b] = 0;
            --cur;
        }
    }
    return need;
}

int shadow_versions(int W, int N, int stage) {
    const int n = 4 * W + 4 * N + 8;
    int need = 0;
    for (const Task& k : plan_nf1b(W, N, n))
        if (k.kind == kFwd && k.stage == stage) need = std::max(need, (int)(k.stage_version - k.net_version));
    return need;
}

int version_diff_simulated(int W, int N) {
    const int n = 4 * W + 4 * N + 8;
    std::vector<Task> tasks = plan_nf1b(W, N, n);
    for (const Task& k : tasks)
        if (k.kind == kBwd && k.stage == W - 1 && k.b == n) return n - k.net_version;
    return -1;
}

}  // namespace tmps

using namespace tmps;

extern "C" int tmps_schedule_plan(int W, int N, int n_minibatches, int32_t* ops_out, size_t cap_ops) {
    if (W < 1 || N < 1 || n_minibatches < 1) return fail(TMPS_EINVAL, "W, N and n_minibatches must be positive");
    std::vector<Task> tasks = plan_nf1b(W, N, n_minibatches);
    if (ops_out) {
        if (cap_ops < tasks.size())
            return fail(TMPS_ECAP, "ops_out holds %zu tasks, %zu needed", cap_ops, tasks.size());
        for (size_t i = 0; i < tasks.size(); ++i) {
            const Task& k = tasks[i];
            int32_t* o = ops_out + 7 * i;
            o[0] = k.t; o[1] = k.stage; o[2] = k.kind; o[3] = k.b; o[4] = k.j;
            o[5] = k.stage_version; o[6] = k.net_version;
        }
    }
    return (int)tasks.size();
}

extern "C" int tmps_schedule_plan_1f1b(int W, int n_batches, int32_t* ops_out, size_t cap_ops) {
    if (W < 1 || n_batches < 1) return fail(TMPS_EINVAL, "W and n_batches must be positive");
    std::vector<Task> tasks = plan_1f1b(W, n_batches);
    if (ops_out) {
        if (cap_ops < tasks.size())
            return fail(TMPS_ECAP, "ops_out holds %zu tasks, %zu needed", cap_ops, tasks.size());
        for (size_t i = 0; i < tasks.size(); ++i) {
            const Task& k = tasks[i];
            int32_t* o = ops_out + 7 * i;
            o[0] = k.t; o[1] = k.stage; o[2] = k.kind; o[3] = k.b; o[4] = k.j;
            o[5] = k.stage_version; o[6] = k.net_version;
        }
    }
    return (int)tasks.size();
}

extern "C" int tmps_schedule_shadow_versions(int W, int N, int stage) {
    if (W < 1 || N < 1 || stage < 0 || stage >= W) return fail(TMPS_EINVAL, "W, N must be positive and 0 <= stage < W");
    return shadow_versions(W, N, stage);
}

extern "C" int tmps_schedule_stash_groups(int W, int N, int stage) {
    if (W < 1 || N < 1 || stage < 0 || stage >= W) return fail(TMPS_EINVAL, "bad W, N or stage");
    return stash_groups(W, N, stage);
}

extern "C" int tmps_version_diff_formula(int W, int N) {
    if (W < 2 || N < 2) return fail(TMPS_EINVAL, "the version difference is defined for W >= 2 and N >= 2");
    return (W + N - 2) / N;
}

extern "C" int tmps_version_diff_simulated(int W, int N) {
    if (W < 1 || N < 1) return fail(TMPS_EINVAL, "W and N must be positive");
    return version_diff_simulated(W, N);
}

// nF1B task list by time-point simulation (host only, integers only).
#pragma once
#include <stdint.h>

#include <vector>

namespace tmps {

struct Task {
    int32_t t, stage, kind, b, j, stage_version, net_version;
};
constexpr int kFwd = 0, kBwd = 1;

// Tasks of W workers, N micro-batches per mini-batch, in (time-point, worker) order.
std::vector<Task> plan_nf1b(int W, int N, int n_minibatches);
// Largest number of mini-batches simultaneously between first forward and backward on `stage`.
int stash_groups(int W, int N, int stage);
int version_diff_simulated(int W, int N);
// Older weight versions `stage` must keep so that every forward pass finds the version it is tagged with.
int shadow_versions(int W, int N, int stage);

}  // namespace tmps

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

// The comparison system (PipeDream-style 1F1B with horizontal weight stashing): every batch makes its own forward and
// backward pass; worker s makes a forward pass only while fewer than W - s batches are in flight on it.  Tasks in
// (time-point, worker) order; j = -1; stage_version = the updates in the weights the task READS (a backward pass:
// those of its forward pass), net_version = the updates the worker had applied before the task.
std::vector<Task> plan_1f1b(int W, int n_batches);

}  // namespace tmps

// One pipeline worker: consecutive layers, activation stash, backward pass, in-place update.
#pragma once
#include <array>
#include <map>
#include <mutex>
#include <shared_mutex>
#include <vector>

#include "common.h"
#include "kernels.h"

struct LayerRT {
    tmps_layer_desc d;
    int64_t in_elems = 0, out_elems = 0;  // per sample
    int64_t w_off = 0, w_count = 0, b_off = 0, b_count = 0;  // positions in the flat parameter arrays
    size_t out_off = 0;    // stash byte offset of this layer's output array (all slots)
    size_t out_esize = 0;  // bytes per element of that array
    size_t aux_off = 0;    // softmax-CE: stash byte offset of the per-row losses (fp32)
    size_t z_off = 0;      // GELU linear: stash byte offset of the stored derivatives gelu'(pre-activation)
    bool relu = false;
    int act = 0;           // 0 none, 1 ReLU, 2 GELU (linear / convolution epilogue)
    int rps = 1;           // rows per sample the layer works on (sequence positions)
    int skip = 0;          // linear: > 0 adds the input of layer (index - skip)
    int in_t = -1;         // which result the layer reads: index of the producing layer, -1 = the stage input
    int in_b = -1;         // residual join: the second result it reads
    bool out_f32 = false;  // the logits layer (followed by softmax-CE) writes fp32
    size_t ws_elems = 0;   // fp32 workspace elements (split-k partial sums, reductions)
    size_t ws_fwd_elems = 0;  // the part of it the forward pass needs
};

struct tmps_stage {
    tmps_stage_cfg cfg;
    std::vector<LayerRT> layers;
    int64_t P = 0;  // flat parameter count (with alignment gaps)
    int64_t in_elems = 0, out_elems = 0;
    size_t asz = 4;  // bytes per activation / gradient element
    size_t in_esize = 4;  // bytes per element of the stage input (int32 tokens in front of an embedding)
    int label_rps = 1;    // labels per sample on the last stage
    int n_gbuf = 2;       // gradient buffers in scratch
    std::vector<int> readers;  // readers[t + 1] = number of layers that read result t (t = -1: the stage input)
    char* params = nullptr;
    char* state = nullptr;
    char* stash = nullptr;
    char* scratch = nullptr;
    float* master = nullptr;
    void* wcopy = nullptr;  // bf16 working copy (null for fp32 stages)
    float* mom = nullptr;
    float* grad = nullptr;
    size_t in_off = 0;  // stash offset of the copied inputs (borrow_input == 0)
    size_t stash_bytes = 0, scratch_bytes = 0;
    size_t gbuf_off[8] = {0, 0, 0, 0, 0, 0, 0, 0}, gbuf_bytes = 0;  // gradient buffers (M rows each)
    size_t dxout_off[2] = {0, 0}, dxout_bytes = 0;  // boundary gradient buffers used by the scheduler
    size_t ws_off = 0;
    size_t ws_fwd_bytes = 0;  // fp32 workspace bytes a forward pass needs (the k-split partial sums of its contractions)
    std::vector<char> slot_used;
    std::vector<const void*> slot_x;
    long version = 0;
    std::vector<hipEvent_t> events;   // tmps_schedule_run: what this worker sends to its neighbours (kept between runs)
    // Graph replay (tmps_stage_use_graphs): the kernels of a forward or backward pass, captured once per distinct
    // set of device addresses they work on and launched as one graph from then on.  A key is the kind of pass and
    // every address that varies between calls; the stage's own regions never move.
    typedef std::array<uintptr_t, 8> GraphKey;
    bool use_graphs = false;
    std::map<GraphKey, hipGraphExec_t> graphs;
    std::map<GraphKey, int> graph_seen;   // calls with a key that has no graph yet (captured at the second)
    size_t lab_off = 0;                   // last stage: stash offset of the copied labels (read by captured loss kernels)
    ~tmps_stage() {
        for (hipEvent_t e : events) (void)hipEventDestroy(e);
        for (auto& g : graphs) (void)hipGraphExecDestroy(g.second);
    }
    // vertical weight stashing: copies of the `params` region as it was after earlier updates
    char* shadow = nullptr;
    int shadow_n = 0;                 // copies the caller's region holds
    size_t param_bytes = 0;           // size of `params` (one copy)
    std::vector<long> shadow_ver;     // version each copy holds (-1: none)

    int M() const { return cfg.micro_batch * cfg.n_micro; }
    // weights the contractions read
    const void* wptr(const LayerRT& L) const {
        return wcopy ? (const void*)((const char*)wcopy + L.w_off * 2) : (const void*)(master + L.w_off);
    }
    const float* bptr(const LayerRT& L) const { return master + L.b_off; }
    // second parameter array in the contraction dtype (position table of an embedding)
    const void* bptr_c(const LayerRT& L) const {
        return wcopy ? (const void*)((const char*)wcopy + L.b_off * 2) : (const void*)(master + L.b_off);
    }
    char* out_ptr(const LayerRT& L, int64_t row) const {
        return stash + L.out_off + (size_t)row * L.out_elems * L.out_esize;
    }
    // elements per sample of result t (-1: the stage input)
    int64_t tensor_elems(int t) const { return t < 0 ? in_elems : layers[t].out_elems; }
};

namespace tmps {
// While a stream is being captured the runtime refuses, in every thread, to make another stream wait for an event that
// was recorded on the capturing stream, also one recorded before the capture began.  A pass that captures holds this
// lock exclusively from the beginning to the end of the capture; the scheduler's threads hold it shared around their
// cross-stream waits.  (Captures are rare: one per distinct set of addresses of a pass.)
std::shared_mutex& capture_lock();
// Fills `st` from the descriptors: shapes, flat parameter layout, stash and scratch layout.
int stage_layout(tmps_stage& st, const tmps_layer_desc* layers, int n_layers, const tmps_stage_cfg* cfg);
// Device address of the boundary-gradient buffer `which` (0/1) of a stage.
void* stage_dxout(tmps_stage* st, int which);
// Per-row losses of a slot on the last stage.
float* stage_row_loss(tmps_stage* st, int slot);
// tmps_forward_micro with the fp32 workspace of its contractions (st->ws_fwd_bytes) given by the caller.
int forward_with_workspace(tmps_stage* st, int slot, const void* x, void* y, const int32_t* labels, float* loss_out,
                           void* hip_stream, float* ws);
}  // namespace tmps

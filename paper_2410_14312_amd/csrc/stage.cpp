// Stage executor: turns a layer list into kernel launches on the caller's stream.
//
// forward_micro : the layers on one micro-batch with the current weights; every layer output goes
//                 into the stash slot (it is the next layer's input, the ReLU mask source and, for
//                 the last layer, what the next worker reads).
// backward      : one pass over the N micro-batches of a mini-batch group, whose stashed rows are
//                 consecutive, so every layer's gradient GEMMs run once over M rows: the sum of the
//                 weight gradient over the micro-batches is the k-loop of that GEMM.  Weights are read
//                 as they are now; activations, ReLU masks, pooling winners and the softmax error
//                 signal are the forward pass's (sections "Challenge 1" and "Challenge 2", Solution).
// update        : fused momentum step over the stage's flat parameter array.
#include "stage.h"

#include "profile.h"

#include <string.h>

#include <algorithm>
#include <initializer_list>

#include <new>
#include <vector>

namespace tmps {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// launch with optional event timing of its kernel class
#define TMPS_RUN(kc, stream, expr)                 \
    do {                                           \
        ::tmps::ProfileScope scope_((kc), (stream)); \
        TMPS_HIP(expr);                            \
    } while (0)

// the contraction launchers time their kernels themselves (per kernel, by dispatch timestamps)
#define TMPS_GEMM(expr) TMPS_HIP(expr)

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static ConvShape conv_shape(const tmps_layer_desc& d, int B) {
    ConvShape c;
    c.B = B; c.H = d.dims[0]; c.W = d.dims[1]; c.Cin = d.dims[2]; c.Cout = d.dims[3];
    c.R = d.dims[4]; c.S = d.dims[5]; c.stride = d.dims[6]; c.pad = d.dims[7];
    c.Ho = (c.H + 2 * c.pad - c.R) / c.stride + 1;
    c.Wo = (c.W + 2 * c.pad - c.S) / c.stride + 1;
    return c;
}

int stage_layout(tmps_stage& st, const tmps_layer_desc* layers, int n_layers, const tmps_stage_cfg* cfg) {
    if (!layers || !cfg || n_layers < 1) return fail(TMPS_EINVAL, "null layers/cfg or no layers");
    if (cfg->dtype != TMPS_F32 && cfg->dtype != TMPS_BF16_F32MASTER) return fail(TMPS_EINVAL, "unknown dtype %d", cfg->dtype);
    if (cfg->micro_batch < 1 || cfg->n_micro < 1) return fail(TMPS_EINVAL, "micro_batch and n_micro must be positive");
    if (cfg->n_micro > 64) return fail(TMPS_EUNSUPPORTED, "at most 64 micro-batches per mini-batch");
    if (cfg->max_stash < cfg->n_micro || cfg->max_stash % cfg->n_micro != 0)
        return fail(TMPS_EMICRO, "max_stash (%d) must be a positive multiple of n_micro (%d): a mini-batch is N equal micro-batches",
                    cfg->max_stash, cfg->n_micro);
    st.cfg = *cfg;
    st.asz = act_bytes(cfg->dtype);
    st.in_esize = st.asz;
    st.layers.clear();
    const int mb = cfg->micro_batch;
    const int M = mb * cfg->n_micro;
    const int64_t rows_all = (int64_t)cfg->max_stash * mb;
    int64_t cur = -1, poff = 0, gmax = 0;
    size_t soff = 0, ws = 0;
    bool any_skip = false;
    for (int i = 0; i < n_layers; ++i) {
        LayerRT L;
        L.d = layers[i];
        const int32_t* d = L.d.dims;
        L.relu = (L.d.flags & TMPS_FLAG_RELU) != 0;
        L.act = L.relu ? 1 : ((L.d.flags & TMPS_FLAG_GELU) ? 2 : 0);
        switch (L.d.kind) {
            case TMPS_LINEAR: {
                if (d[0] < 1 || d[1] < 1) return fail(TMPS_EINVAL, "layer %d: linear dims must be positive", i);
                if ((L.d.flags & TMPS_FLAG_RELU) && (L.d.flags & TMPS_FLAG_GELU))
                    return fail(TMPS_EINVAL, "layer %d: ReLU and GELU are exclusive", i);
                if (d[2] < 0 || d[3] < 0) return fail(TMPS_EINVAL, "layer %d: negative skip or row count", i);
                L.rps = d[3] > 0 ? d[3] : 1;
                L.skip = d[2];
                L.in_elems = (int64_t)L.rps * d[0]; L.out_elems = (int64_t)L.rps * d[1];
                L.w_count = (int64_t)d[0] * d[1]; L.b_count = d[1];
                if (L.skip) {
                    const int src = i - L.skip;
                    if (src < 0) return fail(TMPS_ESHAPE, "layer %d: residual source lies before the stage", i);
                    if (st.layers[src].d.kind != TMPS_LAYERNORM)
                        return fail(TMPS_EUNSUPPORTED, "layer %d: a residual connection must start at the input of a layer-normalisation layer", i);
                    if (st.layers[src].in_elems != L.out_elems)
                        return fail(TMPS_ESHAPE, "layer %d: residual source has %lld elements per sample, the layer output %lld", i,
                                    (long long)st.layers[src].in_elems, (long long)L.out_elems);
                    for (int j = src + 1; j < i; ++j)
                        if (st.layers[j].skip && j - st.layers[j].skip == src)
                            return fail(TMPS_EUNSUPPORTED, "layer %d: two residual connections start at the same layer", i);
                    any_skip = true;
                }
                const int64_t rf = (int64_t)mb * L.rps, rb = (int64_t)M * L.rps;
                L.ws_elems = std::max({gemm_workspace_elems(rf, d[1], d[0], 0), gemm_workspace_elems(rb, d[0], d[1], 0),
                                       gemm_workspace_elems(d[1], d[0], rb, 1)});
                break;
            }
            case TMPS_CONV2D: {
                for (int k = 0; k < 7; ++k)
                    if (d[k] < 1) return fail(TMPS_EINVAL, "layer %d: conv dims must be positive", i);
                if (d[7] < 0) return fail(TMPS_EINVAL, "layer %d: negative padding", i);
                if (L.act == 2) return fail(TMPS_EUNSUPPORTED, "layer %d: GELU on a convolution is not built", i);
                ConvShape c = conv_shape(L.d, M);
                if (c.Ho < 1 || c.Wo < 1) return fail(TMPS_ESHAPE, "layer %d: empty convolution output", i);
                L.in_elems = (int64_t)c.H * c.W * c.Cin;
                L.out_elems = (int64_t)c.Ho * c.Wo * c.Cout;
                L.w_count = (int64_t)c.Cout * c.R * c.S * c.Cin; L.b_count = c.Cout;
                const int64_t kf = (int64_t)c.R * c.S * c.Cin, kd = (int64_t)c.R * c.S * c.Cout;
                L.ws_elems = std::max({gemm_workspace_elems((int64_t)mb * c.Ho * c.Wo, c.Cout, kf, 0),
                                       gemm_workspace_elems((int64_t)M * c.H * c.W, c.Cin, kd, 0),
                                       gemm_workspace_elems(c.Cout, kf, (int64_t)M * c.Ho * c.Wo, 1)});
                break;
            }
            case TMPS_MAXPOOL: {
                if (d[0] < 1 || d[1] < 1 || d[2] < 1 || d[3] < 1 || d[4] < 1 || d[3] > d[0] || d[3] > d[1])
                    return fail(TMPS_EINVAL, "layer %d: bad pooling dims", i);
                int Ho = (d[0] - d[3]) / d[4] + 1, Wo = (d[1] - d[3]) / d[4] + 1;
                L.in_elems = (int64_t)d[0] * d[1] * d[2];
                L.out_elems = (int64_t)Ho * Wo * d[2];
                L.relu = false; L.act = 0;
                break;
            }
            case TMPS_LAYERNORM:
                if (d[0] < 1 || d[1] < 0) return fail(TMPS_EINVAL, "layer %d: bad layer-normalisation dims", i);
                L.rps = d[1] > 0 ? d[1] : 1;
                L.in_elems = L.out_elems = (int64_t)L.rps * d[0];
                L.w_count = d[0]; L.b_count = d[0];
                L.relu = false; L.act = 0;
                L.ws_elems = layernorm_workspace_elems((int64_t)M * L.rps, d[0]);
                break;
            case TMPS_ATTENTION:
                if (d[0] < 1 || d[1] < 1 || d[2] < 1 || d[1] % d[2] != 0)
                    return fail(TMPS_EINVAL, "layer %d: attention needs S, D, heads positive and D a multiple of heads", i);
                L.rps = d[0];
                L.in_elems = (int64_t)d[0] * 3 * d[1];
                L.out_elems = (int64_t)d[0] * d[1];
                L.relu = false; L.act = 0;
                L.ws_elems = attention_workspace_elems(M, d[0], d[2]);
                break;
            case TMPS_EMBEDDING:
                if (i != 0) return fail(TMPS_ESHAPE, "an embedding can only be the first layer of a stage");
                if (d[0] < 1 || d[1] < 1 || d[2] < 1) return fail(TMPS_EINVAL, "layer %d: embedding dims must be positive", i);
                L.rps = d[1];
                L.in_elems = d[1];
                L.out_elems = (int64_t)d[1] * d[2];
                L.w_count = (int64_t)d[0] * d[2]; L.b_count = (int64_t)d[1] * d[2];
                L.relu = false; L.act = 0;
                st.in_esize = 4;
                break;
            case TMPS_SOFTMAX_CE:
                if (i != n_layers - 1 || !cfg->is_last || i == 0)
                    return fail(TMPS_ESHAPE, "softmax-CE must be the last layer of the last stage, after another layer");
                if (d[0] < 1 || d[1] < 0) return fail(TMPS_EINVAL, "layer %d: classes must be positive", i);
                if (st.layers.back().d.kind != TMPS_LINEAR || st.layers.back().act != 0 || st.layers.back().skip)
                    return fail(TMPS_EUNSUPPORTED, "softmax-CE must follow a plain linear layer");
                L.rps = d[1] > 0 ? d[1] : 1;
                if (st.layers.back().rps != L.rps)
                    return fail(TMPS_ESHAPE, "softmax-CE has %d rows per sample, the layer before it %d", L.rps, st.layers.back().rps);
                L.in_elems = L.out_elems = (int64_t)L.rps * d[0];
                L.relu = false; L.act = 0;
                st.label_rps = L.rps;
                break;
            default:
                return fail(TMPS_EUNSUPPORTED, "layer %d: kind %d not built", i, L.d.kind);
        }
        if (cur >= 0 && cur != L.in_elems)
            return fail(TMPS_ESHAPE, "layer %d expects %lld input elements per sample, previous layer gives %lld", i,
                        (long long)L.in_elems, (long long)cur);
        cur = L.out_elems;
        if (L.w_count) {
            L.w_off = poff;
            L.b_off = poff + L.w_count;
            poff = (int64_t)align_up((size_t)(L.b_off + L.b_count), 64);
        }
        // the gradient w.r.t. this layer's input lives in a gradient buffer (the loss layer's is kept in the stash)
        if (i > 0 && L.d.kind != TMPS_SOFTMAX_CE) gmax = std::max(gmax, L.in_elems);
        ws = std::max(ws, L.ws_elems);
        st.layers.push_back(L);
    }
    if (cfg->is_last && st.layers.back().d.kind != TMPS_SOFTMAX_CE)
        return fail(TMPS_ESHAPE, "the last stage must end in softmax-CE");
    if (cfg->is_last) st.layers[n_layers - 2].out_f32 = true;
    if (!cfg->is_last) {
        if (st.layers.back().act == 2) return fail(TMPS_EUNSUPPORTED, "a stage cannot end in a GELU layer");
        if (st.layers.back().relu) gmax = std::max(gmax, st.layers.back().out_elems);
    }
    st.P = poff;
    st.in_elems = st.layers.front().in_elems;
    st.out_elems = cfg->is_last ? st.layers[n_layers - 2].out_elems : st.layers.back().out_elems;

    // stash: [copied inputs] then every layer's output array over all slots, and what else the backward pass needs
    st.in_off = 0;
    if (!cfg->borrow_input) soff = align_up((size_t)rows_all * st.in_elems * st.in_esize, 256);
    for (LayerRT& L : st.layers) {
        L.out_off = soff;
        L.out_esize = L.out_f32 ? 4 : st.asz;
        soff = align_up(soff + (size_t)rows_all * L.out_elems * L.out_esize, 256);
        size_t aux = 0;
        if (L.d.kind == TMPS_SOFTMAX_CE) aux = (size_t)rows_all * L.rps * 4;                  // per-row losses
        if (L.d.kind == TMPS_LAYERNORM) aux = (size_t)rows_all * L.rps * 8;                   // (mean, 1/std) per row
        if (L.d.kind == TMPS_ATTENTION) aux = (size_t)rows_all * L.d.dims[2] * L.d.dims[0] * 4;  // log-sum-exp per head and query
        if (aux) {
            L.aux_off = soff;
            soff = align_up(soff + aux, 256);
        }
        if (L.act == 2) {
            L.z_off = soff;
            soff = align_up(soff + (size_t)rows_all * L.out_elems * st.asz, 256);
        }
    }
    st.stash_bytes = soff;

    // scratch: gradient buffers of M rows, two boundary-gradient buffers, fp32 workspace
    size_t o = 0;
    st.n_gbuf = any_skip ? 4 : 2;
    st.gbuf_bytes = align_up((size_t)M * std::max<int64_t>(gmax, 1) * st.asz, 256);
    for (int k = 0; k < st.n_gbuf; ++k) { st.gbuf_off[k] = o; o += st.gbuf_bytes; }
    st.dxout_bytes = align_up((size_t)M * st.in_elems * st.asz, 256);
    st.dxout_off[0] = o; o += st.dxout_bytes;
    st.dxout_off[1] = o; o += st.dxout_bytes;
    st.ws_off = o; o += align_up(ws * 4, 256);
    st.scratch_bytes = o;
    return TMPS_OK;
}

void* stage_dxout(tmps_stage* st, int which) { return st->scratch + st->dxout_off[which & 1]; }

float* stage_row_loss(tmps_stage* st, int slot) {
    const LayerRT& L = st->layers.back();
    return reinterpret_cast<float*>(st->stash + L.aux_off) + (size_t)slot * st->cfg.micro_batch * L.rps;
}

}  // namespace tmps

using namespace tmps;

extern "C" const char* tmps_last_error(void) { return g_err; }

extern "C" int tmps_stage_bytes(const tmps_layer_desc* layers, int n_layers, const tmps_stage_cfg* cfg,
                                size_t* param_bytes, size_t* state_bytes, size_t* stash_bytes,
                                size_t* scratch_bytes) {
    tmps_stage tmp;
    int rc = stage_layout(tmp, layers, n_layers, cfg);
    if (rc != TMPS_OK) return rc;
    if (param_bytes) *param_bytes = align_up((size_t)tmp.P * (cfg->dtype == TMPS_BF16_F32MASTER ? 6 : 4), 256);
    if (state_bytes) *state_bytes = align_up((size_t)tmp.P * 8, 256);
    if (stash_bytes) *stash_bytes = tmp.stash_bytes;
    if (scratch_bytes) *scratch_bytes = tmp.scratch_bytes;
    return TMPS_OK;
}

extern "C" int tmps_stage_create(tmps_stage** out, const tmps_layer_desc* layers, int n_layers,
                                 const tmps_stage_cfg* cfg, void* params, void* state, void* stash,
                                 void* scratch) {
    if (!out) return fail(TMPS_EINVAL, "out is null");
    *out = nullptr;
    if (!params || !state || !stash || !scratch) return fail(TMPS_EINVAL, "a device region is null");
    for (const void* p : {params, state, stash, scratch})
        if (reinterpret_cast<uintptr_t>(p) & 255) return fail(TMPS_EINVAL, "device regions must be 256-byte aligned");
    tmps_stage* st = new (std::nothrow) tmps_stage();
    if (!st) return fail(TMPS_EINVAL, "out of host memory");
    int rc = stage_layout(*st, layers, n_layers, cfg);
    if (rc != TMPS_OK) {
        delete st;
        return rc;
    }
    st->params = (char*)params; st->state = (char*)state; st->stash = (char*)stash; st->scratch = (char*)scratch;
    st->master = (float*)params;
    st->wcopy = cfg->dtype == TMPS_BF16_F32MASTER ? (void*)(st->params + (size_t)st->P * 4) : nullptr;
    st->mom = (float*)state;
    st->grad = st->mom + st->P;
    st->slot_used.assign(cfg->max_stash, 0);
    st->slot_x.assign(cfg->max_stash, nullptr);
    *out = st;
    return TMPS_OK;
}

extern "C" void tmps_stage_destroy(tmps_stage* stage) { delete stage; }

extern "C" int64_t tmps_stage_param_count(const tmps_stage* stage) { return stage ? stage->P : 0; }

extern "C" int tmps_stage_param_offset(const tmps_stage* stage, int layer, int which, int64_t* offset,
                                       int64_t* count) {
    if (!stage || layer < 0 || layer >= (int)stage->layers.size() || (which != 0 && which != 1))
        return fail(TMPS_EINVAL, "bad stage, layer or selector");
    const LayerRT& L = stage->layers[layer];
    if (offset) *offset = which ? L.b_off : L.w_off;
    if (count) *count = which ? L.b_count : L.w_count;
    return TMPS_OK;
}

extern "C" int64_t tmps_stage_input_elems(const tmps_stage* stage) { return stage ? stage->in_elems : 0; }
extern "C" int64_t tmps_stage_output_elems(const tmps_stage* stage) { return stage ? stage->out_elems : 0; }
extern "C" long tmps_stage_version(const tmps_stage* stage) { return stage ? stage->version : -1; }

extern "C" int tmps_stage_sync_params(tmps_stage* stage, void* hip_stream) {
    if (!stage) return fail(TMPS_EINVAL, "stage is null");
    if (stage->wcopy) TMPS_HIP(cast_f32_to_bf16(stage->master, stage->wcopy, stage->P, (hipStream_t)hip_stream));
    return TMPS_OK;
}

extern "C" void* tmps_stage_output_ptr(const tmps_stage* stage, int slot) {
    if (!stage || slot < 0 || slot >= stage->cfg.max_stash) return nullptr;
    const LayerRT& L = stage->cfg.is_last ? stage->layers[stage->layers.size() - 2] : stage->layers.back();
    return stage->out_ptr(L, (int64_t)slot * stage->cfg.micro_batch);
}

// what layer li reads: the stage input (x0, rows from row0 on) or the stashed output of the layer before it
static const void* layer_input(const tmps_stage* st, int li, const void* x0, int64_t row0) {
    return li == 0 ? x0 : (const void*)st->out_ptr(st->layers[li - 1], row0);
}

extern "C" int tmps_forward_micro(tmps_stage* st, int slot, const void* x, void* y, const int32_t* labels,
                                  float* loss_out, void* hip_stream) {
    if (!st || !x) return fail(TMPS_EINVAL, "stage or x is null");
    if (slot < 0 || slot >= st->cfg.max_stash) return fail(TMPS_ESLOT, "slot %d outside 0..%d", slot, st->cfg.max_stash - 1);
    if (st->slot_used[slot]) return fail(TMPS_ESLOT, "slot %d is in use", slot);
    if (st->cfg.is_last && !labels) return fail(TMPS_EINVAL, "the last stage needs labels");
    hipStream_t s = (hipStream_t)hip_stream;
    const int mb = st->cfg.micro_batch;
    const int dt = st->cfg.dtype;
    const int64_t row0 = (int64_t)slot * mb;
    const void* x0 = x;
    float* ws = reinterpret_cast<float*>(st->scratch + st->ws_off);
    if (!st->cfg.borrow_input) {
        char* dst = st->stash + st->in_off + (size_t)row0 * st->in_elems * st->in_esize;
        TMPS_RUN(kcCopy, s, hipMemcpyAsync(dst, x, (size_t)mb * st->in_elems * st->in_esize, hipMemcpyDeviceToDevice, s));
        x0 = dst;
    }
    st->slot_x[slot] = x;
    const void* in = x0;
    for (size_t li = 0; li < st->layers.size(); ++li) {
        const LayerRT& L = st->layers[li];
        void* out = st->out_ptr(L, row0);
        const int32_t* d = L.d.dims;
        switch (L.d.kind) {
            case TMPS_LINEAR: {
                const void* res = nullptr;
                if (L.skip) {
                    const int src = (int)li - L.skip;
                    res = src == 0 ? x0 : (const void*)st->out_ptr(st->layers[src - 1], row0);
                }
                void* zout = L.act == 2 ? (void*)(st->stash + L.z_off + (size_t)row0 * L.out_elems * st->asz) : nullptr;
                TMPS_GEMM(dense_forward(dt, in, st->wptr(L), st->bptr(L), out, mb * L.rps, d[0], d[1], L.act, L.out_f32, res,
                                        zout, ws, s));
                break;
            }
            case TMPS_CONV2D:
                TMPS_GEMM(conv_forward(dt, in, st->wptr(L), st->bptr(L), out, conv_shape(L.d, mb), L.relu, ws, s));
                break;
            case TMPS_MAXPOOL:
                TMPS_RUN(kcPoolFwd, s, maxpool_forward(dt, in, out, mb, d[0], d[1], d[2], d[3], d[4], s));
                break;
            case TMPS_LAYERNORM:
                TMPS_GEMM(layernorm_forward(dt, in, st->master + L.w_off, st->master + L.b_off, out,
                                            reinterpret_cast<float*>(st->stash + L.aux_off) + (size_t)row0 * L.rps * 2,
                                            (int64_t)mb * L.rps, d[0], 1e-5f, s));
                break;
            case TMPS_ATTENTION:
                TMPS_GEMM(attention_forward(dt, in, out,
                                            reinterpret_cast<float*>(st->stash + L.aux_off) + (size_t)row0 * d[2] * d[0], mb,
                                            d[0], d[1], d[2], s));
                break;
            case TMPS_EMBEDDING:
                TMPS_GEMM(embedding_forward(dt, (const int32_t*)in, st->wptr(L), st->bptr_c(L), out, (int64_t)mb * d[1], d[1],
                                            d[2], d[0], s));
                break;
            case TMPS_SOFTMAX_CE: {
                float* rl = stage_row_loss(st, slot);
                const int rows = mb * L.rps;
                TMPS_RUN(kcSoftmaxCE, s, softmax_ce(dt, (const float*)in, labels, out, rl, rows, d[0],
                                                    1.0f / ((float)st->M() * (float)L.rps), s));
                if (loss_out) TMPS_RUN(kcReduce, s, reduce_scaled_sum(rl, rows, 1.0f / (float)rows, loss_out, s));
                break;
            }
        }
        in = out;
    }
    if (y) {
        const LayerRT& L = st->cfg.is_last ? st->layers[st->layers.size() - 2] : st->layers.back();
        TMPS_RUN(kcCopy, s, hipMemcpyAsync(y, st->out_ptr(L, row0), (size_t)mb * L.out_elems * L.out_esize,
                                hipMemcpyDeviceToDevice, s));
    }
    st->slot_used[slot] = 1;
    return TMPS_OK;
}

extern "C" int tmps_backward(tmps_stage* st, const int* slots, int n_slots, const void* dy, void* dx,
                             void* hip_stream) {
    if (!st || !slots) return fail(TMPS_EINVAL, "stage or slots is null");
    const int N = st->cfg.n_micro, mb = st->cfg.micro_batch, M = st->M();
    if (n_slots != N)
        return fail(TMPS_ESLOT, "a backward pass covers the %d micro-batches of one mini-batch, got %d slots", N, n_slots);
    const int g0 = slots[0];
    if (g0 < 0 || g0 % N != 0 || g0 + N > st->cfg.max_stash)
        return fail(TMPS_ESLOT, "slots must be one group g*N..g*N+N-1; first slot is %d", g0);
    for (int j = 0; j < N; ++j) {
        if (slots[j] != g0 + j) return fail(TMPS_ESLOT, "slots of a group must be consecutive");
        if (!st->slot_used[g0 + j]) return fail(TMPS_ESLOT, "slot %d has not been forwarded", g0 + j);
    }
    if (!st->cfg.is_last && !dy) return fail(TMPS_EINVAL, "dy is null on a stage that is not the last");
    hipStream_t s = (hipStream_t)hip_stream;
    const int dt = st->cfg.dtype;
    const int64_t row0 = (int64_t)g0 * mb;

    const char* x0;
    if (st->cfg.borrow_input) {
        x0 = (const char*)st->slot_x[g0];
        const size_t step = (size_t)mb * st->in_elems * st->in_esize;
        for (int j = 1; j < N; ++j)
            if ((const char*)st->slot_x[g0 + j] != x0 + j * step)
                return fail(TMPS_ESHAPE, "borrowed inputs of a mini-batch must be consecutive in memory");
    } else {
        x0 = st->stash + st->in_off + (size_t)row0 * st->in_elems * st->in_esize;
    }

    // Gradient buffers: the gradient w.r.t. a layer's output is read while the one w.r.t. its input is written;
    // the gradient entering a residual layer is kept until the layer at the start of the connection has added it.
    char* gbuf[4];
    bool busy[4] = {false, false, false, false};
    for (int k = 0; k < st->n_gbuf; ++k) gbuf[k] = st->scratch + st->gbuf_off[k];
    auto take = [&]() -> int {
        for (int k = 0; k < st->n_gbuf; ++k)
            if (!busy[k]) {
                busy[k] = true;
                return k;
            }
        return -1;
    };
    const int nl = (int)st->layers.size();
    std::vector<const void*> held(nl, nullptr);   // by the layer whose input gradient it is added to
    std::vector<int> held_buf(nl, -1);
    float* ws = reinterpret_cast<float*>(st->scratch + st->ws_off);
    int cur = -1;  // which buffer holds g, -1: memory that is not ours
    const void* g;
    int top = nl - 1;
    if (st->cfg.is_last) {
        g = st->out_ptr(st->layers[top], row0);  // softmax error signal stored by the forward passes
        --top;
    } else {
        g = dy;
        const LayerRT& T = st->layers[top];
        if (T.relu) {
            cur = take();
            TMPS_RUN(kcReluMask, s, relu_mask(dt, dy, st->out_ptr(T, row0), gbuf[cur], (int64_t)M * T.out_elems, s));
            g = gbuf[cur];
        }
    }
    for (int li = top; li >= 0; --li) {
        const LayerRT& L = st->layers[li];
        const int32_t* d = L.d.dims;
        const void* in = layer_input(st, li, x0, row0);
        const bool want_dx = (li > 0 || dx != nullptr) && L.d.kind != TMPS_EMBEDDING;
        void* dst = nullptr;
        int dst_buf = -1;
        if (want_dx) {
            if (li == 0) {
                dst = dx;
            } else {
                dst_buf = take();
                if (dst_buf < 0) return fail(TMPS_EUNSUPPORTED, "out of gradient buffers (nested residual connections)");
                dst = gbuf[dst_buf];
            }
        }
        // the gradient written for the layer below passes through that layer's stored activation
        const void* mask = nullptr;
        int mask_mode = 1;
        if (li > 0) {
            const LayerRT& Bl = st->layers[li - 1];
            if (Bl.act == 1) mask = in;
            if (Bl.act == 2) {
                mask = st->stash + Bl.z_off + (size_t)row0 * Bl.out_elems * st->asz;
                mask_mode = 2;
            }
        }
        float* gw = st->grad + L.w_off;
        bool keep_g = false;
        if (held[li] && L.d.kind != TMPS_LAYERNORM) return fail(TMPS_EUNSUPPORTED, "residual connection into layer kind %d", L.d.kind);
        switch (L.d.kind) {
            case TMPS_LINEAR: {
                const int rows = M * L.rps;
                if (L.skip) {
                    held[li - L.skip] = g;
                    held_buf[li - L.skip] = cur;
                    keep_g = true;
                }
                TMPS_GEMM(dense_wgrad(dt, g, in, gw, rows, d[0], d[1], ws, s));
                if (want_dx) TMPS_GEMM(dense_dgrad(dt, g, st->wptr(L), dst, mask, mask_mode, rows, d[0], d[1], ws, s));
                break;
            }
            case TMPS_CONV2D: {
                ConvShape c = conv_shape(L.d, M);
                TMPS_GEMM(conv_wgrad(dt, g, in, gw, c, ws, s));
                if (want_dx) TMPS_GEMM(conv_dgrad(dt, g, st->wptr(L), dst, mask, c, ws, s));
                break;
            }
            case TMPS_MAXPOOL:
                if (want_dx)
                    TMPS_RUN(kcPoolBwd, s, maxpool_backward(dt, in, g, dst, M, d[0], d[1], d[2], d[3], d[4], mask ? 1 : 0, s));
                break;
            case TMPS_LAYERNORM:
                if (mask) return fail(TMPS_EUNSUPPORTED, "layer normalisation directly after an activation");
                TMPS_GEMM(layernorm_backward(dt, g, in, reinterpret_cast<const float*>(st->stash + L.aux_off) + (size_t)row0 * L.rps * 2,
                                             st->master + L.w_off, held[li], want_dx ? dst : nullptr, gw, ws, (int64_t)M * L.rps,
                                             d[0], s));
                if (held_buf[li] >= 0) busy[held_buf[li]] = false;
                held[li] = nullptr;
                break;
            case TMPS_ATTENTION:
                if (mask) return fail(TMPS_EUNSUPPORTED, "attention directly after an activation");
                if (want_dx)
                    TMPS_GEMM(attention_backward(dt, in, st->out_ptr(L, row0), g,
                                                 reinterpret_cast<const float*>(st->stash + L.aux_off) + (size_t)row0 * d[2] * d[0], ws,
                                                 dst, M, d[0], d[1], d[2], s));
                break;
            case TMPS_EMBEDDING:
                TMPS_GEMM(embedding_backward(dt, (const int32_t*)in, g, gw, st->grad + L.b_off, M, d[1], d[2], d[0], s));
                break;
            default:
                return fail(TMPS_EUNSUPPORTED, "layer kind %d has no backward", L.d.kind);
        }
        if (cur >= 0 && !keep_g) busy[cur] = false;
        if (want_dx && li > 0) {
            cur = dst_buf;
            g = dst;
        }
    }
    for (int j = 0; j < N; ++j) {
        st->slot_used[g0 + j] = 0;
        st->slot_x[g0 + j] = nullptr;
    }
    return TMPS_OK;
}

extern "C" int tmps_update(tmps_stage* st, void* hip_stream) {
    if (!st) return fail(TMPS_EINVAL, "stage is null");
    hipStream_t s = (hipStream_t)hip_stream;
    {
        // an empty bracket: what a pair of timing events costs by itself on this stream
        ProfileScope empty(kcEventPair, s);
    }
    TMPS_RUN(kcUpdate, s, sgd_momentum(st->master, st->mom, st->grad, st->wcopy, st->P, st->cfg.lr, st->cfg.momentum, s));
    ++st->version;
    return TMPS_OK;
}

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
    st.ws_fwd_bytes = 0;
    const int mb = cfg->micro_batch;
    const int M = mb * cfg->n_micro;
    const int64_t rows_all = (int64_t)cfg->max_stash * mb;
    int64_t poff = 0, gmax = 0;
    size_t soff = 0, ws = 0;
    bool any_skip = false, any_join = false;
    for (int i = 0; i < n_layers; ++i) {
        LayerRT L;
        L.d = layers[i];
        const int32_t* d = L.d.dims;
        L.relu = (L.d.flags & TMPS_FLAG_RELU) != 0;
        L.act = L.relu ? 1 : ((L.d.flags & TMPS_FLAG_GELU) ? 2 : 0);
        L.in_t = i - 1;
        const int src = (L.d.flags >> 8) & 0xff;
        if (src > 1) {
            if (L.d.kind != TMPS_CONV2D) return fail(TMPS_EUNSUPPORTED, "layer %d: only a convolution can read an earlier layer's result", i);
            if (i - src < -1) return fail(TMPS_ESHAPE, "layer %d: its source lies before the stage input", i);
            L.in_t = i - src;
            any_join = true;
        }
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
                L.ws_fwd_elems = gemm_workspace_elems(rf, d[1], d[0], 0);
                L.ws_elems = std::max({L.ws_fwd_elems, gemm_workspace_elems(rb, d[0], d[1], 0),
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
                L.ws_fwd_elems = gemm_workspace_elems((int64_t)mb * c.Ho * c.Wo, c.Cout, kf, 0);
                L.ws_elems = std::max({L.ws_fwd_elems,
                                       gemm_workspace_elems((int64_t)M * c.H * c.W, c.Cin, kd, 0),
                                       gemm_workspace_elems(c.Cout, kf, (int64_t)M * c.Ho * c.Wo, 1)});
                break;
            }
            case TMPS_MAXPOOL: {
                if (d[0] < 1 || d[1] < 1 || d[2] < 1 || d[3] < 1 || d[4] < 1 || d[5] < 0 || d[5] >= d[3] ||
                    d[3] > d[0] + 2 * d[5] || d[3] > d[1] + 2 * d[5])
                    return fail(TMPS_EINVAL, "layer %d: bad pooling dims", i);
                int Ho = (d[0] + 2 * d[5] - d[3]) / d[4] + 1, Wo = (d[1] + 2 * d[5] - d[3]) / d[4] + 1;
                L.in_elems = (int64_t)d[0] * d[1] * d[2];
                L.out_elems = (int64_t)Ho * Wo * d[2];
                L.relu = false; L.act = 0;
                break;
            }
            case TMPS_AFFINE:
                if (d[0] < 1 || d[1] < 1 || d[2] < 1) return fail(TMPS_EINVAL, "layer %d: affine dims must be positive", i);
                if (L.act == 2) return fail(TMPS_EUNSUPPORTED, "layer %d: GELU on an affine layer is not built", i);
                if (i == 0 || st.layers[i - 1].act != 0)
                    return fail(TMPS_EUNSUPPORTED, "layer %d: an affine layer must follow a layer without activation", i);
                L.in_elems = L.out_elems = (int64_t)d[0] * d[1] * d[2];
                L.w_count = d[2]; L.b_count = d[2];
                L.ws_elems = affine_workspace_elems((int64_t)M * d[0] * d[1], d[2]);
                break;
            case TMPS_RESADD:
                if (d[0] < 1 || d[1] < 1 || d[2] < 1 || d[3] < 1) return fail(TMPS_EINVAL, "layer %d: bad residual join", i);
                if (L.act == 2) return fail(TMPS_EUNSUPPORTED, "layer %d: GELU on a residual join is not built", i);
                if (i == 0 || i - d[3] < -1) return fail(TMPS_ESHAPE, "layer %d: a source of the join lies before the stage input", i);
                if (st.layers[i - 1].act != 0)
                    return fail(TMPS_EUNSUPPORTED, "layer %d: the layer before a residual join must have no activation", i);
                L.in_b = i - d[3];
                L.in_elems = L.out_elems = (int64_t)d[0] * d[1] * d[2];
                any_join = true;
                break;
            case TMPS_AVGPOOL:
                if (d[0] < 1 || d[1] < 1 || d[2] < 1) return fail(TMPS_EINVAL, "layer %d: pooling dims must be positive", i);
                L.in_elems = (int64_t)d[0] * d[1] * d[2];
                L.out_elems = d[2];
                L.relu = false; L.act = 0;
                break;
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
        if (i == 0) st.in_elems = L.in_elems;
        for (int t : {L.in_t, L.d.kind == TMPS_RESADD ? L.in_b : L.in_t}) {
            const int64_t have = t < 0 ? st.in_elems : st.layers[t].out_elems;
            if (have != L.in_elems)
                return fail(TMPS_ESHAPE, "layer %d expects %lld input elements per sample, its source gives %lld", i,
                            (long long)L.in_elems, (long long)have);
        }
        if (L.w_count) {
            L.w_off = poff;
            L.b_off = poff + L.w_count;
            poff = (int64_t)align_up((size_t)(L.b_off + L.b_count), 64);
        }
        // the gradient w.r.t. this layer's input lives in a gradient buffer (the loss layer's is kept in the stash)
        if (i > 0 && L.d.kind != TMPS_SOFTMAX_CE) gmax = std::max(gmax, L.in_elems);
        ws = std::max(ws, L.ws_elems);
        st.ws_fwd_bytes = std::max(st.ws_fwd_bytes, L.ws_fwd_elems * 4);
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
    if (cfg->is_last) {
        st.lab_off = soff;
        soff = align_up(soff + (size_t)rows_all * st.label_rps * 4, 256);
    }
    st.stash_bytes = soff;

    // scratch: gradient buffers of M rows, two boundary-gradient buffers, fp32 workspace
    size_t o = 0;
    st.n_gbuf = any_join ? 6 : (any_skip ? 4 : 2);
    // how many layers read each result (the backward pass collects one gradient contribution per reader)
    st.readers.assign(n_layers + 1, 0);
    for (int i = 0; i < n_layers; ++i) {
        const LayerRT& L = st.layers[i];
        if (L.d.kind == TMPS_EMBEDDING) continue;
        ++st.readers[L.in_t + 1];
        if (L.d.kind == TMPS_RESADD) ++st.readers[L.in_b + 1];
        if (L.d.kind == TMPS_LINEAR && L.skip) ++st.readers[st.layers[i - L.skip].in_t + 1];
    }
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

static size_t params_region_bytes(const tmps_stage& st) {
    return align_up((size_t)st.P * (st.cfg.dtype == TMPS_BF16_F32MASTER ? 6 : 4), 256);
}

extern "C" int tmps_stage_set_shadow(tmps_stage* stage, void* shadow, size_t bytes, int n_versions) {
    if (!stage) return fail(TMPS_EINVAL, "stage is null");
    if (n_versions < 0 || (n_versions > 0 && !shadow)) return fail(TMPS_EINVAL, "shadow region is null or n_versions negative");
    if (reinterpret_cast<uintptr_t>(shadow) & 255) return fail(TMPS_EINVAL, "the shadow region must be 256-byte aligned");
    const size_t one = params_region_bytes(*stage);
    if (bytes < one * (size_t)n_versions)
        return fail(TMPS_EINVAL, "%d versions of %zu bytes need %zu bytes, got %zu", n_versions, one, one * (size_t)n_versions, bytes);
    for (char u : stage->slot_used)
        if (u) return fail(TMPS_ESLOT, "a stash slot is in use");
    stage->shadow = n_versions ? (char*)shadow : nullptr;
    stage->shadow_n = n_versions;
    stage->param_bytes = one;
    stage->shadow_ver.assign((size_t)n_versions, -1L);
    return TMPS_OK;
}

extern "C" int tmps_stage_set_version(tmps_stage* stage, long version) {
    if (!stage) return fail(TMPS_EINVAL, "stage is null");
    if (version < 0) return fail(TMPS_EINVAL, "version %ld is negative", version);
    for (char u : stage->slot_used)
        if (u) return fail(TMPS_ESLOT, "a stash slot is in use: the version is restored between mini-batches");
    stage->version = version;
    std::fill(stage->shadow_ver.begin(), stage->shadow_ver.end(), -1L);   // kept copies belong to the old numbering
    return TMPS_OK;
}

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
// Runs `work` (which launches kernels on stream s and nothing else) either directly or, on a stage that replays
// graphs, as a captured graph: the first call with a key runs directly (one-off argument sets are never captured, and
// every kernel's first-launch set-up happens outside a capture), the second is captured, instantiated and launched,
// later ones launch the instantiated graph.  While per-kernel timing is on, and on the default stream, everything
// runs directly.
std::shared_mutex& tmps::capture_lock() {
    static std::shared_mutex m;
    return m;
}

template <class Work> static int run_or_replay(tmps_stage* st, const tmps_stage::GraphKey& key, hipStream_t s, Work&& work) {
    if (!st->use_graphs || s == nullptr || profile_on()) return work();   // (the default stream cannot be captured)
    auto it = st->graphs.find(key);
    if (it != st->graphs.end()) {
        TMPS_HIP(hipGraphLaunch(it->second, s));
        return TMPS_OK;
    }
    if (st->graph_seen.size() > 4096) st->graph_seen.clear();   // addresses that never repeat: forget them
    if (++st->graph_seen[key] < 2) return work();
    hipGraph_t graph = nullptr;
    int rc;
    hipError_t e;
    {
        std::unique_lock<std::shared_mutex> alone(capture_lock());
        TMPS_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
        rc = work();
        e = hipStreamEndCapture(s, &graph);
    }
    if (rc != TMPS_OK || e != hipSuccess || !graph) {
        if (graph) (void)hipGraphDestroy(graph);
        if (rc != TMPS_OK) return rc;
        return fail(TMPS_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
    }
    hipGraphExec_t exec = nullptr;
    const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (ei != hipSuccess) return fail(TMPS_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(ei));
    st->graph_seen.erase(key);
    st->graphs[key] = exec;
    TMPS_HIP(hipGraphLaunch(exec, s));
    return TMPS_OK;
}

extern "C" int tmps_stage_use_graphs(tmps_stage* st, int on) {
    if (!st) return fail(TMPS_EINVAL, "stage is null");
    st->use_graphs = on != 0;
    return TMPS_OK;
}

static const void* layer_input(const tmps_stage* st, int li, const void* x0, int64_t row0) {
    return li == 0 ? x0 : (const void*)st->out_ptr(st->layers[li - 1], row0);
}

extern "C" int tmps_forward_micro(tmps_stage* st, int slot, const void* x, void* y, const int32_t* labels,
                                  float* loss_out, void* hip_stream) {
    if (!st) return fail(TMPS_EINVAL, "stage or x is null");
    return forward_with_workspace(st, slot, x, y, labels, loss_out, hip_stream, reinterpret_cast<float*>(st->scratch + st->ws_off));
}

int tmps::forward_with_workspace(tmps_stage* st, int slot, const void* x, void* y, const int32_t* labels, float* loss_out,
                                 void* hip_stream, float* ws) {
    if (!st || !x) return fail(TMPS_EINVAL, "stage or x is null");
    if (slot < 0 || slot >= st->cfg.max_stash) return fail(TMPS_ESLOT, "slot %d outside 0..%d", slot, st->cfg.max_stash - 1);
    if (st->slot_used[slot]) return fail(TMPS_ESLOT, "slot %d is in use", slot);
    if (st->cfg.is_last && !labels) return fail(TMPS_EINVAL, "the last stage needs labels");
    hipStream_t s = (hipStream_t)hip_stream;
    const int mb = st->cfg.micro_batch;
    const int dt = st->cfg.dtype;
    const int64_t row0 = (int64_t)slot * mb;
    const void* x0 = x;
    if (!st->cfg.borrow_input) {
        char* dst = st->stash + st->in_off + (size_t)row0 * st->in_elems * st->in_esize;
        TMPS_RUN(kcCopy, s, hipMemcpyAsync(dst, x, (size_t)mb * st->in_elems * st->in_esize, hipMemcpyDeviceToDevice, s));
        x0 = dst;
    }
    st->slot_x[slot] = x;
    if (st->use_graphs && st->cfg.is_last) {
        // a captured loss kernel reads its labels at a fixed address: the stage's own copy of this slot's labels
        int32_t* lab = reinterpret_cast<int32_t*>(st->stash + st->lab_off) + (size_t)row0 * st->label_rps;
        TMPS_RUN(kcCopy, s, hipMemcpyAsync(lab, labels, (size_t)mb * st->label_rps * 4, hipMemcpyDeviceToDevice, s));
        labels = lab;
    }
    const tmps_stage::GraphKey key = {1, (uintptr_t)slot, (uintptr_t)x0, (uintptr_t)labels, (uintptr_t)loss_out, (uintptr_t)ws,
                                      (uintptr_t)st->master, (uintptr_t)st->wcopy};
    const int rc = run_or_replay(st, key, s, [&]() -> int {
    for (size_t li = 0; li < st->layers.size(); ++li) {
        const LayerRT& L = st->layers[li];
        void* out = st->out_ptr(L, row0);
        const int32_t* d = L.d.dims;
        const void* in = L.in_t < 0 ? x0 : (const void*)st->out_ptr(st->layers[L.in_t], row0);
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
            case TMPS_CONV2D: {
                // A convolution without activation whose only reader is a per-channel affine layer runs fused with
                // it, and with the residual join after the affine layer when that follows directly.
                const size_t nl = st->layers.size();
                if (L.act == 0 && li + 1 < nl && st->layers[li + 1].d.kind == TMPS_AFFINE && st->readers[li + 1] == 1) {
                    const LayerRT& A = st->layers[li + 1];
                    const bool join = !A.relu && li + 2 < nl && st->layers[li + 2].d.kind == TMPS_RESADD &&
                                      st->readers[li + 2] == 1;
                    void* aout = st->out_ptr(A, row0);
                    if (join) {
                        // the affine result itself is not stored: only the join reads it, and no gradient needs it
                        const LayerRT& J = st->layers[li + 2];
                        const void* b = J.in_b < 0 ? x0 : (const void*)st->out_ptr(st->layers[J.in_b], row0);
                        TMPS_GEMM(conv_affine_forward(dt, in, st->wptr(L), st->bptr(L), out, st->master + A.w_off, st->master + A.b_off,
                                                      nullptr, b, st->out_ptr(J, row0), J.relu, conv_shape(L.d, mb), ws, s));
                        li += 2;
                    } else {
                        TMPS_GEMM(conv_affine_forward(dt, in, st->wptr(L), st->bptr(L), out, st->master + A.w_off, st->master + A.b_off,
                                                      nullptr, nullptr, aout, A.relu, conv_shape(L.d, mb), ws, s));
                        li += 1;
                    }
                    break;
                }
                TMPS_GEMM(conv_forward(dt, in, st->wptr(L), st->bptr(L), out, conv_shape(L.d, mb), L.relu, ws, s));
                break;
            }
            case TMPS_MAXPOOL:
                TMPS_RUN(kcPoolFwd, s, maxpool_forward(dt, in, out, mb, d[0], d[1], d[2], d[3], d[4], d[5], s));
                break;
            case TMPS_AFFINE:
                TMPS_GEMM(affine_forward(dt, in, st->master + L.w_off, st->master + L.b_off, out, (int64_t)mb * d[0] * d[1], d[2],
                                         L.relu, s));
                break;
            case TMPS_RESADD: {
                const void* b = L.in_b < 0 ? x0 : (const void*)st->out_ptr(st->layers[L.in_b], row0);
                TMPS_GEMM(resadd_forward(dt, in, b, out, (int64_t)mb * L.out_elems, L.relu, s));
                break;
            }
            case TMPS_AVGPOOL:
                TMPS_GEMM(avgpool_forward(dt, in, out, mb, d[0] * d[1], d[2], s));
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
    }
    return TMPS_OK;
    });
    if (rc != TMPS_OK) return rc;
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
                return fail(TMPS_ESHAPE, "borrowed inputs of a mini-batch must be consecutive in memory: slot %d holds %p, expected %p (slot %d + %d x %zu bytes)",
                            g0 + j, st->slot_x[g0 + j], (const void*)(x0 + j * step), g0, j, step);
    } else {
        x0 = st->stash + st->in_off + (size_t)row0 * st->in_elems * st->in_esize;
    }
    // The arguments are accepted.  From here on the slots are given up whatever happens: a pass that fails midway
    // has written part of the gradients, and the stage must be able to take the next mini-batch.
    struct FreeSlots {
        tmps_stage* st; int g0, N;
        ~FreeSlots() {
            for (int j = 0; j < N; ++j) {
                st->slot_used[g0 + j] = 0;
                st->slot_x[g0 + j] = nullptr;
            }
        }
    } free_slots{st, g0, N};

    const tmps_stage::GraphKey key = {2, (uintptr_t)g0, (uintptr_t)x0, (uintptr_t)dy, (uintptr_t)dx, 0,
                                      (uintptr_t)st->master, (uintptr_t)st->wcopy};
    return run_or_replay(st, key, s, [&]() -> int {
    // Gradients are kept per result: grads[t + 1] is the gradient w.r.t. the result of layer t (t = -1: the stage
    // input).  Layers are visited last to first; every layer that reads a result contributes to its gradient: the
    // first contribution is written, later ones are added to what is there (in the epilogue of the kernel that
    // computes them).  Buffers come from a small pool and are shared by reference count: a residual connection
    // hands the SAME gradient to both of its sources without copying it.
    struct Grad {
        const void* ptr = nullptr;
        int buf = -1;      // pool buffer that holds it; -1: memory that is not ours to write or free (dy, the stash, dx)
        bool set = false;
    };
    const int nl = (int)st->layers.size();
    std::vector<Grad> grads(nl + 1);
    std::vector<int> remaining(st->readers);
    char* gbuf[8];
    int refs[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int k = 0; k < st->n_gbuf; ++k) gbuf[k] = st->scratch + st->gbuf_off[k];
    auto take = [&]() -> int {
        for (int k = 0; k < st->n_gbuf; ++k)
            if (refs[k] == 0) {
                refs[k] = 1;
                return k;
            }
        return -1;
    };
    auto release = [&](int buf) {
        if (buf >= 0) --refs[buf];
    };
    float* ws = reinterpret_cast<float*>(st->scratch + st->ws_off);
    // the stored activation that a gradient written for result t has to pass through (mode 1: ReLU, 2: GELU)
    auto mask_of = [&](int t, int& mode) -> const void* {
        mode = 1;
        if (t < 0) return nullptr;
        const LayerRT& P = st->layers[t];
        if (P.act == 1) return st->out_ptr(P, row0);
        if (P.act == 2) {
            mode = 2;
            return st->stash + P.z_off + (size_t)row0 * P.out_elems * st->asz;
        }
        return nullptr;
    };
    // Where the contribution of a kernel to result t goes: `dst` to write, `add` to join first (null: nothing yet).
    struct Target {
        void* dst = nullptr;
        const void* add = nullptr;
        int buf = -1;
        bool wanted = false;
    };
    auto target = [&](int t, Target& T) -> int {
        T = Target();
        Grad& G = grads[t + 1];
        if (t < 0) {
            if (!dx) return TMPS_OK;   // nobody wants the gradient w.r.t. the stage input
            T.wanted = true;
            T.dst = dx;
            T.add = G.set ? dx : nullptr;
            return TMPS_OK;
        }
        T.wanted = true;
        if (G.set && G.buf >= 0 && refs[G.buf] == 1) {   // ours alone: add in place
            T.dst = gbuf[G.buf];
            T.add = G.ptr;
            T.buf = G.buf;
            return TMPS_OK;
        }
        T.buf = take();
        if (T.buf < 0) return fail(TMPS_EUNSUPPORTED, "out of gradient buffers (too many open residual connections)");
        T.dst = gbuf[T.buf];
        T.add = G.set ? G.ptr : nullptr;
        return TMPS_OK;
    };
    auto commit = [&](int t, const Target& T) {
        Grad& G = grads[t + 1];
        if (G.set && G.buf != T.buf) release(G.buf);
        G.ptr = T.dst;
        G.buf = T.buf;
        G.set = true;
        --remaining[t + 1];
    };
    // hand an existing gradient (g) to result t as its contribution, without a kernel when it is the first
    auto share = [&](int t, const Grad& g) -> int {
        if (t < 0 && !dx) return TMPS_OK;
        Grad& G = grads[t + 1];
        const int64_t n = (int64_t)M * st->tensor_elems(t);
        if (t < 0) {
            if (G.set) TMPS_GEMM(resadd_forward(dt, dx, g.ptr, dx, n, 0, s));
            else TMPS_RUN(kcCopy, s, copy_bytes(dx, g.ptr, (size_t)n * st->asz, s));
            G.ptr = dx; G.buf = -1; G.set = true;
        } else if (!G.set) {
            G = g;
            if (g.buf >= 0) ++refs[g.buf];
        } else {
            Target T;
            int rc = target(t, T);
            if (rc != TMPS_OK) return rc;
            TMPS_GEMM(resadd_forward(dt, T.add, g.ptr, T.dst, n, 0, s));
            if (G.buf != T.buf) release(G.buf);
            G.ptr = T.dst; G.buf = T.buf;
        }
        --remaining[t + 1];
        return TMPS_OK;
    };

    int top = nl - 1;
    if (st->cfg.is_last) {
        // the loss layer's contribution to the logits: the softmax error signal stored by the forward passes
        Grad& G = grads[top];   // result top - 1
        G.ptr = st->out_ptr(st->layers[top], row0);
        G.buf = -1;
        G.set = true;
        --remaining[top];
        --top;
    } else {
        Grad& G = grads[top + 1];
        G.ptr = dy;
        G.buf = -1;
        G.set = true;
        const LayerRT& T = st->layers[top];
        if (T.relu) {
            const int k = take();
            TMPS_RUN(kcReluMask, s, relu_mask(dt, dy, st->out_ptr(T, row0), gbuf[k], (int64_t)M * T.out_elems, s));
            G.ptr = gbuf[k];
            G.buf = k;
        }
    }
    for (int li = top; li >= 0; --li) {
        const LayerRT& L = st->layers[li];
        const int32_t* d = L.d.dims;
        const Grad g = grads[li + 1];
        if (!g.set || remaining[li + 1] != 0) return fail(TMPS_ESHAPE, "layer %d: its result has no complete gradient", li);
        const int t_in = L.in_t;
        const void* in = t_in < 0 ? (const void*)x0 : (const void*)st->out_ptr(st->layers[t_in], row0);
        int mask_mode = 1;
        const void* mask = mask_of(t_in, mask_mode);
        float* gw = st->grad + L.w_off;
        Target T;
        int rc;
        switch (L.d.kind) {
            case TMPS_LINEAR: {
                const int rows = M * L.rps;
                if (L.skip && (rc = share(st->layers[li - L.skip].in_t, g)) != TMPS_OK) return rc;
                TMPS_GEMM(dense_wgrad(dt, g.ptr, in, gw, rows, d[0], d[1], ws, s));
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                if (T.wanted) {
                    TMPS_GEMM(dense_dgrad(dt, g.ptr, st->wptr(L), T.dst, mask, mask_mode, T.add, rows, d[0], d[1], ws, s));
                    commit(t_in, T);
                }
                break;
            }
            case TMPS_CONV2D: {
                ConvShape c = conv_shape(L.d, M);
                TMPS_GEMM(conv_wgrad(dt, g.ptr, in, gw, c, ws, s));
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                if (T.wanted) {
                    if (mask_mode == 2) return fail(TMPS_EUNSUPPORTED, "a convolution directly after a GELU layer");
                    TMPS_GEMM(conv_dgrad(dt, g.ptr, st->wptr(L), T.dst, mask, T.add, c, ws, s));
                    commit(t_in, T);
                }
                break;
            }
            case TMPS_MAXPOOL:
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                if (T.wanted) {
                    if (T.add || mask_mode == 2) return fail(TMPS_EUNSUPPORTED, "max pooling on a shared or GELU input");
                    TMPS_RUN(kcPoolBwd, s, maxpool_backward(dt, in, g.ptr, T.dst, M, d[0], d[1], d[2], d[3], d[4], d[5], mask ? 1 : 0, s));
                    commit(t_in, T);
                }
                break;
            case TMPS_AVGPOOL:
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                if (T.wanted) {
                    if (T.add || mask_mode == 2) return fail(TMPS_EUNSUPPORTED, "average pooling on a shared or GELU input");
                    TMPS_GEMM(avgpool_backward(dt, g.ptr, in, T.dst, M, d[0] * d[1], d[2], mask ? 1 : 0, s));
                    commit(t_in, T);
                }
                break;
            case TMPS_AFFINE:
                // the layer before has no activation (checked at creation): nothing to pass through
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                if (T.add) return fail(TMPS_EUNSUPPORTED, "an affine layer on a shared input");
                TMPS_GEMM(affine_backward(dt, g.ptr, in, st->master + L.w_off, T.wanted ? T.dst : nullptr, gw, ws,
                                          (int64_t)M * d[0] * d[1], d[2], s));
                if (T.wanted) commit(t_in, T);
                break;
            case TMPS_RESADD:
                // d(a + b) = the incoming gradient for both sources (it has already passed through this layer's ReLU)
                if ((rc = share(L.in_b, g)) != TMPS_OK) return rc;
                if ((rc = share(t_in, g)) != TMPS_OK) return rc;
                break;
            case TMPS_LAYERNORM:
                if (mask) return fail(TMPS_EUNSUPPORTED, "layer normalisation directly after an activation");
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                TMPS_GEMM(layernorm_backward(dt, g.ptr, in, reinterpret_cast<const float*>(st->stash + L.aux_off) + (size_t)row0 * L.rps * 2,
                                             st->master + L.w_off, T.add, T.wanted ? T.dst : nullptr, gw, ws, (int64_t)M * L.rps,
                                             d[0], s));
                if (T.wanted) commit(t_in, T);
                break;
            case TMPS_ATTENTION:
                if (mask) return fail(TMPS_EUNSUPPORTED, "attention directly after an activation");
                if ((rc = target(t_in, T)) != TMPS_OK) return rc;
                if (T.wanted) {
                    if (T.add) return fail(TMPS_EUNSUPPORTED, "attention on a shared input");
                    TMPS_GEMM(attention_backward(dt, in, st->out_ptr(L, row0), g.ptr,
                                                 reinterpret_cast<const float*>(st->stash + L.aux_off) + (size_t)row0 * d[2] * d[0], ws,
                                                 T.dst, M, d[0], d[1], d[2], s));
                    commit(t_in, T);
                }
                break;
            case TMPS_EMBEDDING:
                TMPS_GEMM(embedding_backward(dt, (const int32_t*)in, g.ptr, gw, st->grad + L.b_off, M, d[1], d[2], d[0], s));
                break;
            default:
                return fail(TMPS_EUNSUPPORTED, "layer kind %d has no backward", L.d.kind);
        }
        release(g.buf);
        grads[li + 1].set = false;
        // A result whose gradient is complete but was only handed over (never written through a kernel that applies
        // the activation of its producer) still has to pass through that activation.
        if (t_in >= 0 && remaining[t_in + 1] == 0 && grads[t_in + 1].set && L.d.kind == TMPS_RESADD) {
            int mm = 1;
            const void* mk = mask_of(t_in, mm);
            if (mk) return fail(TMPS_EUNSUPPORTED, "a residual join whose first source ends in an activation");
        }
        if (L.d.kind == TMPS_RESADD && L.in_b >= 0 && remaining[L.in_b + 1] == 0 && st->layers[L.in_b].act != 0)
            return fail(TMPS_EUNSUPPORTED, "a residual connection must start at a result that another, earlier layer reads too");
    }
    return TMPS_OK;
    });   // (free_slots releases the group)
}

extern "C" int tmps_update(tmps_stage* st, void* hip_stream) {
    if (!st) return fail(TMPS_EINVAL, "stage is null");
    hipStream_t s = (hipStream_t)hip_stream;
    {
        // an empty bracket: what a pair of timing events costs by itself on this stream
        ProfileScope empty(kcEventPair, s);
    }
    if (st->shadow_n > 0) {
        // vertical weight stashing: the version about to be superseded is kept for the forward passes tagged with it
        const int slot = (int)(st->version % st->shadow_n);
        TMPS_RUN(kcCopy, s, hipMemcpyAsync(st->shadow + (size_t)slot * st->param_bytes, st->params, st->param_bytes,
                                           hipMemcpyDeviceToDevice, s));
        st->shadow_ver[slot] = st->version;
    }
    TMPS_RUN(kcUpdate, s, sgd_momentum(st->master, st->mom, st->grad, st->wcopy, st->P, st->cfg.lr, st->cfg.momentum, s));
    ++st->version;
    return TMPS_OK;
}

extern "C" int tmps_backward_at(tmps_stage* st, long version, const int* slots, int n_slots, const void* dy, void* dx,
                                void* hip_stream) {
    if (!st) return fail(TMPS_EINVAL, "stage is null");
    if (version == st->version) return tmps_backward(st, slots, n_slots, dy, dx, hip_stream);
    int found = -1;
    for (int k = 0; k < st->shadow_n; ++k)
        if (st->shadow_ver[k] == version) found = k;
    if (found < 0)
        return fail(TMPS_EINVAL, "weights after %ld updates are not kept (the stage is at %ld and keeps %d older versions)",
                    version, st->version, st->shadow_n);
    // as in tmps_forward_micro_at: the kernels take their weight pointers at launch; the gradients still go to the
    // stage's own gradient array, and the update that follows changes the live weights
    float* const live_master = st->master;
    void* const live_wcopy = st->wcopy;
    char* base = st->shadow + (size_t)found * st->param_bytes;
    st->master = reinterpret_cast<float*>(base);
    if (live_wcopy) st->wcopy = base + (size_t)st->P * 4;
    const int rc = tmps_backward(st, slots, n_slots, dy, dx, hip_stream);
    st->master = live_master;
    st->wcopy = live_wcopy;
    return rc;
}

extern "C" int tmps_forward_micro_at(tmps_stage* st, long version, int slot, const void* x, void* y, const int32_t* labels,
                                     float* loss_out, void* hip_stream) {
    if (!st) return fail(TMPS_EINVAL, "stage is null");
    if (version == st->version) return tmps_forward_micro(st, slot, x, y, labels, loss_out, hip_stream);
    int found = -1;
    for (int k = 0; k < st->shadow_n; ++k)
        if (st->shadow_ver[k] == version) found = k;
    if (found < 0)
        return fail(TMPS_EINVAL, "weights after %ld updates are not kept (the stage is at %ld and keeps %d older versions)",
                    version, st->version, st->shadow_n);
    // The kernels take their weight pointers when they are launched: point the stage at the kept copy for the
    // duration of this call.  (Calls on one stage come from one host thread at a time.)
    float* const live_master = st->master;
    void* const live_wcopy = st->wcopy;
    char* base = st->shadow + (size_t)found * st->param_bytes;
    st->master = reinterpret_cast<float*>(base);
    if (live_wcopy) st->wcopy = base + (size_t)st->P * 4;
    const int rc = tmps_forward_micro(st, slot, x, y, labels, loss_out, hip_stream);
    st->master = live_master;
    st->wcopy = live_wcopy;
    return rc;
}

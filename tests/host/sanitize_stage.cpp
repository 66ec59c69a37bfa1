// Host-only driver for a sanitizer build (g++ -fsanitize=address,undefined) of the stage executor's host logic
// (paper_2410_14312_amd/csrc/stage.cpp, with tests/host/kernel_stubs.cpp in place of the kernel launchers and
// csrc/profile.cpp left as it is: profiling stays off, so no HIP call is made).  It walks the layout and
// argument checks: valid layer lists of every kind, lists that do not chain, sources before the stage, bad
// enums and sizes, a few thousand random descriptor lists; then the slot and buffer bookkeeping of forward /
// backward / update on a created stage whose "device" regions are plain aligned host memory (the stubs launch nothing).
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/tmps.h"

static int bad = 0;
static void expect(bool ok, const char* what) {
    if (!ok) {
        fprintf(stderr, "FAILED: %s (%s)\n", what, tmps_last_error());
        ++bad;
    }
}

static tmps_layer_desc L(int kind, std::initializer_list<int> dims, int flags = 0) {
    tmps_layer_desc d;
    memset(&d, 0, sizeof(d));
    d.kind = kind;
    int i = 0;
    for (int v : dims) d.dims[i++] = v;
    d.flags = flags;
    return d;
}

static tmps_stage_cfg cfg(int dtype, int micro, int N, int stash, int last, int borrow) {
    tmps_stage_cfg c;
    c.dtype = dtype; c.micro_batch = micro; c.n_micro = N; c.max_stash = stash; c.is_last = last; c.borrow_input = borrow;
    c.lr = 0.01f; c.momentum = 0.9f;
    return c;
}

static int bytes(const std::vector<tmps_layer_desc>& ls, const tmps_stage_cfg& c, size_t out[4]) {
    return tmps_stage_bytes(ls.data(), (int)ls.size(), &c, &out[0], &out[1], &out[2], &out[3]);
}

struct Regions {
    void* p[4];
    explicit Regions(const size_t sz[4]) {
        for (int i = 0; i < 4; ++i) p[i] = aligned_alloc(256, (sz[i] + 255) / 256 * 256 + 256);
    }
    ~Regions() {
        for (void* q : p) free(q);
    }
};

static unsigned rnd_state = 12345;
static int rnd(int n) {
    rnd_state = rnd_state * 1664525u + 1013904223u;
    return (int)((rnd_state >> 8) % (unsigned)n);
}

int main() {
    size_t sz[4];
    const int R = TMPS_FLAG_RELU;
    // ---- valid lists of every layer kind ----
    std::vector<tmps_layer_desc> mlp = {L(TMPS_LINEAR, {64, 128, 0, 1}, R), L(TMPS_LINEAR, {128, 10, 0, 1}), L(TMPS_SOFTMAX_CE, {10, 1})};
    expect(bytes(mlp, cfg(TMPS_F32, 8, 4, 8, 1, 0), sz) == TMPS_OK, "mlp");
    std::vector<tmps_layer_desc> tf = {L(TMPS_EMBEDDING, {50, 6, 16}), L(TMPS_LAYERNORM, {16, 6}), L(TMPS_LINEAR, {16, 48, 0, 6}),
                                      L(TMPS_ATTENTION, {6, 16, 2}), L(TMPS_LINEAR, {16, 16, 3, 6}), L(TMPS_LAYERNORM, {16, 6}),
                                      L(TMPS_LINEAR, {16, 24, 0, 6}, TMPS_FLAG_GELU), L(TMPS_LINEAR, {24, 16, 2, 6}),
                                      L(TMPS_LAYERNORM, {16, 6}), L(TMPS_LINEAR, {16, 50, 0, 6}), L(TMPS_SOFTMAX_CE, {50, 6})};
    expect(bytes(tf, cfg(TMPS_BF16_F32MASTER, 2, 2, 4, 1, 0), sz) == TMPS_OK, "transformer");
    std::vector<tmps_layer_desc> res = {L(TMPS_CONV2D, {8, 8, 8, 4, 1, 1, 1, 0}), L(TMPS_AFFINE, {8, 8, 4}, R),
                                       L(TMPS_CONV2D, {8, 8, 4, 4, 3, 3, 2, 1}), L(TMPS_AFFINE, {4, 4, 4}, R),
                                       L(TMPS_CONV2D, {4, 4, 4, 16, 1, 1, 1, 0}), L(TMPS_AFFINE, {4, 4, 16}),
                                       L(TMPS_CONV2D, {8, 8, 8, 16, 1, 1, 2, 0}, TMPS_FLAG_SRC(7)), L(TMPS_AFFINE, {4, 4, 16}),
                                       L(TMPS_RESADD, {4, 4, 16, 3}, R), L(TMPS_MAXPOOL, {4, 4, 16, 2, 2, 0}),
                                       L(TMPS_AVGPOOL, {2, 2, 16}), L(TMPS_LINEAR, {16, 5, 0, 1}), L(TMPS_SOFTMAX_CE, {5, 1})};
    expect(bytes(res, cfg(TMPS_BF16_F32MASTER, 2, 2, 2, 1, 1), sz) == TMPS_OK, "residual");

    // ---- lists that must be refused ----
    auto refused = [&](std::vector<tmps_layer_desc> ls, tmps_stage_cfg c, int code, const char* what) {
        size_t s4[4];
        expect(bytes(ls, c, s4) == code, what);
    };
    refused({L(TMPS_LINEAR, {64, 128, 0, 1}), L(TMPS_LINEAR, {100, 10, 0, 1})}, cfg(0, 8, 4, 4, 0, 0), TMPS_ESHAPE, "layers that do not chain");
    refused(mlp, cfg(0, 8, 4, 6, 1, 0), TMPS_EMICRO, "stash not a whole number of mini-batches");
    refused(mlp, cfg(7, 8, 4, 4, 1, 0), TMPS_EINVAL, "unknown dtype");
    refused(mlp, cfg(0, 0, 4, 4, 1, 0), TMPS_EINVAL, "empty micro-batch");
    refused(mlp, cfg(0, 8, 65, 65, 1, 0), TMPS_EUNSUPPORTED, "too many micro-batches");
    refused({L(TMPS_LINEAR, {64, 10, 0, 1}), L(TMPS_SOFTMAX_CE, {10, 1})}, cfg(0, 8, 4, 4, 0, 0), TMPS_ESHAPE, "loss on a stage that is not the last");
    refused({L(TMPS_LINEAR, {64, 10, 0, 1})}, cfg(0, 8, 4, 4, 1, 0), TMPS_ESHAPE, "last stage without loss");
    refused({L(TMPS_LINEAR, {16, 16, 5, 1})}, cfg(0, 8, 4, 4, 0, 0), TMPS_ESHAPE, "residual source before the stage");
    refused({L(TMPS_LINEAR, {16, 16, 0, 1}), L(TMPS_LINEAR, {16, 16, 1, 1})}, cfg(0, 8, 4, 4, 0, 0), TMPS_EUNSUPPORTED, "residual source is no layer normalisation");
    refused({L(TMPS_CONV2D, {8, 8, 8, 4, 1, 1, 1, 0}, TMPS_FLAG_SRC(9))}, cfg(0, 2, 2, 2, 0, 0), TMPS_ESHAPE, "convolution source before the stage");
    refused({L(TMPS_LINEAR, {16, 16, 0, 1}, TMPS_FLAG_SRC(2))}, cfg(0, 2, 2, 2, 0, 0), TMPS_EUNSUPPORTED, "source flag on a linear layer");
    refused({L(TMPS_CONV2D, {8, 8, 8, 4, 1, 1, 1, 0}), L(TMPS_RESADD, {8, 8, 4, 9}, R)}, cfg(0, 2, 2, 2, 0, 0), TMPS_ESHAPE, "join source before the stage");
    refused({L(TMPS_RESADD, {8, 8, 4, 1}, R)}, cfg(0, 2, 2, 2, 0, 0), TMPS_ESHAPE, "join as the first layer");
    refused({L(TMPS_LINEAR, {16, 16, 0, 1}), L(TMPS_EMBEDDING, {50, 6, 16})}, cfg(0, 2, 2, 2, 0, 0), TMPS_ESHAPE, "embedding not first");
    refused({L(TMPS_MAXPOOL, {4, 4, 8, 9, 2, 0})}, cfg(0, 2, 2, 2, 0, 0), TMPS_EINVAL, "window larger than the map");
    refused({L(TMPS_ATTENTION, {6, 16, 3})}, cfg(0, 2, 2, 2, 0, 0), TMPS_EINVAL, "heads do not divide the width");
    refused({L(99, {1, 1})}, cfg(0, 2, 2, 2, 0, 0), TMPS_EUNSUPPORTED, "unknown layer kind");
    expect(tmps_stage_bytes(nullptr, 1, nullptr, nullptr, nullptr, nullptr, nullptr) == TMPS_EINVAL, "null descriptors");

    // ---- random descriptor lists: any answer is fine, reading or writing out of bounds is not ----
    for (int it = 0; it < 4000; ++it) {
        std::vector<tmps_layer_desc> ls;
        const int n = 1 + rnd(7);
        for (int i = 0; i < n; ++i) {
            tmps_layer_desc d;
            memset(&d, 0, sizeof(d));
            d.kind = rnd(12);
            for (int k = 0; k < 8; ++k) d.dims[k] = rnd(10) == 0 ? -rnd(3) : rnd(rnd(2) ? 9 : 40);
            d.flags = rnd(4) | (rnd(3) == 0 ? TMPS_FLAG_SRC(rnd(12)) : 0);
            ls.push_back(d);
        }
        size_t s4[4];
        const int N = 1 + rnd(3);
        (void)bytes(ls, cfg(rnd(2), 1 + rnd(3), N, N * (1 + rnd(2)), rnd(2), rnd(2)), s4);
    }

    // ---- a created stage: offsets, slots, versions; the stubs launch nothing ----
    for (auto* net : {&mlp, &tf, &res}) {
        const bool is_tf = net == &tf;
        tmps_stage_cfg c = cfg(TMPS_BF16_F32MASTER, 2, 2, 4, 1, 0);
        expect(bytes(*net, c, sz) == TMPS_OK, "sizes");
        Regions r(sz);
        tmps_stage* st = nullptr;
        expect(tmps_stage_create(&st, net->data(), (int)net->size(), &c, r.p[0], r.p[1], r.p[2], r.p[3]) == TMPS_OK && st, "create");
        if (!st) continue;
        const int64_t P = tmps_stage_param_count(st);
        for (int li = -1; li <= (int)net->size(); ++li)
            for (int which = 0; which < 3; ++which) {
                int64_t off = 0, cnt = 0;
                const int rc = tmps_stage_param_offset(st, li, which, &off, &cnt);
                if (li < 0 || li >= (int)net->size() || which > 1) expect(rc == TMPS_EINVAL, "offset query out of range");
                else expect(rc == TMPS_OK && off >= 0 && off + cnt <= P, "offset inside the parameter array");
            }
        expect(tmps_stage_output_ptr(st, -1) == nullptr && tmps_stage_output_ptr(st, 4) == nullptr, "output pointer of a bad slot");
        int32_t labels[64] = {0};
        std::vector<char> x((size_t)2 * tmps_stage_input_elems(st) * 4 + 64);
        (void)is_tf;
        expect(tmps_forward_micro(st, 4, x.data(), nullptr, labels, nullptr, nullptr) == TMPS_ESLOT, "slot out of range");
        expect(tmps_forward_micro(st, 0, x.data(), nullptr, nullptr, nullptr, nullptr) == TMPS_EINVAL, "labels missing");
        expect(tmps_forward_micro(st, 2, x.data(), nullptr, labels, nullptr, nullptr) == TMPS_OK, "forward into slot 2");
        expect(tmps_forward_micro(st, 2, x.data(), nullptr, labels, nullptr, nullptr) == TMPS_ESLOT, "slot in use");
        expect(tmps_stage_set_version(st, 3) == TMPS_ESLOT, "version change while a slot is in use");
        int slots[2] = {2, 3};
        expect(tmps_backward(st, slots, 2, nullptr, nullptr, nullptr) == TMPS_ESLOT, "slot 3 not forwarded");
        expect(tmps_forward_micro(st, 3, x.data(), nullptr, labels, nullptr, nullptr) == TMPS_OK, "forward into slot 3");
        int wrong[2] = {1, 2};
        expect(tmps_backward(st, wrong, 2, nullptr, nullptr, nullptr) == TMPS_ESLOT, "slots that are no group");
        expect(tmps_backward(st, slots, 1, nullptr, nullptr, nullptr) == TMPS_ESLOT, "not a whole mini-batch");
        expect(tmps_backward(st, slots, 2, nullptr, nullptr, nullptr) == TMPS_OK, "backward");
        expect(tmps_update(st, nullptr) == TMPS_OK && tmps_stage_version(st) == 1, "update");
        expect(tmps_forward_micro(st, 2, x.data(), nullptr, labels, nullptr, nullptr) == TMPS_OK, "slot free again");
        expect(tmps_stage_set_version(st, -1) == TMPS_EINVAL, "negative version");
        expect(tmps_stage_set_shadow(st, nullptr, 0, 2) == TMPS_EINVAL, "shadow region missing");
        tmps_stage_destroy(st);
    }
    return bad ? 1 : 0;
}

"""ctypes binding of libtmps.so: same names as the C ABI, argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtmps.so")
_lib = None

TMPS_F32, TMPS_BF16_F32MASTER = 0, 1
TMPS_LINEAR, TMPS_CONV2D, TMPS_MAXPOOL, TMPS_SOFTMAX_CE, TMPS_LAYERNORM, TMPS_ATTENTION, TMPS_EMBEDDING = 1, 2, 3, 4, 5, 6, 7
TMPS_AFFINE, TMPS_RESADD, TMPS_AVGPOOL = 8, 9, 10
TMPS_FLAG_RELU, TMPS_FLAG_GELU = 1, 2


class TmpsError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libtmps error %d: %s" % (code, text))
        self.code = code


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dims", C.c_int32 * 8), ("flags", C.c_int32)]


class StageCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("micro_batch", C.c_int32), ("n_micro", C.c_int32),
                ("max_stash", C.c_int32), ("is_last", C.c_int32), ("borrow_input", C.c_int32),
                ("lr", C.c_float), ("momentum", C.c_float)]


EXPORTS = {
    "tmps_stage_bytes": (C.c_int, [C.POINTER(LayerDesc), C.c_int, C.POINTER(StageCfg), C.POINTER(C.c_size_t),
                                   C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "tmps_stage_create": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(LayerDesc), C.c_int, C.POINTER(StageCfg),
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "tmps_stage_destroy": (None, [C.c_void_p]),
    "tmps_stage_param_count": (C.c_int64, [C.c_void_p]),
    "tmps_stage_param_offset": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "tmps_stage_input_elems": (C.c_int64, [C.c_void_p]),
    "tmps_stage_output_elems": (C.c_int64, [C.c_void_p]),
    "tmps_stage_sync_params": (C.c_int, [C.c_void_p, C.c_void_p]),
    "tmps_stage_output_ptr": (C.c_void_p, [C.c_void_p, C.c_int]),
    "tmps_stage_version": (C.c_long, [C.c_void_p]),
    "tmps_stage_set_version": (C.c_int, [C.c_void_p, C.c_long]),
    "tmps_stage_use_graphs": (C.c_int, [C.c_void_p, C.c_int]),
    "tmps_stage_set_shadow": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]),
    "tmps_forward_micro_at": (C.c_int, [C.c_void_p, C.c_long, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]),
    "tmps_schedule_shadow_versions": (C.c_int, [C.c_int, C.c_int, C.c_int]),
    "tmps_forward_micro": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "tmps_forward_micro_static": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "tmps_backward": (C.c_int, [C.c_void_p, C.POINTER(C.c_int), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "tmps_backward_at": (C.c_int, [C.c_void_p, C.c_long, C.POINTER(C.c_int), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "tmps_schedule_plan_1f1b": (C.c_int, [C.c_int, C.c_int, C.POINTER(C.c_int32), C.c_size_t]),
    "tmps_schedule_run_1f1b": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                         C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(C.c_int32)]),
    "tmps_update": (C.c_int, [C.c_void_p, C.c_void_p]),
    "tmps_schedule_plan": (C.c_int, [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32), C.c_size_t]),
    "tmps_schedule_stash_groups": (C.c_int, [C.c_int, C.c_int, C.c_int]),
    "tmps_version_diff_formula": (C.c_int, [C.c_int, C.c_int]),
    "tmps_version_diff_simulated": (C.c_int, [C.c_int, C.c_int]),
    "tmps_schedule_run": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                    C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(C.c_int32)]),
    "tmps_schedule_run_vsync": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                          C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(C.c_int32)]),
    "tmps_streams_create": (C.c_int, [C.POINTER(C.c_void_p), C.c_int]),
    "tmps_streams_destroy": (C.c_int, [C.POINTER(C.c_void_p), C.c_int]),
    "tmps_profile_enable": (C.c_int, [C.c_int]),
    "tmps_profile_read": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]),
    "tmps_last_error": (C.c_char_p, []),
}


def load_library():
    """Load libtmps.so and declare every exported symbol; raises if the library is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libtmps.so is not built (%s): run `python __graft_entry__.py`" % _LIB_PATH)
    lib_ = C.CDLL(_LIB_PATH)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib_, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib_
    return _lib


def lib():
    return load_library()


def _check(rc):
    if rc < 0:
        raise TmpsError(rc, lib().tmps_last_error().decode())
    return rc


# ------------------------------------------------------------------------------- host-only calls
def schedule_plan(W, N, n_minibatches):
    n = _check(lib().tmps_schedule_plan(W, N, n_minibatches, None, 0))
    buf = (C.c_int32 * (7 * n))()
    _check(lib().tmps_schedule_plan(W, N, n_minibatches, buf, n))
    return np.frombuffer(buf, dtype=np.int32).reshape(n, 7).copy()


def schedule_plan_1f1b(W, n_batches):
    n = _check(lib().tmps_schedule_plan_1f1b(W, n_batches, None, 0))
    buf = (C.c_int32 * (7 * n))()
    _check(lib().tmps_schedule_plan_1f1b(W, n_batches, buf, n))
    return np.frombuffer(buf, dtype=np.int32).reshape(n, 7).copy()


def schedule_stash_groups(W, N, stage):
    return _check(lib().tmps_schedule_stash_groups(W, N, stage))


def schedule_shadow_versions(W, N, stage):
    return _check(lib().tmps_schedule_shadow_versions(W, N, stage))


def version_diff_formula(W, N):
    return _check(lib().tmps_version_diff_formula(W, N))


def version_diff_simulated(W, N):
    return _check(lib().tmps_version_diff_simulated(W, N))


KERNEL_CLASSES = ["dense_fwd", "dense_dgrad", "dense_wgrad", "conv_fwd", "conv_dgrad", "conv_wgrad", "softmax_ce",
                  "update", "pool_fwd", "pool_bwd", "relu_mask", "reduce", "copy", "event_pair", "splitk_finish", "slice_sum",
                  "layernorm", "attn_fwd", "attn_bwd", "embedding", "affine", "resadd"]


def profile_enable(on):
    _check(lib().tmps_profile_enable(int(bool(on))))


def profile_read():
    """{class name: (total milliseconds, launches)} since the last read."""
    n = len(KERNEL_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib().tmps_profile_read(ms, cnt, n))
    return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}


def layer_descs(specs):
    """Neutral layer dicts (workloads.configs) -> array of tmps_layer_desc."""
    arr = (LayerDesc * len(specs))()
    for d, sp in zip(arr, specs):
        k = sp["kind"]
        dims = [0] * 8
        if k == "linear":
            d.kind, dims[:4] = TMPS_LINEAR, [sp["din"], sp["dout"], sp.get("skip", 0), sp.get("rows", 1)]
            d.flags = TMPS_FLAG_RELU if sp["relu"] else (TMPS_FLAG_GELU if sp.get("act") == "gelu" else 0)
        elif k == "layernorm":
            if abs(sp["eps"] - 1e-5) > 1e-12:
                raise ValueError("the library's layer normalisation uses eps = 1e-5")
            d.kind, dims[:2] = TMPS_LAYERNORM, [sp["d"], sp["rows"]]
        elif k == "attention":
            d.kind, dims[:3] = TMPS_ATTENTION, [sp["s"], sp["d"], sp["heads"]]
        elif k == "embedding":
            d.kind, dims[:3] = TMPS_EMBEDDING, [sp["vocab"], sp["s"], sp["d"]]
        elif k == "conv":
            d.kind = TMPS_CONV2D
            dims[:8] = [sp["h"], sp["w"], sp["cin"], sp["cout"], sp["r"], sp["s"], sp["stride"], sp["pad"]]
            d.flags = (TMPS_FLAG_RELU if sp["relu"] else 0) | ((sp.get("src", 1) << 8) if sp.get("src", 1) > 1 else 0)
        elif k == "maxpool":
            d.kind, dims[:6] = TMPS_MAXPOOL, [sp["h"], sp["w"], sp["c"], sp["k"], sp["stride"], sp.get("pad", 0)]
        elif k == "affine":
            d.kind, dims[:3] = TMPS_AFFINE, [sp["h"], sp["w"], sp["c"]]
            d.flags = TMPS_FLAG_RELU if sp["relu"] else 0
        elif k == "resadd":
            d.kind, dims[:4] = TMPS_RESADD, [sp["h"], sp["w"], sp["c"], sp["src_b"]]
            d.flags = TMPS_FLAG_RELU if sp["relu"] else 0
        elif k == "avgpool":
            d.kind, dims[:3] = TMPS_AVGPOOL, [sp["h"], sp["w"], sp["c"]]
        elif k == "softmax_ce":
            d.kind, dims[:2] = TMPS_SOFTMAX_CE, [sp["classes"], sp.get("rows", 1)]
        else:
            raise ValueError("unknown layer kind %r" % k)
        for i, v in enumerate(dims):
            d.dims[i] = int(v)
    return arr


def stage_bytes(specs, cfg):
    out = [C.c_size_t() for _ in range(4)]
    descs = layer_descs(specs)
    _check(lib().tmps_stage_bytes(descs, len(specs), C.byref(cfg), *[C.byref(o) for o in out]))
    return tuple(o.value for o in out)


# ------------------------------------------------------------------------------------ device side
class Stage:
    """One pipeline worker on a GPU.  Owns the four device regions (torch tensors) the library works in."""

    def __init__(self, specs, dtype, micro_batch, n_micro, max_stash, lr, momentum, borrow_input=False,
                 device="cuda:0"):
        import torch
        self.torch = torch
        self.logical_specs = list(specs)
        # bf16 contractions fetch 8 channels per 16-byte load: a stage that starts with a convolution on
        # fewer channels (an RGB image) is handed channel-padded inputs and filters (zeros), which leaves
        # every result unchanged; set_params / get_* / prepare_input / crop_input_grad convert.
        self.cin, self.cin_pad = None, None
        specs = list(specs)
        if dtype == "bf16" and specs[0]["kind"] == "conv" and specs[0]["cin"] % 8 != 0:
            self.cin = specs[0]["cin"]
            self.cin_pad = (self.cin + 7) // 8 * 8
            specs[0] = dict(specs[0], cin=self.cin_pad)
        self.specs = specs
        self.device = torch.device(device)
        self.is_last = specs[-1]["kind"] == "softmax_ce"
        self.cfg = StageCfg(TMPS_BF16_F32MASTER if dtype == "bf16" else TMPS_F32, micro_batch, n_micro, max_stash,
                            int(self.is_last), int(borrow_input), lr, momentum)
        self.act_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.descs = layer_descs(specs)
        sizes = stage_bytes(specs, self.cfg)
        self.regions = [torch.zeros(max(s, 256), dtype=torch.uint8, device=self.device) for s in sizes]
        h = C.c_void_p()
        _check(lib().tmps_stage_create(C.byref(h), self.descs, len(specs), C.byref(self.cfg),
                                       *[C.c_void_p(r.data_ptr()) for r in self.regions]))
        self.handle = h
        self.P = lib().tmps_stage_param_count(h)
        self.in_elems = lib().tmps_stage_input_elems(h)
        self.out_elems = lib().tmps_stage_output_elems(h)
        self.micro, self.N = micro_batch, n_micro

    def __del__(self):
        if getattr(self, "handle", None) is not None and _lib is not None:
            _lib.tmps_stage_destroy(self.handle)
            self.handle = None

    # flat fp32 views into the device regions
    def _flat(self, region, index):
        t = self.regions[region][index * self.P * 4:(index + 1) * self.P * 4]
        return t.view(self.torch.float32)

    def param_offset(self, layer, which):
        off, cnt = C.c_int64(), C.c_int64()
        _check(lib().tmps_stage_param_offset(self.handle, layer, which, C.byref(off), C.byref(cnt)))
        return off.value, cnt.value

    def _get(self, flat):
        host = flat.cpu().numpy()
        out = []
        for li, sp in enumerate(self.specs):
            p = {}
            for which, key in ((0, "w"), (1, "b")):
                off, cnt = self.param_offset(li, which)
                if cnt:
                    p[key] = host[off:off + cnt].copy()
            if "w" in p:
                if sp["kind"] == "linear":
                    p["w"] = p["w"].reshape(sp["dout"], sp["din"])
                elif sp["kind"] == "conv":
                    p["w"] = p["w"].reshape(sp["cout"], sp["r"], sp["s"], sp["cin"])
                    if li == 0 and self.cin_pad:
                        p["w"] = np.ascontiguousarray(p["w"][..., :self.cin])
                elif sp["kind"] == "embedding":
                    p["w"] = p["w"].reshape(sp["vocab"], sp["d"])
                    p["b"] = p["b"].reshape(sp["s"], sp["d"])
            out.append(p)
        return out

    def set_params(self, params, stream=None):
        """Write fp32 master parameters (per layer dicts with 'w', 'b'), clear momentum, refresh the working copy."""
        torch = self.torch
        host = np.zeros(self.P, dtype=np.float32)
        for li, p in enumerate(params):
            for which, key in ((0, "w"), (1, "b")):
                off, cnt = self.param_offset(li, which)
                if cnt:
                    v = np.asarray(p[key], dtype=np.float32)
                    if li == 0 and key == "w" and self.cin_pad:
                        v = np.concatenate([v, np.zeros(v.shape[:-1] + (self.cin_pad - self.cin,), np.float32)], axis=-1)
                    host[off:off + cnt] = v.reshape(-1)
        self._flat(0, 0).copy_(torch.from_numpy(host))
        self.regions[1].zero_()
        torch.cuda.synchronize(self.device)
        _check(lib().tmps_stage_sync_params(self.handle, C.c_void_p(self._stream(stream))))
        torch.cuda.synchronize(self.device)

    def prepare_input(self, x):
        """Host array [rows, ...] -> device tensor in the layout and dtype the stage reads."""
        torch = self.torch
        if self.specs[0]["kind"] == "embedding":
            return torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.int32))).to(self.device)
        x = np.asarray(x, dtype=np.float32)
        if self.cin_pad:
            x = np.concatenate([x, np.zeros(x.shape[:-1] + (self.cin_pad - self.cin,), np.float32)], axis=-1)
        return torch.from_numpy(np.ascontiguousarray(x)).to(self.act_dtype).to(self.device)

    def crop_input_grad(self, dx, rows):
        """Device gradient w.r.t. the stage input -> host fp32 array with the logical channel count."""
        a = dx.float().cpu().numpy().reshape(rows, -1)
        if self.cin_pad:
            a = a.reshape(-1, self.cin_pad)[:, :self.cin].reshape(rows, -1)
        return a

    def get_params(self):
        return self._get(self._flat(0, 0))

    def get_grads(self):
        return self._get(self._flat(1, 1))

    def get_momentum(self):
        return self._get(self._flat(1, 0))

    def _stream(self, stream):
        if stream is None:
            return self.torch.cuda.current_stream(self.device).cuda_stream
        return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)

    def version(self):
        return lib().tmps_stage_version(self.handle)

    def set_shadow(self, n_versions):
        """Vertical weight stashing: keep the parameters of the last n_versions updates (a device region of its own)."""
        torch = self.torch
        one = self.regions[0].numel()
        self.shadow = torch.zeros(max(one * n_versions, 256), dtype=torch.uint8, device=self.device) if n_versions else None
        _check(lib().tmps_stage_set_shadow(self.handle, C.c_void_p(self.shadow.data_ptr()) if n_versions else None,
                                           one * n_versions, n_versions))

    def forward_micro_at(self, version, slot, x, y=None, labels=None, loss_out=None, stream=None):
        _check(lib().tmps_forward_micro_at(
            self.handle, version, slot, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()) if y is not None else None,
            C.c_void_p(labels.data_ptr()) if labels is not None else None,
            C.c_void_p(loss_out.data_ptr()) if loss_out is not None else None, C.c_void_p(self._stream(stream))))

    # ---- stage-wise checkpoints (section "Checkpointing") ----
    def save_checkpoint(self, directory, stage_index, epoch):
        """Write this stage's master parameters, momentum and version to its own file (no other stage is involved)."""
        from . import checkpoint
        self.torch.cuda.synchronize(self.device)
        return checkpoint.write_stage(directory, stage_index, epoch, self.version(), self._flat(0, 0).cpu().numpy(),
                                      self._flat(1, 0).cpu().numpy())

    def load_checkpoint(self, directory, stage_index, epoch, stream=None):
        from . import checkpoint
        torch = self.torch
        ck = checkpoint.read_stage(directory, stage_index, epoch)
        if ck["params"].size != self.P:
            raise checkpoint.CheckpointError("stage %d: %d parameters in the file, %d in the stage"
                                             % (stage_index, ck["params"].size, self.P))
        self._flat(0, 0).copy_(torch.from_numpy(ck["params"]))
        self._flat(1, 0).copy_(torch.from_numpy(ck["momentum"]))
        torch.cuda.synchronize(self.device)
        _check(lib().tmps_stage_sync_params(self.handle, C.c_void_p(self._stream(stream))))
        _check(lib().tmps_stage_set_version(self.handle, int(ck["version"])))
        torch.cuda.synchronize(self.device)

    def output_ptr(self, slot):
        return lib().tmps_stage_output_ptr(self.handle, slot)

    def forward_micro(self, slot, x, y=None, labels=None, loss_out=None, stream=None):
        _check(lib().tmps_forward_micro(
            self.handle, slot, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()) if y is not None else None,
            C.c_void_p(labels.data_ptr()) if labels is not None else None,
            C.c_void_p(loss_out.data_ptr()) if loss_out is not None else None, C.c_void_p(self._stream(stream))))

    def forward_micro_static(self, slot, x, y=None, labels=None, loss_out=None, stream=None):
        _check(lib().tmps_forward_micro_static(
            self.handle, slot, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()) if y is not None else None,
            C.c_void_p(labels.data_ptr()) if labels is not None else None,
            C.c_void_p(loss_out.data_ptr()) if loss_out is not None else None, C.c_void_p(self._stream(stream))))

    def backward(self, slots, dy=None, dx=None, stream=None):
        arr = (C.c_int * len(slots))(*slots)
        _check(lib().tmps_backward(self.handle, arr, len(slots),
                                   C.c_void_p(dy.data_ptr()) if dy is not None else None,
                                   C.c_void_p(dx.data_ptr()) if dx is not None else None,
                                   C.c_void_p(self._stream(stream))))

    def backward_at(self, version, slots, dy=None, dx=None, stream=None):
        arr = (C.c_int * len(slots))(*slots)
        _check(lib().tmps_backward_at(self.handle, version, arr, len(slots),
                                      C.c_void_p(dy.data_ptr()) if dy is not None else None,
                                      C.c_void_p(dx.data_ptr()) if dx is not None else None,
                                      C.c_void_p(self._stream(stream))))

    def update(self, stream=None):
        _check(lib().tmps_update(self.handle, C.c_void_p(self._stream(stream))))

    def use_graphs(self, on=True):
        """Forward and backward passes replay captured HIP graphs (see tmps_stage_use_graphs)."""
        _check(lib().tmps_stage_use_graphs(self.handle, 1 if on else 0))

    def device_bytes(self):
        """Bytes of the stage's device regions: parameters (masters + working copy), optimizer state and gradients,
        activation stash, scratch, kept weight versions."""
        names = ("params", "state", "stash", "scratch")
        out = {n: int(r.numel()) for n, r in zip(names, self.regions)}
        sh = getattr(self, "shadow", None)
        out["kept_versions"] = int(sh.numel()) if sh is not None else 0
        return out


class Pipeline:
    """K stages of a workloads.Config on K streams of one GPU, run in nF1B order by tmps_schedule_run."""

    def __init__(self, cfg, params, device="cuda:0", extra_groups=0, one_stream=False, vertical_sync=False,
                 baseline_1f1b=False, batch=None, graphs=False):
        """graphs: every stage replays captured HIP graphs of its passes (for configurations of many short kernels);
        the first stage then copies its input into its stash instead of borrowing the caller's array, whose
        addresses never repeat.
        vertical_sync: forward passes read the weight version they are tagged with (the paper's vertical weight
        stashing; every stage keeps the older versions the schedule needs) instead of the live weights.
        baseline_1f1b: the comparison system instead of TiMePReSt: batches of `batch` samples (default: the
        configuration's micro-batch size), each with its own forward and backward pass, in 1F1B order, backward passes
        on the weights of their forward passes (every stage keeps the K - s - 1 older versions that takes)."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.vertical_sync = bool(vertical_sync)
        self.baseline_1f1b = bool(baseline_1f1b)
        self.device = torch.device(device)
        K, N = cfg.K, cfg.N
        self.batch = int(batch) if batch else cfg.micro
        self.stages = []
        for s in range(K):
            if self.baseline_1f1b:
                st = Stage(cfg.stages[s], cfg.dtype, self.batch, 1, K - s + extra_groups, cfg.lr, cfg.momentum,
                           borrow_input=True, device=device)
                st.set_params(params[s])
                st.set_shadow(K - s - 1)
                self.stages.append(st)
                continue
            groups = schedule_stash_groups(K, N, s) + extra_groups
            st = Stage(cfg.stages[s], cfg.dtype, cfg.micro, N, groups * N, cfg.lr, cfg.momentum,
                       borrow_input=not (graphs and s == 0), device=device)
            st.set_params(params[s])
            if graphs:
                st.use_graphs(True)
            if self.vertical_sync:
                st.set_shadow(schedule_shadow_versions(K, N, s))
            self.stages.append(st)
        # K streams created back to back by the library, so that they land on distinct hardware queues (streams from
        # torch's pool may share one, and then two workers run one after the other); wrapped for torch.
        # one_stream: every worker issues on the same stream, so kernels never overlap (for per-kernel timing)
        n = 1 if one_stream else K
        self._raw_streams = (C.c_void_p * n)()
        with torch.cuda.device(self.device):
            _check(lib().tmps_streams_create(self._raw_streams, n))
        ext = [torch.cuda.ExternalStream(int(self._raw_streams[i]), device=self.device) for i in range(n)]
        self.streams = [ext[0] if one_stream else ext[s] for s in range(K)]
        self.act_dtype = self.stages[0].act_dtype

    def __del__(self):
        raw = getattr(self, "_raw_streams", None)
        if raw is not None and _lib is not None:
            try:
                self.torch.cuda.synchronize(self.device)
                _lib.tmps_streams_destroy(raw, len(raw))
            except Exception:
                pass
            self._raw_streams = None

    def upload(self, batches):
        """Concatenate mini-batches and place them in HBM (inputs in the activation dtype, labels int32)."""
        torch = self.torch
        x = self.stages[0].prepare_input(np.concatenate([b[0] for b in batches], axis=0))
        y = torch.from_numpy(np.concatenate([b[1] for b in batches], axis=0).astype(np.int32))
        return x.contiguous(), y.to(self.device).contiguous()

    def run_device(self, x_dev, y_dev, n_minibatches, losses_dev, want_log=True, one_stream=False):
        """Launch on resident inputs.  Returns the version log (n_tasks x 7 int32) or None.
        one_stream: this run issues every worker on the first stream (kernels never share the device)."""
        K, N = self.cfg.K, self.cfg.N
        handles = (C.c_void_p * K)(*[st.handle for st in self.stages])
        streams = (C.c_void_p * K)(*[(self.streams[0] if one_stream else s).cuda_stream for s in self.streams])
        log = None
        logp = None
        if want_log:
            if self.baseline_1f1b:
                n_tasks = _check(lib().tmps_schedule_plan_1f1b(K, n_minibatches, None, 0))
            else:
                n_tasks = _check(lib().tmps_schedule_plan(K, N, n_minibatches, None, 0))
            log = (C.c_int32 * (7 * n_tasks))()
            logp = log
        if self.baseline_1f1b:   # n_minibatches counts batches here
            _check(lib().tmps_schedule_run_1f1b(handles, K, n_minibatches, C.c_void_p(x_dev.data_ptr()),
                                                C.c_void_p(y_dev.data_ptr()), streams, C.c_void_p(losses_dev.data_ptr()), logp))
        else:
            run = lib().tmps_schedule_run_vsync if self.vertical_sync else lib().tmps_schedule_run
            _check(run(handles, K, N, n_minibatches, C.c_void_p(x_dev.data_ptr()), C.c_void_p(y_dev.data_ptr()), streams,
                       C.c_void_p(losses_dev.data_ptr()), logp))
        if log is None:
            return None
        return np.frombuffer(log, dtype=np.int32).reshape(-1, 7).copy()

    def run(self, batches):
        torch = self.torch
        x, y = self.upload(batches)
        losses = torch.zeros(len(batches), dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        log = self.run_device(x, y, len(batches), losses)
        torch.cuda.synchronize(self.device)
        return losses.cpu().numpy().tolist(), log

    def get_params(self, s):
        return self.stages[s].get_params()

    def save_checkpoint(self, directory, epoch):
        """Every stage writes its own file for `epoch` (call between runs: the pipeline is drained)."""
        return [st.save_checkpoint(directory, s, epoch) for s, st in enumerate(self.stages)]

    def resume(self, directory):
        """Load the latest epoch whose checkpoints of ALL stages are intact; returns that epoch, or None."""
        from . import checkpoint
        epoch = checkpoint.last_complete_epoch(directory, self.cfg.K)
        if epoch is None:
            return None
        for s, st in enumerate(self.stages):
            st.load_checkpoint(directory, s, epoch)
        return epoch

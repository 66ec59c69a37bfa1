"""One pipeline worker of the CPU oracle: consecutive layers, stash, backward, update.

Test infrastructure (CPU oracle).  Follows the Methodology section: a
micro-batch of M/N samples is the unit of the forward pass; once the N
micro-batches of a mini-batch have been forwarded, ONE backward pass is made
over the whole mini-batch on the gradient of the average micro-batch loss,
with the stage's weights as they are at that moment (no weight version is
kept from the forward pass); then the weights are updated in place
(update rule of TiMePReSt with SGD; momentum, which the paper leaves open, is
buf <- mu*buf + g, w <- w - lr*buf, buf_0 = 0).

precision="bf16" applies the storage policy of oracle/precision.py: the weights the layers read are
the bfloat16 rounding of the master weights, layer outputs and propagated gradients are rounded
when stored (the logits, which feed the loss directly, are not); weight gradients, momentum and
master weights stay unrounded.
"""
import numpy as np

from . import layers as L
from .precision import storage_rounding


class Stage:
    def __init__(self, layer_specs, params, lr, momentum, M, N, precision="f64"):
        if M % N != 0:
            raise ValueError("mini-batch size must be a multiple of the number of micro-batches")
        self.specs = layer_specs
        self.params = [{k: np.array(v, dtype=np.float64) for k, v in p.items()} for p in params]
        self.bufs = [{k: np.zeros_like(v) for k, v in p.items()} for p in self.params]
        self.grads = [None] * len(layer_specs)
        self.lr, self.mu, self.M, self.N = float(lr), float(momentum), M, N
        self.is_last = layer_specs[-1]["kind"] == "softmax_ce"
        self.stash = {}
        self.version = 0
        self.keep_versions = 0   # older weight versions kept for vertical weight stashing
        self.history = {}        # version -> parameters after that many updates
        self.q = storage_rounding(precision)

    # -- forward of one micro-batch -------------------------------------------------------
    def forward_micro(self, slot, x, labels=None, version=None):
        """Returns the stage output; on the last stage returns (logits, micro-batch mean loss).
        version: vertical weight stashing (Methodology, first paragraph; "GPU Memory Overhead"): run the layers on
        this stage's weights as they were after `version` updates (kept by keep_versions) instead of the live ones."""
        if slot in self.stash:
            raise RuntimeError("stash slot %r is in use" % (slot,))
        caches = []
        q = self.q
        a = x if self.specs[0]["kind"] == "embedding" else q(x)
        x_in = a
        loss = None
        inputs = []   # inputs[li] = what layer li read (a residual connection adds one of these)
        outs = []     # outs[li] = what layer li produced

        def earlier(li, k):
            """Result of the layer k positions before layer li; one before the first layer is the stage input."""
            return outs[li - k] if li - k >= 0 else x_in

        weights = self.params if version is None or version == self.version else self.history[version]
        for li, (spec, p) in enumerate(zip(self.specs, weights)):
            k = spec["kind"]
            if k == "conv" and spec.get("src", 1) != 1:
                a = earlier(li, spec["src"])
            inputs.append(a)
            feeds_loss = li + 1 < len(self.specs) and self.specs[li + 1]["kind"] == "softmax_ce"
            if k == "linear":
                skip = inputs[li - spec["skip"]] if spec.get("skip") else None
                a, c = L.linear_forward(a, q(p["w"]), p["b"], spec["relu"], spec.get("act"), spec.get("rows", 1),
                                        skip, round_z=q)
                if not feeds_loss:
                    a = c["y"] = q(a)
            elif k == "conv":
                a = a.reshape(a.shape[0], spec["h"], spec["w"], spec["cin"])
                a, c = L.conv_forward(a, q(p["w"]), p["b"], spec["stride"], spec["pad"], spec["relu"])
                a = c["y"] = q(a)
            elif k == "maxpool":
                a, c = L.maxpool_forward(a, spec["k"], spec["stride"], spec.get("pad", 0))
            elif k == "affine":
                a, c = L.affine_forward(a.reshape(a.shape[0], spec["h"], spec["w"], spec["c"]), p["w"], p["b"], spec["relu"])
                a = c["y"] = q(a)
            elif k == "resadd":
                a, c = L.resadd_forward(a, earlier(li, spec["src_b"]), spec["relu"])
                a = c["y"] = q(a)
            elif k == "avgpool":
                a, c = L.avgpool_forward(a.reshape(a.shape[0], spec["h"], spec["w"], spec["c"]))
                a = q(a)
            elif k == "layernorm":
                a, c = L.layernorm_forward(a, p["w"], p["b"], spec["d"], spec["eps"])
                a = q(a)
            elif k == "attention":
                a, c = L.attention_forward(a, spec["s"], spec["d"], spec["heads"])
                a = q(a)
            elif k == "embedding":
                a, c = L.embedding_forward(a, q(p["w"]), q(p["b"]))
                a = q(a)
            elif k == "softmax_ce":
                rows = spec.get("rows", 1)
                loss, c = L.softmax_ce_forward(a.reshape(a.shape[0] * rows, -1), np.asarray(labels).reshape(-1))
            else:
                raise ValueError(k)
            caches.append(c)
            outs.append(a)
        self.stash[slot] = caches
        return (a, loss) if self.is_last else a

    # -- one backward pass over the mini-batch --------------------------------------------
    def backward(self, slots, dy=None, version=None):
        """dy: gradient w.r.t. the stage output for all M samples (rows in slot order); None on
        the last stage.  Returns the gradient w.r.t. the stage input, same row order.  Consumes
        the slots.  Parameter gradients are summed over the micro-batches.
        version: None = differentiate at the weights as they are now (TiMePReSt).  A number = at this stage's
        weights as they were after that many updates, kept by keep_versions: horizontal weight stashing, the
        policy of the PipeDream baseline (related work, the update rule of PipeDream), where a backward pass
        reads the version its forward pass read."""
        if len(slots) != self.N:
            raise ValueError("a backward pass covers the N micro-batches of one mini-batch")
        weights = self.params if version is None or version == self.version else self.history[version]
        micro = self.M // self.N
        acc = [None] * len(self.specs)
        dxs = []
        for i, slot in enumerate(slots):
            caches = self.stash.pop(slot)
            q = self.q
            n_l = len(self.specs)
            # Gradients by the result they belong to: index li = result of layer li, -1 = the stage input.  A
            # result that several layers read (the start of a residual connection) collects one contribution
            # from each reader, in reverse layer order; under the bf16 policy the stored sum is rounded after
            # every contribution, as a stored tensor is.
            grad_of = {}

            def give(t, contribution):
                c2 = contribution.reshape(contribution.shape[0], -1)
                grad_of[t] = q(c2) if t not in grad_of else q(grad_of[t] + c2)

            if dy is not None:
                give(n_l - 1, dy[i * micro:(i + 1) * micro])
            held = {}   # layer index -> gradient of a residual connection that joins that layer's input
            for li in range(n_l - 1, -1, -1):
                spec, p, c = self.specs[li], weights[li], caches[li]
                k = spec["kind"]
                dw = db = None
                g = grad_of.pop(li, None)
                src = li - (spec.get("src", 1) if k == "conv" else 1)
                if k == "softmax_ce":
                    g = L.softmax_ce_backward(c, self.M * spec.get("rows", 1))
                elif k == "linear":
                    if spec.get("skip"):
                        held[li - spec["skip"]] = g
                    g, dw, db = L.linear_backward(g, c, q(p["w"]), spec["relu"], spec.get("act"))
                elif k == "conv":
                    g = g.reshape(c["y"].shape)
                    g, dw, db = L.conv_backward(g, c, q(p["w"]), spec["stride"], spec["pad"], spec["relu"])
                elif k == "maxpool":
                    g = L.maxpool_backward(g.reshape(c["win"].shape), c, spec["k"], spec["stride"], spec.get("pad", 0))
                elif k == "affine":
                    g, dw, db = L.affine_backward(g, c, p["w"], spec["relu"])
                elif k == "resadd":
                    g = L.resadd_backward(g, c, spec["relu"])
                    give(max(li - spec["src_b"], -1), g)
                elif k == "avgpool":
                    g = L.avgpool_backward(g, c)
                elif k == "layernorm":
                    g, dw, db = L.layernorm_backward(g, c, p["w"])
                elif k == "attention":
                    g = L.attention_backward(g, c)
                elif k == "embedding":
                    dw, db = L.embedding_backward(g, c, spec["vocab"], spec["d"])
                    g = None
                if li in held:
                    g = g.reshape(g.shape[0], -1) + held.pop(li).reshape(g.shape[0], -1)
                if g is not None:
                    give(max(src, -1), g)
                if dw is None:
                    continue
                if acc[li] is None:
                    acc[li] = {"w": dw, "b": db}
                else:
                    acc[li]["w"] = acc[li]["w"] + dw
                    acc[li]["b"] = acc[li]["b"] + db
            g = grad_of.pop(-1, None)
            dxs.append(g)
        self.grads = acc
        return None if dxs[0] is None else np.concatenate(dxs, axis=0)

    # -- in-place update -------------------------------------------------------------------
    def update(self):
        if self.keep_versions:
            # the superseded weights stay until no forward pass needs them ("GPU Memory Overhead")
            self.history[self.version] = [{k: v.copy() for k, v in p.items()} for p in self.params]
            for old in [v for v in self.history if v < self.version + 1 - self.keep_versions]:
                del self.history[old]
        for p, buf, g in zip(self.params, self.bufs, self.grads):
            if g is None:
                continue
            for k in p:
                buf[k] *= self.mu
                buf[k] += g[k]
                p[k] -= self.lr * buf[k]
        self.version += 1

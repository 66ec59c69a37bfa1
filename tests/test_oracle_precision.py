"""Pins of the oracle's bf16 storage policy: the rounding against a library conversion and exact
cases, and the policy as a whole against the unrounded oracle within the bf16 error bound."""
import numpy as np
import torch

from oracle import pipeline
from oracle.precision import round_to_bf16
from tests.util import rel_err, rel_l2
from workloads import get_config, init_params, make_batch


def test_rounding_matches_library_bfloat16():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, 1.0, -1.0, 3.0e38, 1e-38, np.inf, -np.inf])]).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = round_to_bf16(a)
    assert np.array_equal(got.astype(np.float32), want)


def test_rounding_exact_cases():
    # values with at most 8 significant bits are unchanged
    for v in (1.0, 1.5, 255.0, 0.00390625, -96.0, 1.0078125):
        assert round_to_bf16(np.array([v]))[0] == v
    # spacing at 1.0 is 2^-7; exact ties go to the even neighbour
    ulp = 2.0 ** -7
    assert round_to_bf16(np.array([1.0 + ulp / 2]))[0] == 1.0              # tie -> even (1.0)
    assert round_to_bf16(np.array([1.0 + 3 * ulp / 2]))[0] == 1.0 + 2 * ulp  # tie -> even
    assert round_to_bf16(np.array([1.0 + 0.51 * ulp]))[0] == 1.0 + ulp
    assert round_to_bf16(np.array([1.0 + 0.49 * ulp]))[0] == 1.0
    # relative error bound 2^-9 (half a unit in the last place, worst case at a power of two), idempotent
    rng = np.random.default_rng(1)
    x = rng.standard_normal(10000)
    r = round_to_bf16(x)
    assert np.max(np.abs(r - x) / np.abs(x)) <= 2.0 ** -8
    assert np.array_equal(round_to_bf16(r), r)


def test_bf16_policy_stays_within_the_bf16_error_bound_of_the_exact_oracle():
    cfg = get_config("mlp4x1024_bf16")
    params = init_params(cfg)
    batches = [make_batch(cfg, i) for i in range(2)]
    ta, tb = {}, {}
    a = pipeline.run(cfg, params, batches, trace=ta, precision="f64")
    b = pipeline.run(cfg, params, batches, trace=tb, precision="bf16")
    assert a["ops"] == b["ops"]
    for la, lb in zip(a["losses"], b["losses"]):
        assert abs(la - lb) < 2e-2 * abs(la)
    # first mini-batch, before any trajectory drift: forward activations carry the storage error
    # directly (2^-9 per rounding, a few roundings deep) ...
    for s in range(cfg.K):
        assert rel_err(tb[("F", 1, 0, s)], ta[("F", 1, 0, s)]) < 2e-2
        # ... while a weight gradient is a sum over the 256 samples of products with both signs: the
        # sum cancels to about 1/sqrt(256) of its terms' size and the rounding errors of the terms do
        # not, so its relative error is that much larger.  The direction is still the exact one.
        for ga, gb in zip(ta[("G", 1, -1, s)], tb[("G", 1, -1, s)]):
            if ga is not None:
                assert rel_l2(gb["w"], ga["w"]) < 0.15
                cos = np.sum(ga["w"] * gb["w"]) / (np.linalg.norm(ga["w"]) * np.linalg.norm(gb["w"]))
                assert cos > 0.99

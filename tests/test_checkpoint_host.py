"""Stage-wise checkpoint files and resume (section "Checkpointing"): host logic, no GPU.

* a stage's file round-trips its parameters, momentum and update counter exactly;
* a run resumes from the latest epoch for which ALL stages' files are intact: a stage that failed before or while
  writing its latest file (file missing, truncated, or corrupted) pulls the pipeline back to the last epoch every
  stage completed;
* the oracle pipeline resumed from the state at the end of an epoch continues exactly as the uninterrupted run of the
  same epochs does (the pipeline is drained at an epoch's end, so two runs of n mini-batches are the reference).
"""
import os

import numpy as np
import pytest

from oracle import pipeline
from paper_2410_14312_amd import checkpoint as ck
from workloads import get_config, init_params, make_batch


def _state(seed, n=1000):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)


def test_round_trip(tmp_path):
    p, m = _state(1)
    path = ck.write_stage(str(tmp_path), 2, 5, 17, p, m)
    assert os.path.basename(path) == "stage002_epoch000005.npz"
    got = ck.read_stage(str(tmp_path), 2, 5)
    assert got["version"] == 17 and np.array_equal(got["params"], p) and np.array_equal(got["momentum"], m)
    assert not any(n.endswith(".part") for n in os.listdir(tmp_path))


def test_resume_picks_the_last_epoch_complete_on_all_stages(tmp_path):
    d = str(tmp_path)
    assert ck.last_complete_epoch(d, 3) is None
    for epoch in (1, 2, 3):
        for s in range(3):
            if epoch == 3 and s == 1:
                continue            # stage 1 failed before it wrote epoch 3
            p, m = _state(10 * epoch + s)
            ck.write_stage(d, s, epoch, 4 * epoch, p, m)
    assert ck.epochs_on_disk(d, 0) == [1, 2, 3] and ck.epochs_on_disk(d, 1) == [1, 2]
    assert ck.last_complete_epoch(d, 3) == 2
    # ... and then stage 2's epoch-2 file turns out to be cut short: back to epoch 1
    path = ck.stage_file(d, 2, 2)
    data = open(path, "rb").read()
    open(path, "wb").write(data[:len(data) // 2])
    with pytest.raises(ck.CheckpointError):
        ck.read_stage(d, 2, 2)
    assert ck.last_complete_epoch(d, 3) == 1


def test_flipped_bytes_and_misplaced_files_are_rejected(tmp_path):
    d = str(tmp_path)
    p, m = _state(3)
    path = ck.write_stage(d, 0, 1, 9, p, m)
    data = bytearray(open(path, "rb").read())
    # npz members are stored uncompressed: flip one byte in the middle of the parameter array
    data[len(data) // 3] ^= 0x40
    open(path, "wb").write(bytes(data))
    with pytest.raises(ck.CheckpointError):
        ck.read_stage(d, 0, 1)
    assert ck.last_complete_epoch(d, 1) is None
    # a file renamed to another stage's or epoch's name is not accepted either
    good = ck.write_stage(d, 0, 2, 9, p, m)
    os.replace(good, ck.stage_file(d, 1, 2))
    with pytest.raises(ck.CheckpointError):
        ck.read_stage(d, 1, 2)


def test_oracle_resumed_run_equals_uninterrupted_run():
    cfg = get_config("tiny_mlp_f32")
    params = init_params(cfg)
    batches = [make_batch(cfg, i) for i in range(6)]
    first = pipeline.run(cfg, params, batches[:3])
    state_p = [[{k: v.copy() for k, v in p.items()} for p in st.params] for st in first["stages"]]
    state_m = [[{k: v.copy() for k, v in b.items()} for b in st.bufs] for st in first["stages"]]
    versions = [st.version for st in first["stages"]]
    assert versions == [3] * cfg.K
    # uninterrupted: the same Stage objects go on with the next epoch
    second = pipeline.run(cfg, state_p, batches[3:], momentum=state_m, versions=versions)
    # resumed from what a checkpoint holds: fp32 parameters and momentum, the update counters
    ck_p = [[{k: v.astype(np.float32) for k, v in p.items()} for p in st] for st in state_p]
    ck_m = [[{k: v.astype(np.float32) for k, v in b.items()} for b in st] for st in state_m]
    resumed = pipeline.run(cfg, ck_p, batches[3:], momentum=ck_m, versions=versions)
    assert [st.version for st in resumed["stages"]] == [6] * cfg.K
    assert np.allclose(resumed["losses"], second["losses"], rtol=1e-6)
    # momentum matters: dropping it changes the continuation
    cold = pipeline.run(cfg, ck_p, batches[3:], versions=versions)
    assert not np.allclose(cold["losses"][1:], second["losses"][1:], rtol=1e-6)

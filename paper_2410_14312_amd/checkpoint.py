"""Stage-wise checkpoint files (host side only; section "Checkpointing" of the paper).

Every stage writes its own file after the backward pass of an epoch's last mini-batch, without talking to any other
stage.  A run that ended abnormally resumes from the latest epoch for which the files of ALL stages are intact; a
stage whose latest file is missing or damaged (it failed while writing, or never got there) pulls the whole pipeline
back to the last epoch every stage completed.

The paper's update rule has no optimizer state; with momentum the buffer is part of a stage's state and is saved
beside the parameters, as is the stage's update counter.  A file is written under a temporary name and renamed, and
carries a CRC-32 of its arrays, so a truncated or partly written file is recognised and never loaded.
"""
import os
import re
import zipfile
import zlib

import numpy as np


class CheckpointError(RuntimeError):
    pass


def stage_file(directory, stage_index, epoch):
    return os.path.join(directory, "stage%03d_epoch%06d.npz" % (stage_index, epoch))


def _crc(params, momentum, version):
    c = zlib.crc32(np.ascontiguousarray(params, dtype=np.float32).tobytes())
    c = zlib.crc32(np.ascontiguousarray(momentum, dtype=np.float32).tobytes(), c)
    return zlib.crc32(np.int64(version).tobytes(), c) & 0xFFFFFFFF


def write_stage(directory, stage_index, epoch, version, params, momentum):
    """params, momentum: flat fp32 arrays of the stage's master parameters and momentum buffers."""
    os.makedirs(directory, exist_ok=True)
    params = np.ascontiguousarray(params, dtype=np.float32).ravel()
    momentum = np.ascontiguousarray(momentum, dtype=np.float32).ravel()
    if params.shape != momentum.shape:
        raise CheckpointError("parameters and momentum differ in size")
    path = stage_file(directory, stage_index, epoch)
    tmp = path + ".part"
    with open(tmp, "wb") as f:
        np.savez(f, params=params, momentum=momentum, version=np.int64(version), epoch=np.int64(epoch),
                 stage=np.int64(stage_index), crc=np.uint32(_crc(params, momentum, version)))
        f.flush()
        os.fsync(f.fileno())
    os.replace(tmp, path)
    return path


def read_stage(directory, stage_index, epoch):
    """The stage's state at the end of `epoch`; raises CheckpointError if the file is missing or damaged."""
    path = stage_file(directory, stage_index, epoch)
    try:
        with np.load(path, allow_pickle=False) as z:
            ck = {k: z[k] for k in ("params", "momentum", "version", "epoch", "stage", "crc")}
    except (OSError, ValueError, KeyError, EOFError, zipfile.BadZipFile, zlib.error) as e:
        raise CheckpointError("%s: %s" % (path, e)) from e
    if int(ck["epoch"]) != epoch or int(ck["stage"]) != stage_index:
        raise CheckpointError("%s holds stage %d, epoch %d" % (path, int(ck["stage"]), int(ck["epoch"])))
    if int(ck["crc"]) != _crc(ck["params"], ck["momentum"], int(ck["version"])):
        raise CheckpointError("%s: checksum mismatch" % path)
    return {"params": ck["params"], "momentum": ck["momentum"], "version": int(ck["version"])}


def epochs_on_disk(directory, stage_index):
    """Epochs for which a file of this stage exists (intact or not), ascending."""
    pat = re.compile(r"^stage%03d_epoch(\d{6})\.npz$" % stage_index)
    try:
        names = os.listdir(directory)
    except FileNotFoundError:
        return []
    return sorted(int(m.group(1)) for m in (pat.match(n) for n in names) if m)


def last_complete_epoch(directory, n_stages):
    """The latest epoch whose checkpoints of all n_stages stages can be read, or None."""
    common = None
    for s in range(n_stages):
        e = set(epochs_on_disk(directory, s))
        common = e if common is None else common & e
    for epoch in sorted(common or (), reverse=True):
        try:
            for s in range(n_stages):
                read_stage(directory, s, epoch)
        except CheckpointError:
            continue
        return epoch
    return None

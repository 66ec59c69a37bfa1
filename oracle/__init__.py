"""CPU oracle for the TiMePReSt stage-training path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy implementation of what the hot path computes,
written from the paper (arXiv 2410.14312) and independent of the HIP code: it
shares no kernels, headers, helpers or constants with it.  Only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import it; the
product path never does.

Modules
  schedule  nF1B time-point simulation, version bookkeeping, closed forms
            (sections "Work Scheduling" and "Multiple Sequence Problem").
  layers    forward/backward of each layer kind, written from the definitions.
  stage     one worker: forward per micro-batch, one backward per mini-batch
            with the weights as they are at that moment, in-place update
            (Methodology; the update rule for TiMePReSt).
  pipeline  K workers driven by the simulated schedule.

Pins (see tests/test_oracle_*.py): the schedule against every fact the paper
states about its figures; layers against finite differences and against
library autograd; the stage against full-batch evaluation and textbook SGD.
Training trajectories for K >= 2 have no printed values in the paper:
parity unpinned for those beyond the invariants above.
"""

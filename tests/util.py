"""Helpers shared by the GPU parity tests: workload assembly, progress notes, comparisons."""
from __future__ import annotations

import os
import time

import numpy as np

E = 0xFFFFFFFF
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def note(msg: str) -> None:
    """Progress line that survives pytest's capture: appended to a log file in the run's output folder."""
    d = os.path.join(ROOT, "gpurun_out")
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def progress_path() -> str:
    d = os.path.join(ROOT, "gpurun_out")
    os.makedirs(d, exist_ok=True)
    return os.path.join(d, "test_progress.log")


def assert_topk_matches(ids_gpu, scores_gpu, ids_ref, scores_ref, all_scores_ref=None, rtol=1e-5):
    """ids/scores [nq, k].  Scores within rtol; ids equal except where reference scores tie within 2*rtol."""
    ids_gpu = np.asarray(ids_gpu)
    ids_ref = np.asarray(ids_ref)
    pad = ids_ref == E
    assert (ids_gpu[pad] == E).all()
    assert np.isneginf(scores_gpu[pad]).all()
    ok = ~pad
    np.testing.assert_allclose(scores_gpu[ok], scores_ref[ok], rtol=rtol, atol=1e-7)
    diff = (ids_gpu != ids_ref) & ok
    for qi, r in zip(*np.nonzero(diff)):
        # a swap is only acceptable between (near-)equal reference scores
        s = scores_ref[qi, r]
        tol = 2 * rtol * max(1.0, abs(float(s)))
        j = np.nonzero(ids_ref[qi] == ids_gpu[qi, r])[0]
        if j.size:
            assert abs(float(scores_ref[qi, j[0]]) - float(s)) <= tol, (qi, r)
        else:
            # the id came from beyond the reference top-k: its score must tie with the k-th score
            assert abs(float(scores_gpu[qi, r]) - float(scores_ref[qi, -1])) <= tol, (qi, r)


def recall_at_k(ids, gt) -> float:
    ids = np.asarray(ids)
    hits = 0
    for a, b in zip(ids, gt):
        hits += len(set(a.tolist()) & set(b.tolist()))
    return hits / gt.size

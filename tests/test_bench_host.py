"""Host logic of bench.py that needs no GPU: the flagged / mismatched row accounting against the oracle, and the
refusal of more than one GPU."""
import os
import subprocess
import sys

import numpy as np

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _rows():
    rng = np.random.default_rng(11)
    probs = rng.random((6, 300)).astype(np.float32) ** 4
    probs[2] = 0.25                                   # uniform row: every prefix mass sits on a boundary somewhere
    probs[2, :4] = [0.4, 0.2, 0.2, 0.2]
    return probs


def test_compare_lists_counts_flagged_and_mismatched_rows_separately():
    probs = _rows()
    ref = oracle.topp_select(probs, 0.9)
    idx = np.array(ref.indices, copy=True)
    cnt = np.array(ref.counts, copy=True)
    tau = np.array(ref.tau, copy=True)
    flagged = int(((ref.flags & oracle.ROW_NEAR_BOUNDARY) != 0).sum())
    assert bench.compare_lists(ref, idx, cnt, tau) == (flagged, 0, 0)
    clear = [r for r in range(probs.shape[0]) if not ref.flags[r] & oracle.ROW_NEAR_BOUNDARY]
    assert len(clear) >= 3
    # a wrong count, a wrong threshold and a wrong list entry on three unflagged rows
    cnt[clear[0]] += 1
    tau[clear[1]] = np.nextafter(tau[clear[1]], np.float32(1.0))
    idx[clear[2], 0] += 1
    assert bench.compare_lists(ref, idx, cnt, tau) == (flagged, 0, 3)
    # entries past a row's count are not part of its list
    idx2 = np.array(ref.indices, copy=True)
    idx2[clear[0], int(ref.counts[clear[0]]):] = -5
    assert bench.compare_lists(ref, idx2, ref.counts, ref.tau) == (flagged, 0, 0)


def test_compare_lists_reports_mismatches_on_flagged_rows_as_such():
    probs = np.array([[0.4, 0.2, 0.2, 0.2], [0.2, 0.4, 0.2, 0.2]], dtype=np.float32)   # 0.4 of the sum sits on the target
    ref = oracle.topp_select(probs, 0.4)
    assert (ref.flags & oracle.ROW_NEAR_BOUNDARY).all()
    cnt = np.array(ref.counts, copy=True)
    cnt[1] -= 1
    assert bench.compare_lists(ref, ref.indices, cnt, ref.tau) == (2, 1, 0)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "ONE GPU" in (p.stderr + p.stdout)

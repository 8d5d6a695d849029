"""The library's integer mask / index code (csrc/mask_index.h: row limits, first seeing query, tile classes, the
simulation band) compiled for the HOST with AddressSanitizer and UndefinedBehaviorSanitizer and swept over window
sizes, offsets, ragged shapes, tile sizes, simulation steps and sizes near the top of the accepted int32 range.
Any signed overflow, bad shift or out-of-range access aborts the driver; its printed values are compared with the
masks the oracle builds element by element from the paper's prose.  CPU only."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import beagle_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))
INT32_MAX = 2 ** 31 - 1


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path_factory.mktemp("san") / "mask_index_driver")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           os.path.join(HERE, "mask_index_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def _run(exe, lines):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)       # the sanitizer runtime must come first in the driver's own process
    r = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, "sanitizer or driver failure:\n" + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout.splitlines()


def test_grids_match_the_prose_built_masks(driver):
    cases = []
    for k in (1, 2, 3, 4, 5, 8, 16, 40):                        # 40 > S for the small shapes: k larger than the sequence
        for eps in sorted(e for e in {0, 1, k // 2, k - 1} if 0 <= e < k):
            for S, L in ((1, 1), (7, 7), (33, 33), (64, 20), (20, 64), (130, 130)):
                for tq, tk in ((128, 64), (32, 16), (48, 20), (1, 1) if S * L <= 64 else (7, 5)):
                    for t in (0, 1, k - 1, k, k + 3):
                        cases.append((S, L, k, eps, tq, tk, t))
    out = _run(driver, ["G %d %d %d %d %d %d %d" % c for c in cases])
    assert len(out) == 5 * len(cases)
    masks = {}
    for i, (S, L, k, eps, tq, tk, t) in enumerate(cases):
        head, lim, fq, cls, band = out[5 * i:5 * i + 5]
        assert head == "G %d %d %d %d %d %d %d" % (S, L, k, eps, tq, tk, t)
        key = (S, L, k, eps)
        if key not in masks:
            masks[key] = orc.dense_mask_loops(S, L, k, eps)
        m = masks[key]
        lim = np.array(lim.split()[1:], int)
        assert np.array_equal(lim, m.sum(1)), (key, "row limits")
        assert all(m[p, :lim[p]].all() and not m[p, lim[p]:].any() for p in range(S))
        fq = np.array(fq.split()[1:], int)
        for j in range(L):
            seen = np.flatnonzero(m[:, j])
            if len(seen):
                assert fq[j] == seen[0] and m[seen[0]:, j].all(), (key, j)
            else:
                assert fq[j] >= S, (key, j)
        cls = np.array(cls.split()[1:], int).reshape(-(-S // tq), -(-L // tk))
        for a in range(cls.shape[0]):
            for c in range(cls.shape[1]):
                blk = m[a * tq:(a + 1) * tq, c * tk:(c + 1) * tk]
                assert cls[a, c] == (0 if not blk.any() else (2 if blk.all() else 1)), (key, tq, tk, a, c)
        band = np.array(band.split()[1:], int).reshape(S, 2)
        pm = orc.sim_pred_mask_loops(S, L, k, eps, t)
        for p in range(S):
            want = np.zeros(L, bool)
            lo, hi = band[p]
            if hi > lo:
                assert 0 <= lo and hi <= L
                want[lo:hi] = True
            assert np.array_equal(pm[p], want), (key, t, p)


def test_positions_near_the_top_of_the_accepted_range(driver):
    """Sequence lengths up to 2^30 (the descriptor check's limit on B*S, B*L), every window size and offset, and any
    non-negative simulation step up to INT32_MAX: no overflow, and the values agree with the prose rule evaluated
    in Python integers (the window holding p starts at eps + k*floor((p - eps)/k); its queries see the keys
    before that start; step t shows the first t positions of the own window that lie before the query)."""
    top = 2 ** 30
    cases = []
    for L in (top, top - 1, 12345):
        for k in (1, 2, 5, 8, 4096, top - 1, top):
            for eps in sorted(e for e in {0, 1, k // 2, k - 1} if 0 <= e < k):
                for p in sorted(q for q in {0, 1, k - 1, k, L // 2, L - 2, L - 1} if 0 <= q < L):
                    for j in (0, L // 3, L - 1):
                        for t in (0, 1, k - 1, k, INT32_MAX):
                            cases.append((p, j, k, eps, L, t))
    out = _run(driver, ["P %d %d %d %d %d %d" % c for c in cases])
    assert len(out) == len(cases)
    for (p, j, k, eps, L, t), line in zip(cases, out):
        lim, fq, ws, wraw, lo, hi = (int(v) for v in line.split()[1:])
        w0 = eps + k * ((p - eps) // k)                          # Python floors toward minus infinity
        assert wraw == w0 and ws == max(w0, 0) and lim == min(max(w0, 0), L), (p, k, eps, L)
        wj = eps + k * ((j - eps) // k)                          # key j's window: the next window's queries see it
        assert fq == wj + k, (j, k, eps)
        band = range(max(w0, 0), min(p, w0 + t, L))
        assert (hi > lo and (lo, hi) == (band.start, band.stop)) or (hi <= lo and len(band) == 0), (p, k, eps, t, lo, hi)

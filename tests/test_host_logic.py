"""Host-side logic of the library that needs no GPU: the rule that cuts examined rows into pieces
(jot_plan_split in csrc/jot_device.h, evaluated identically by the host layout code and by every
kernel of a step).  The header is compiled into a small host program with hipcc and run here."""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def plan(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path_factory.mktemp("plan") / "plan_split_probe")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-o", exe, os.path.join(ROOT, "tests", "plan_split_probe.hip")],
                   check=True, capture_output=True)

    def run(cases):
        text = "".join(f"{n} {V} {t} {a}\n" for n, V, t, a in cases)
        out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True).stdout.split()
        vals = np.array(out, dtype=np.int64).reshape(-1, 2)
        assert len(vals) == len(cases)
        return vals
    return run


# (workgroups of the grid = items a step aims for, elements per batch) of the two element types
SHAPES = [(1024, 4096), (256, 32768), (1280, 4096), (256, 8192)]
VOCABS = [2, 17, 4095, 4096, 4097, 32768, 126464, 152064, 300007, 3000001]


def test_pieces_cover_the_row_once_and_never_outnumber_the_workgroups(plan):
    rng = np.random.default_rng(5)
    cases = []
    for target, align in SHAPES:
        for V in VOCABS:
            ns = {0, 1, 2, 3, target // 2 - 1, target // 2, target // 2 + 1, target - 1, target, target + 1, 3 * target}
            ns |= {int(x) for x in rng.integers(1, 2 * target, 12)}
            cases += [(n, V, target, align) for n in sorted(ns)]
    got = plan(cases)
    for (n, V, target, align), (S, chunk) in zip(cases, got):
        where = f"n={n} V={V} target={target} align={align} -> S={S} chunk={chunk}"
        assert S >= 1, where
        if S == 1:
            assert chunk == V, where
            continue
        # pieces: whole batches, the last one possibly shorter but not empty, together exactly the row
        assert chunk % align == 0 and chunk >= align, where
        assert (S - 1) * chunk < V <= S * chunk, where
        # one round of the grid: never more work items than workgroups
        assert 0 < n * S <= target, where
        # and no piece more than the row allows
        assert S <= V // align, where


def test_rows_are_left_whole_when_there_are_enough_of_them_or_they_are_short(plan):
    got = plan([(1024, 152064, 1024, 4096), (5000, 152064, 1024, 4096), (513, 152064, 1024, 4096),
                (10, 4095, 1024, 4096), (10, 8191, 1024, 4096), (0, 152064, 1024, 4096)])
    assert [int(S) for S, _ in got] == [1, 1, 1, 1, 1, 1]


def test_as_many_pieces_as_fit(plan):
    # 256 rows on 1024 workgroups: four pieces each; 242 rows: still four (five would need 1210 items)
    got = plan([(256, 126464, 1024, 4096), (242, 126464, 1024, 4096), (512, 126464, 1024, 4096), (1, 152064, 1024, 4096)])
    assert [int(S) for S, _ in got] == [4, 4, 2, 19]          # a single row: 37 batches of 4096 -> 19 pieces of two batches
    assert int(got[3][1]) == 8192

"""Layout heuristic and plan (Section IV.A, IV.D): the oracle against what the
paper reports, then the library (host code, no GPU needed) against the oracle."""
import os

import numpy as np
import pytest

import oracle
import paper_1610_03618_amd as cm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
NCHW, CHWN = 0, 1
CONV, POOL, OTHER = 0, 1, 2


def _conv_rows():
    with open(os.path.join(GOLDEN, "table1_conv_layouts.txt")) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_oracle_heuristic_reproduces_the_papers_choices_for_table1():
    for name, n, ci, want in _conv_rows():
        got = oracle.choose_layout(CONV, int(n), int(ci), 32, 128)
        assert got == (CHWN if want == "CHWN" else NCHW), name


def test_oracle_heuristic_thresholds_are_strict_and_inclusive_as_stated():
    # "C smaller than Ct" -> CHWN; "N greater than or equal to Nt" -> CHWN
    assert oracle.choose_layout(CONV, 64, 31, 32, 128) == CHWN
    assert oracle.choose_layout(CONV, 64, 32, 32, 128) == NCHW
    assert oracle.choose_layout(CONV, 127, 64, 32, 128) == NCHW
    assert oracle.choose_layout(CONV, 128, 64, 32, 128) == CHWN
    # second GPU of the paper: (128, 64)
    assert oracle.choose_layout(CONV, 64, 256, 128, 64) == CHWN
    assert oracle.choose_layout(CONV, 32, 128, 128, 64) == NCHW
    assert oracle.choose_layout(POOL, 32, 512, 32, 128) == CHWN     # Section IV.B: always CHWN
    assert oracle.choose_layout(OTHER, 32, 512, 32, 128) == -1


def test_oracle_plan_hand_worked():
    # conv(C=3) pool conv(C=96, N=64) pool conv(C=256) other, thresholds (32, 128), input NCHW
    layers = [(CONV, 64, 3), (POOL, 64, 96), (CONV, 64, 96), (POOL, 64, 256), (CONV, 64, 256), (OTHER, 64, 256)]
    layouts, tb, n = oracle.plan_layouts(layers, 32, 128, NCHW)
    assert layouts == [CHWN, CHWN, NCHW, CHWN, NCHW, NCHW]
    assert tb == [1, 0, 1, 1, 1, 0] and n == 4
    # pooling that keeps its input layout saves the two transforms around the second pool
    layouts, tb, n = oracle.plan_layouts(layers, 32, 128, NCHW, pool_keeps_layout=True)
    assert layouts == [CHWN, CHWN, NCHW, NCHW, NCHW, NCHW]
    assert tb == [1, 0, 1, 0, 0, 0] and n == 2
    # input already in CHWN: no transform in front of the first layer
    layouts, tb, n = oracle.plan_layouts(layers[:2], 32, 128, CHWN)
    assert tb == [0, 0] and n == 0


def test_library_heuristic_matches_oracle():
    for name, n, ci, _ in _conv_rows():
        for ct, nt in [(32, 128), (128, 64), (0, 10**6), (10**6, 0)]:
            st, got = cm.cnnmem_choose_layout(CONV, int(n), int(ci), ct, nt)
            assert st == 0 and got == oracle.choose_layout(CONV, int(n), int(ci), ct, nt), (name, ct, nt)
    assert cm.cnnmem_choose_layout(POOL, 8, 8, 32, 128) == (0, CHWN)
    assert cm.cnnmem_choose_layout(OTHER, 8, 8, 32, 128, default=NCHW) == (0, NCHW)
    assert cm.cnnmem_choose_layout(OTHER, 8, 8, 32, 128, default=CHWN) == (0, CHWN)
    assert cm.cnnmem_choose_layout(7, 8, 8, 32, 128)[0] == 1
    assert cm.cnnmem_choose_layout(CONV, 0, 8, 32, 128)[0] == 1
    assert cm.cnnmem_choose_layout(CONV, 8, 8, -1, 128)[0] == 1
    assert cm.library().cnnmem_choose_layout(CONV, 8, 8, 32, 128, None) == 1


def test_library_plan_matches_oracle_on_random_networks():
    rng = np.random.default_rng(3)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        layers = [(int(rng.integers(0, 3)), int(rng.choice([16, 32, 64, 128, 256])),
                   int(rng.choice([1, 3, 16, 31, 32, 64, 96, 256]))) for _ in range(n)]
        ct, nt = int(rng.choice([16, 32, 128])), int(rng.choice([64, 128]))
        inp = int(rng.integers(0, 2))
        for policy, keeps in ((cm.POOL_PREFERS_CHWN, False), (cm.POOL_KEEPS_LAYOUT, True)):
            st, layouts, tb, cnt = cm.cnnmem_plan_layouts(layers, ct, nt, inp, policy)
            want = oracle.plan_layouts(layers, ct, nt, inp, keeps)
            assert st == 0 and (layouts, tb, cnt) == want


def test_library_plan_rejects_bad_input():
    ok = [(CONV, 64, 3), (POOL, 64, 96)]
    assert cm.cnnmem_plan_layouts(ok, 32, 128, 2)[0] == 1                  # bad input layout
    assert cm.cnnmem_plan_layouts(ok, 32, 128, NCHW, 5)[0] == 1            # bad policy
    assert cm.cnnmem_plan_layouts([(9, 64, 3)], 32, 128, NCHW)[0] == 1     # bad kind
    assert cm.cnnmem_plan_layouts([(CONV, 64, 0)], 32, 128, NCHW)[0] == 1  # bad C
    assert cm.cnnmem_plan_layouts([], 32, 128, NCHW)[0] == 1               # empty network

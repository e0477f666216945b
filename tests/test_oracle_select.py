"""Pins for the oracle's selection / commit rule (CPU only, integer-exact)."""
import itertools

import numpy as np
import pytest

from oracle.denoise import select_commit, apply_commit
from brute_force import select_brute


def test_planted_confidences_threshold():
    conf = np.array([[0.95, 0.85, 0.99, 0.10, 0.91, 0.5]])
    mask = np.array([[1, 1, 0, 1, 1, 1]], np.uint8)               # position 2 already committed
    c, n, rem = select_commit(conf, mask, rule="threshold", tau=0.9)
    assert c.tolist() == [[1, 0, 0, 0, 1, 0]] and n.tolist() == [2] and rem.tolist() == [3]
    # nothing reaches tau: only the most confident masked one commits
    c, n, rem = select_commit(conf, mask, rule="threshold", tau=0.999)
    assert c.tolist() == [[1, 0, 0, 0, 0, 0]] and n.tolist() == [1] and rem.tolist() == [4]
    # >= not >
    c, _, _ = select_commit(conf, mask, rule="threshold", tau=0.85)
    assert c.tolist() == [[1, 1, 0, 0, 1, 0]]
    # tau <= 0 commits everything masked at once; unmasked never commit
    c, n, rem = select_commit(conf, mask, rule="threshold", tau=0.0)
    assert c.tolist() == [[1, 1, 0, 1, 1, 1]] and rem.tolist() == [0]
    # without the forced pick nothing may commit
    c, n, _ = select_commit(conf, mask, rule="threshold", tau=0.999, force_top1=False)
    assert n.tolist() == [0]


def test_ties_go_to_lowest_index():
    conf = np.full((1, 6), 0.3)
    mask = np.array([[0, 1, 1, 1, 1, 1]], np.uint8)
    c, _, _ = select_commit(conf, mask, rule="threshold", tau=0.9)
    assert c.tolist() == [[0, 1, 0, 0, 0, 0]]
    c, _, _ = select_commit(conf, mask, rule="topk", k=3)
    assert c.tolist() == [[0, 1, 1, 1, 0, 0]]


def test_topk_planted_and_short_groups():
    conf = np.array([[0.2, 0.9, 0.4, 0.8, 0.1, 0.7, 0.6, 0.3]])
    mask = np.array([[1, 1, 1, 0, 1, 1, 1, 1]], np.uint8)
    c, n, rem = select_commit(conf, mask, rule="topk", k=2)
    assert c.tolist() == [[0, 1, 0, 0, 0, 1, 0, 0]] and n.tolist() == [2] and rem.tolist() == [5]
    c, n, rem = select_commit(conf, mask, rule="topk", k=50)
    assert np.array_equal(c, mask) and rem.tolist() == [0]
    # groups of 4: rule applied per group, counts summed per sequence
    c, n, rem = select_commit(conf, mask, rule="topk", k=1, group_len=4)
    assert c.tolist() == [[0, 1, 0, 0, 0, 1, 0, 0]] and n.tolist() == [2] and rem.tolist() == [5]
    c, n, rem = select_commit(conf, np.array([[0, 0, 0, 0, 1, 1, 0, 0]], np.uint8), rule="threshold",
                              tau=0.95, group_len=4)
    assert c.tolist() == [[0, 0, 0, 0, 0, 1, 0, 0]] and n.tolist() == [1] and rem.tolist() == [1]


@pytest.mark.parametrize("rule", ["threshold", "topk"])
def test_against_set_definition_randomised(rule):
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(1, 10))
        conf = np.round(rng.random((2, n)), 1)                    # coarse grid -> many ties
        mask = (rng.random((2, n)) < 0.6).astype(np.uint8)
        tau, k = float(rng.choice([0.0, 0.3, 0.5, 0.9, 1.5])), int(rng.integers(1, 5))
        c, ncom, rem = select_commit(conf, mask, rule=rule, tau=tau, k=k)
        for b in range(2):
            want = select_brute(conf[b].tolist(), mask[b].tolist(), rule, tau, k)
            assert set(np.flatnonzero(c[b]).tolist()) == want
            assert ncom[b] == len(want) and rem[b] == int(mask[b].sum()) - len(want)


def test_step_counts_closed_forms():
    rng = np.random.default_rng(9)
    # fixed schedule: ceil(m / k) steps; tau > 1: one commit per step in descending confidence
    for m, k in [(32, 2), (32, 4), (16, 4), (7, 3)]:
        mask = np.zeros((1, 32), np.uint8)
        mask[0, rng.permutation(32)[:m]] = 1
        steps = 0
        while mask.any():
            conf = rng.random((1, 32))
            c, _, _ = select_commit(conf, mask, rule="topk", k=k)
            mask = mask & ~c
            steps += 1
        assert steps == -(-m // k)
    conf = rng.random((1, 32))
    mask = np.ones((1, 32), np.uint8)
    order = []
    while mask.any():
        c, n, _ = select_commit(conf, mask, rule="threshold", tau=1.5)
        assert n[0] == 1
        order.append(int(np.flatnonzero(c[0])[0]))
        mask = mask & ~c
    assert order == sorted(range(32), key=lambda i: (-conf[0, i], i))


def test_apply_commit_touches_only_committed():
    x = np.arange(20, dtype=np.int32).reshape(2, 10)
    mask = np.array([[1, 0, 1, 1], [0, 0, 1, 0]], np.uint8)
    tok = np.array([[100, 101, 102, 103], [200, 201, 202, 203]], np.int32)
    commit = np.array([[1, 0, 0, 1], [0, 0, 1, 0]], np.uint8)
    x0 = x.copy()
    apply_commit(x, 3, mask, tok, commit)
    assert x[0, 3] == 100 and x[0, 6] == 103 and x[1, 5] == 202
    changed = (x != x0)
    assert changed.sum() == 3
    assert mask.tolist() == [[0, 0, 1, 0], [0, 0, 0, 0]]


def test_golden_schedule_from_paper():
    """Section 4.1: response 512 with 256 diffusion steps and response 256 with 128 steps, block 32."""
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "schedule_sec4_1.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(t) for t in line.split()])
    assert rows
    rng = np.random.default_rng(1)
    for resp, steps, blk, k, steps_per_block in rows:
        assert resp // steps == k and blk // k == steps_per_block
        mask = np.ones((3, blk), np.uint8)
        count = 0
        while mask.any():
            c, n, _ = select_commit(rng.random((3, blk)), mask, rule="topk", k=k)
            assert np.all(n == k)
            mask = mask & ~c
            count += 1
        assert count == steps_per_block

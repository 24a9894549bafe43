"""Pins for the contract checker of the oracle (CPU only): every flag is raised by a hand-made violation and by nothing else."""
import numpy as np

import oracle
import ygg_workloads as wl

PARENT, SEQ, DEPTH, TOKEN, LOGIT = 1, 2, 4, 8, 16


def _good(B=3, D=3, W=4, V=50):
    N = 1 + D * W
    parent = np.stack([wl.level_tree(5, D, W, "dirichlet", 0.5, sub=b) for b in range(B)]).astype(np.int32)
    token = np.stack([np.arange(N) % V for _ in range(B)]).astype(np.int32)
    lens = np.array([0, 7, 16], np.int32)[:B]
    logits = np.zeros((B, 2, V), np.float32)
    return parent, lens, token, logits, D, V


def test_valid_inputs_raise_nothing():
    parent, lens, token, logits, D, V = _good()
    assert np.all(parent[:, 0] == -1)
    f = oracle.validate(D, V, 16, parent, lens, token, logits)
    assert list(f) == [0, 0, 0]
    assert list(oracle.validate(D, V, 16, parent_idx=parent)) == [0, 0, 0]


def test_each_violation_sets_its_own_bit_in_its_own_sequence():
    parent, lens, token, logits, D, V = _good()
    p = parent.copy(); p[1, 5] = 5                       # a node that is its own parent
    assert list(oracle.validate(D, V, 16, p, lens, token, logits)) == [0, PARENT, 0]
    p = parent.copy(); p[2, 0] = 0                       # the root must carry -1
    assert list(oracle.validate(D, V, 16, p, lens, token, logits)) == [0, 0, PARENT]
    p = parent.copy(); p[0, 3] = 7                       # a parent that comes later
    assert list(oracle.validate(D, V, 16, p, lens, token, logits)) == [PARENT, 0, 0]
    l = lens.copy(); l[0] = -1; l[2] = 17
    assert list(oracle.validate(D, V, 16, parent, l, token, logits)) == [SEQ, 0, SEQ]
    t = token.copy(); t[1, 2] = V; t[2, 9] = -3
    assert list(oracle.validate(D, V, 16, parent, lens, t, logits)) == [0, TOKEN, TOKEN]
    x = logits.copy(); x[0, 1, V - 1] = np.nan; x[1, 0, 0] = np.inf    # an infinity is not a violation
    assert list(oracle.validate(D, V, 16, parent, lens, token, x)) == [LOGIT, 0, 0]


def test_depth_bound_and_combined_flags():
    N = 9
    chain = wl.chain_tree(N).astype(np.int32)[None]
    assert list(oracle.validate(8, 10, 4, chain)) == [0]
    assert list(oracle.validate(7, 10, 4, chain)) == [DEPTH]
    star = np.array([[-1] + [0] * (N - 1)], np.int32)
    assert list(oracle.validate(1, 10, 4, star)) == [0]
    bad = chain.copy(); bad[0, 4] = 6                     # invalid parents: the depth is not judged
    lens = np.array([9], np.int32)
    token = np.full((1, N), 10, np.int32)
    assert list(oracle.validate(2, 10, 4, bad, lens, token)) == [PARENT | SEQ | TOKEN]

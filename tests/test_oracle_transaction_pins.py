"""Pins of the oracle's transaction key (oracle/transaction.c; Sec. 4.1 of the paper: a function is bound to a
hashing key generated from its fetches and feeds).  The paper names no hash, so there is no value of the paper's
to compare with; what is pinned is (a) the mixing step against the published outputs of SplitMix64, (b) the
properties a key must have, by brute force over small inputs."""
import itertools

import numpy as np

import oracle

G = 0x9E3779B97F4A7C15
MASK = 2**64 - 1


def test_mixing_step_is_the_output_function_of_splitmix64():
    # SplitMix64 seeded with 0 (state += G, output = mix(state)): first outputs of the public-domain reference
    # implementation, as quoted wherever it seeds other generators
    expected = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    state, got = 0, []
    for _ in expected:
        state = (state + G) & MASK
        got.append(oracle.mix64(state))
    assert got == expected
    assert oracle.mix64(0) == 0                              # its one fixed point


def _digest(sets, Q=None):
    Q = len(sets) if Q is None else Q
    rowptr = np.concatenate([[0], np.cumsum([len(s) for s in sets])]).astype(np.int32)
    idx = np.asarray([t for s in sets for t in s], dtype=np.int32)
    return oracle.target_digest(Q, rowptr, idx)


def test_equal_target_sets_have_equal_keys_and_any_change_shows():
    base = [[3, 9, 4], [], [7], [1, 1]]
    d = _digest(base)
    assert d == _digest([list(s) for s in base])
    changed = [
        [[3, 9, 5], [], [7], [1, 1]],        # one id
        [[9, 3, 4], [], [7], [1, 1]],        # order inside a set (the prune would colour the same, the key is of the
                                             # sets as given: a cache may miss, it must never hit wrongly)
        [[3, 9], [4], [7], [1, 1]],          # a target moved to the next set: same idx, other row pointers
        [[3, 9, 4], [7], [], [1, 1]],        # the empty set elsewhere
        [[3, 9, 4], [], [7], [1]],           # a duplicate dropped
        [[3, 9, 4], [], [7], [1, 1], []],    # one more (empty) set
    ]
    keys = {d} | {_digest(c) for c in changed}
    assert len(keys) == 1 + len(changed)
    assert _digest(base, Q=2) != d                          # same arrays, two graphs of two sets each


def test_no_collisions_over_all_small_inputs():
    """Every way of giving up to three targets out of four tensors to two sets: all keys distinct, in both
    halves on their own (a dropped term, a position that is not keyed or a half that ignores the value would
    collide here)."""
    seen0, seen1, n = set(), set(), 0
    for m in range(4):
        for idx in itertools.product(range(4), repeat=m):
            for cut in range(m + 1):
                d0, d1 = _digest([list(idx[:cut]), list(idx[cut:])])
                seen0.add(d0); seen1.add(d1); n += 1
    assert len(seen0) == n and len(seen1) == n


def test_key_is_a_sum_of_position_keyed_terms():
    """Swapping two words changes the key by exactly the four terms involved -- checked by rebuilding the key
    from single-word differences, which a definition that mixed words into a running state would not allow."""
    a = _digest([[5, 8]])
    b = _digest([[8, 5]])
    c = _digest([[5, 5]])
    e = _digest([[8, 8]])
    for k in (0, 1):
        assert (a[k] + b[k]) & MASK == (c[k] + e[k]) & MASK
    # negative ids (never valid targets, but the key is defined on the words as given) are taken as unsigned
    assert _digest([[-1]]) != _digest([[2**31 - 1]])

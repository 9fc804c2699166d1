"""Pins of the checker's population generator step (Sec. 4.1: candidates kept, the rest re-initialised from
them with an optional mutation): exact copies without mutation, numpy's own binary32 arithmetic with it,
and the bookkeeping of who is whose parent."""
import numpy as np

import oracle


def _case(P=7, count=13, seed=0):
    rng = np.random.default_rng(seed)
    params = rng.standard_normal((P, count)).astype(np.float32)
    noise = rng.standard_normal((P, count)).astype(np.float32)
    rank = rng.permutation(P).astype(np.int32)
    return params, noise, rank


def test_without_mutation_losers_are_exact_copies_of_the_candidates_in_turn():
    params, _, rank = _case()
    out = oracle.population_refill(params, rank, 3, 0.0)
    for j in range(7):
        src = rank[j] if j < 3 else rank[(j - 3) % 3]
        assert np.array_equal(out[rank[j]], params[src]), j
    # parents in the order best, second, third, best, ...
    assert np.array_equal(out[rank[3]], params[rank[0]]) and np.array_equal(out[rank[6]], params[rank[0]])
    assert np.array_equal(out[rank[4]], params[rank[1]]) and np.array_equal(out[rank[5]], params[rank[2]])


def test_mutation_is_parent_plus_sigma_noise_in_binary32():
    params, noise, rank = _case(P=5, count=1001, seed=3)
    sigma = np.float32(0.0625 + 2.0 ** -12)
    out = oracle.population_refill(params, rank, 2, float(sigma), noise)
    for j in range(2, 5):
        want = params[rank[(j - 2) % 2]] + (sigma * noise[rank[j]]).astype(np.float32)   # numpy rounds each op to fp32
        assert np.array_equal(out[rank[j]].view(np.uint32), want.astype(np.float32).view(np.uint32))
        assert not np.array_equal(out[rank[j]], params[rank[j]])
    for j in range(2):
        assert np.array_equal(out[rank[j]], params[rank[j]])


def test_keep_everyone_or_only_the_best():
    params, noise, rank = _case(P=6, count=4, seed=5)
    assert np.array_equal(oracle.population_refill(params, rank, 6, 0.5, noise), params)
    out = oracle.population_refill(params, rank, 1, 0.0)
    assert all(np.array_equal(out[a], params[rank[0]]) for a in range(6))
    # the noise row used is the child's own, not the parent's
    out = oracle.population_refill(np.zeros_like(params), rank, 1, 1.0, noise)
    for j in range(1, 6):
        assert np.array_equal(out[rank[j]], noise[rank[j]])

"""Pins for the oracle's fit (Section 3.2 "Model Compression": grouping, per-group k-means, shared-pattern
k-means, index histogram, codebooks).  The fitted pattern *values* for a given tensor cannot be pinned -- the
paper prints none -- but every step of the algorithm can: planted patterns must be recovered, the shared-pattern
objective must fall and end in a fixed point of Lloyd's iteration, degenerate inputs must be reproduced exactly,
the histogram must be a recount of what the encoder's quantiser returns, and the subsample must be a sample
without replacement.  Each test is built so that one plausible mistake (centroids never updated, a wrong group
picked, a histogram of the wrong groups, a biased or repeating sample) fails it.  No GPU, no HIP library.
"""
from __future__ import annotations

import numpy as np
import pytest

G, K = 128, 16


def _planted_patterns():
    """Four hand-made, well separated, ascending 16-vectors in [-1, 1]; each ends in +1 so that the group's
    largest magnitude is that element and normalisation leaves the others as they are."""
    lin = np.linspace(-0.9, 1.0, K)
    p0 = lin
    p1 = np.tanh(1.5 * lin) / np.tanh(1.5)
    p2 = np.concatenate([np.linspace(-0.30, 0.30, K - 1), [1.0]])
    p3 = np.concatenate([np.linspace(-0.95, -0.55, 8), np.linspace(0.55, 0.93, 7), [1.0]])
    P = np.stack([p0, p1, p2, p3])
    assert (np.diff(P, axis=1) > 0.035).all() and (P[:, -1] == 1.0).all()
    return P


def _groups_from_patterns(P, per_pattern, noise, rng, scales=(0.02, 0.5, 3.0)):
    """Groups whose per-group 16-level k-means is known in advance: every level of the planted pattern (plus one
    noise value per group and level, none on the last level) appears eight times, times the group's scale."""
    groups, truth, owner = [], [], []
    for s in range(P.shape[0]):
        for g in range(per_pattern):
            e = rng.normal(0.0, noise, K)
            e[-1] = 0.0
            level = np.sort(P[s] + e)
            assert level[-1] == 1.0 and np.abs(level).max() == 1.0
            vals = np.repeat(level, G // K) * scales[g % len(scales)]
            groups.append(rng.permutation(vals))
            truth.append(level)
            owner.append(s)
    return np.array(groups), np.array(truth), np.array(owner)


def _match_rows(found, want):
    """For every row of `want` the index of the nearest row of `found` (Euclidean)."""
    d = ((want[:, None, :] - found[None, :, :]) ** 2).sum(axis=2)
    return d.argmin(axis=1), np.sqrt(d.min(axis=1))


@pytest.mark.parametrize("seed", [0, 1, 7, 12345])
def test_planted_patterns_are_recovered(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    P = _planted_patterns()
    noise, per = 0.01, 150
    x, truth, owner = _groups_from_patterns(P, per, noise, rng)
    order = rng.permutation(len(x))  # clusters interleaved in memory
    x, truth, owner = x[order], truth[order], owner[order]
    t = oracle.fit_trace(x.astype(np.float16).view(np.uint16), 4, 12, seed)
    # step 3: every group's own pattern is the planted one with that group's noise (fp16 storage of the values and
    # the FP32 division move it by a few 1e-4)
    assert np.abs(t["patterns"] - truth).max() < 2e-3
    # step 4: the shared patterns are the four cluster means -- within the noise of a mean over 150 groups
    # (0.01 / sqrt(150) = 8e-4 per element) plus fp16 rounding, far inside the noise of a single group (0.01):
    # a k-means that never moved its seeds off the groups they were drawn from would miss by ~0.01 per element
    got = t["cent"].view(np.float16).astype(np.float64)
    idx, _ = _match_rows(got, P)
    assert sorted(idx) == [0, 1, 2, 3]  # one shared pattern per planted one
    means = np.stack([truth[owner == s].mean(axis=0) for s in range(4)])
    assert np.abs(got[idx] - means).max() < 1.2e-3
    assert np.abs(got[idx] - P).max() < 4.5e-3
    single = np.abs(truth - P[owner]).max(axis=1)
    assert np.median(single) > 0.015  # a single group is typically further off than the bound above in some element
    # step 5: every group is quantised with the pattern of its own cluster
    for s in range(4):
        assert t["hist"][idx[s]].sum() == per * G


def test_shared_pattern_objective_falls_to_a_fixed_point(oracle):
    from paper_2505_06901_amd import workloads as W
    w = W.config_weight("tiny")
    for S, seed in ((16, 0), (5, 3), (64, 9)):
        t = oracle.fit_trace(w.view(np.uint16), S, 12, seed)
        obj = t["objective"]
        assert len(obj) >= 3
        # Lloyd's iteration never increases the objective (the empty-cluster restart moves an unused centre onto a
        # data point, which cannot increase it either); the tolerance covers the double-precision sums
        assert (np.diff(obj) <= 1e-9 * obj[0]).all()
        assert obj[-1] < 0.9 * obj[0]  # and it does move: the seeding alone is clearly worse
        # the objective is what it says: recomputed in numpy from the per-group patterns, it lies between the last
        # assignment pass (centres before rounding) and a few fp16 roundings of the centres away from it
        pats = t["patterns"]
        cent = t["cent"].view(np.float16).astype(np.float64)
        d = ((pats[:, None, :] - cent[None, :, :]) ** 2).sum(axis=2)
        assert d.min(axis=1).sum() == pytest.approx(obj[-1], rel=2e-2)
        if len(obj) < 50:
            # converged: no group changed its pattern in the last pass, so the centres are the means of their groups and
            # one more Lloyd step (from the fp16 centres, in numpy) has next to nothing left to gain
            a = d.argmin(axis=1)
            after = 0.0
            for s in range(S):
                if (a == s).any():
                    after += ((pats[a == s] - pats[a == s].mean(axis=0)) ** 2).sum()
            assert after >= 0.98 * d.min(axis=1).sum()


def test_per_group_patterns_are_the_1d_kmeans_of_the_normalised_group(oracle):
    from paper_2505_06901_amd import workloads as W
    w = W.config_weight("tiny").reshape(-1, G)
    t = oracle.fit_trace(w.view(np.uint16), 4, 12, 0)
    assert np.array_equal(t["pick"], np.arange(len(w)))  # 512 groups: all of them, in order
    for g in (0, 1, 17, 255, 511):
        v = w[g].astype(np.float32)
        v = v / np.abs(v).max()  # FP32 division by the group's largest magnitude
        c, _, _ = oracle.kmeans_1d(v, K, 25)
        assert np.array_equal(c, t["patterns"][g])
    assert (np.diff(t["patterns"], axis=1) >= 0).all()
    assert np.abs(t["patterns"]).max() <= 1.0


def test_fewer_distinct_groups_than_patterns_are_reproduced_exactly(oracle):
    rng = np.random.default_rng(5)
    P = _planted_patterns()
    x, truth, _ = _groups_from_patterns(P, 1, 0.0, rng)  # four distinct groups
    x = np.concatenate([x, x[:2] * 2.0])               # two repeats at another scale: same normalised pattern
    for S in (4, 6, 9):
        t = oracle.fit_trace(x.astype(np.float16).view(np.uint16), S, 12, 2)
        assert t["objective"][-1] < 1e-20  # every group sits on a shared pattern
        got = t["cent"].view(np.float16).astype(np.float64)
        _, dist = _match_rows(got, t["patterns"])
        assert dist.max() < 1.5e-3  # fp16 rounding of 16 elements
        # and the quantiser then reproduces every value of these groups to within fp16 rounding of centroid x scale
        cent, lens = t["cent"], t["lens"]
        blocks, meta = oracle.encode(cent, lens, x.astype(np.float16).view(np.uint16))
        dec = oracle.decode(cent, lens, blocks, meta).view(np.float16).astype(np.float64)
        ref = x.astype(np.float16).astype(np.float64)
        assert np.abs(dec - ref).max() <= 2e-3 * np.abs(ref).max(axis=1, keepdims=True).max()


def test_histogram_is_a_recount_of_the_quantiser(oracle):
    from paper_2505_06901_amd import workloads as W
    w = W.config_weight("tiny").reshape(-1, G)
    t = oracle.fit_trace(w.view(np.uint16), 16, 12, 0)
    hist = np.zeros((16, K), np.uint64)
    for g in t["pick"]:
        _, p, idx, _ = oracle.quantize_group(t["cent"], w[g].view(np.uint16))
        hist[p] += np.bincount(idx, minlength=K).astype(np.uint64)
    assert np.array_equal(hist, t["hist"])
    # the codebooks come from these counts (+1 each): optimal cost for them, checked against plain Huffman
    for p in range(16):
        if hist[p].sum():
            free = oracle.huffman_lengths(hist[p] + 1)
            if free.max() <= 12:
                assert ((hist[p] + 1) * t["lens"][p]).sum() == ((hist[p] + 1) * free).sum()


def test_subsample_is_a_seeded_sample_without_replacement(oracle):
    n_all = 65536 + 5000
    rng = np.random.default_rng(11)
    # two kinds of groups, recognisable from their data: the first half of the tensor follows planted pattern 0,
    # the second half pattern 3, each group with its own small noise on the levels
    P = _planted_patterns()[[0, 3]]
    kind = (np.arange(n_all) >= n_all // 2).astype(np.int64)
    e = rng.normal(0.0, 0.004, (n_all, K))
    e[:, -1] = 0.0
    levels = np.sort(P[kind] + e, axis=1)
    xh = np.repeat(levels, G // K, axis=1).astype(np.float16)
    t = oracle.fit_trace(xh.view(np.uint16), 2, 12, 42)
    pick = t["pick"]
    assert t["n_fit"] == 65536 and len(pick) == 65536
    assert (np.diff(pick) > 0).all()                # ascending and distinct: no group twice
    assert pick.min() >= 0 and pick.max() < n_all
    # roughly uniform over the tensor: 5000 of 70536 are left out, spread over the deciles (a sample that took the
    # first 65536 groups, or every group of a prefix, fails this)
    left_out = np.setdiff1d(np.arange(n_all), pick)
    assert len(left_out) == 5000
    counts = np.bincount((left_out * 10) // n_all, minlength=10)
    assert counts.min() > 380 and counts.max() < 620  # 500 +- 5 sigma
    # the per-group patterns belong to the picked groups: entry i is the k-means of group pick[i]
    for i in (0, 1, 30000, 65535):
        v = xh[pick[i]].astype(np.float32)
        c, _, _ = oracle.kmeans_1d(v / np.abs(v).max(), K, 25)
        assert np.array_equal(c, t["patterns"][i])
    # the two shared patterns are the two planted ones, and the histogram counts exactly the picked groups:
    # a recount over x[pick] through the encoder (whose indices are tied to the quantiser elsewhere) gives the
    # same table; a histogram over the first 65 536 groups instead would hold 35 268 groups of the first kind
    got = t["cent"].view(np.float16).astype(np.float64)
    idx, dist = _match_rows(got, P)
    assert sorted(idx) == [0, 1] and dist.max() < 5e-3
    picked_kinds = np.bincount(kind[pick], minlength=2)
    assert picked_kinds[0] != n_all // 2 and abs(int(picked_kinds[0]) - 32768) < 400
    for s in range(2):
        assert t["hist"][idx[s]].sum() == picked_kinds[s] * G
    blocks, meta = oracle.encode(t["cent"], t["lens"], xh[pick].view(np.uint16))
    sym, _ = oracle.decode_indices(t["lens"], 2, blocks, meta)
    pat = (meta >> 16) & 63
    recount = np.zeros((2, K), np.uint64)
    for s in range(2):
        recount[s] = np.bincount(sym[pat == s].reshape(-1), minlength=K)
    assert np.array_equal(recount, t["hist"])
    # another seed picks other groups; the same seed the same ones
    t2 = oracle.fit_trace(xh.view(np.uint16), 2, 12, 43)
    assert not np.array_equal(t2["pick"], pick)
    t3 = oracle.fit_trace(xh.view(np.uint16), 2, 12, 42)
    assert np.array_equal(t3["pick"], pick) and np.array_equal(t3["cent"], t["cent"])


def test_fit_and_fit_trace_agree(oracle):
    from paper_2505_06901_amd import workloads as W
    w = W.config_weight("tiny")
    cent, lens, hist, nfit = oracle.fit(w.view(np.uint16), 16, 12, 0)
    t = oracle.fit_trace(w.view(np.uint16), 16, 12, 0)
    assert np.array_equal(cent, t["cent"]) and np.array_equal(lens, t["lens"])
    assert np.array_equal(hist, t["hist"]) and nfit == t["n_fit"]

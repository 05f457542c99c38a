"""Pins of the fp64 ASG oracle (criterion named in Sec. 2.3; the paper prints no formula, so the
oracle's definition is a stated reading -- these tests pin the code to that definition and to
what the mathematics fixes, by means that share nothing with the oracle's recursions):
brute-force enumeration of every labelling / alignment, closed forms for degenerate cases,
central finite differences, and invariants."""
import itertools
import math

import numpy as np
import pytest

import oracle


def path_score(f, g, pi):
    s = sum(f[t, c] for t, c in enumerate(pi))
    s += sum(g[pi[t], pi[t - 1]] for t in range(1, len(pi)))
    return s


def alignments(T, L):
    """all s_0..s_{T-1} with s_0 = 0, s_{T-1} = L-1, steps in {0, 1}"""
    if L < 1 or L > T:
        return
    for steps in itertools.product((0, 1), repeat=T - 1):
        if sum(steps) == L - 1:
            s = [0]
            for d in steps:
                s.append(s[-1] + d)
            yield s


def brute(f, g, y):
    """(FCC, FAL, node occupancy difference [T,C], edge occupancy difference [C,C]) by enumeration"""
    T, C = f.shape
    full = [(pi, path_score(f, g, pi)) for pi in itertools.product(range(C), repeat=T)]
    forced = [(tuple(y[s] for s in al), None) for al in alignments(T, len(y))]
    forced = [(pi, path_score(f, g, pi)) for pi, _ in forced]

    def lse(v):
        m = max(v)
        return m + math.log(sum(math.exp(x - m) for x in v))

    fcc, fal = lse([s for _, s in full]), lse([s for _, s in forced])
    node, edge = np.zeros((T, C)), np.zeros((C, C))
    for paths, z, sign in ((full, fcc, 1.0), (forced, fal, -1.0)):
        for pi, s in paths:
            p = sign * math.exp(s - z)
            for t, c in enumerate(pi):
                node[t, c] += p
                if t >= 1:
                    edge[c, pi[t - 1]] += p
    return fcc, fal, node, edge


@pytest.mark.parametrize("seed,T,C,y", [(0, 4, 3, [1, 2]), (1, 5, 3, [0, 0, 2]), (2, 3, 4, [3, 1, 2]), (3, 5, 2, [1]),
                                        (4, 6, 3, [2, 1, 2, 0]), (5, 1, 3, [2])])
def test_asg_matches_enumeration(seed, T, C, y):
    rng = np.random.default_rng(seed)
    f = rng.normal(scale=2.0, size=(T + 2, C))      # two padded frames that must not matter
    g = rng.normal(scale=1.5, size=(C, C))
    fcc, fal, node, edge = brute(f[:T], g, y)
    loss, ge, gt, ofcc, ofal = oracle.asg(f[None], g, [y], [T], [len(y)], want_terms=True)
    assert abs(ofcc[0] - fcc) < 1e-12 * max(1, abs(fcc))
    assert abs(ofal[0] - fal) < 1e-12 * max(1, abs(fal))
    assert abs(loss[0] - (fcc - fal)) < 1e-11
    assert np.allclose(ge[0, :T], node, atol=1e-12)
    assert np.all(ge[0, T:] == 0)
    assert np.allclose(gt, edge, atol=1e-12)


def test_asg_batch_sums_transition_gradient_and_scales():
    rng = np.random.default_rng(7)
    C, Tp = 3, 5
    f = rng.normal(size=(3, Tp, C))
    g = rng.normal(size=(C, C))
    ys, Ts = [[0, 1], [2], [1, 1, 0]], [5, 3, 4]
    tg = np.zeros((3, 3), dtype=np.int32)
    for b, y in enumerate(ys):
        tg[b, :len(y)] = y
    loss, ge, gt = oracle.asg(f, g, tg, Ts, [len(y) for y in ys], grad_scale=0.5)
    edge_sum = np.zeros((C, C))
    for b, y in enumerate(ys):
        fcc, fal, node, edge = brute(f[b, :Ts[b]], g, y)
        assert abs(loss[b] - (fcc - fal)) < 1e-11
        assert np.allclose(ge[b, :Ts[b]], 0.5 * node, atol=1e-12)
        edge_sum += edge
    assert np.allclose(gt, 0.5 * edge_sum, atol=1e-12)


def test_asg_closed_forms():
    rng = np.random.default_rng(11)
    T, C = 9, 5
    f = rng.normal(scale=3.0, size=(1, T, C))
    # zero transitions: the labellings factor over frames
    g0 = np.zeros((C, C))
    _, _, _, fcc, _ = oracle.asg(f, g0, [[1]], [T], [1], want_terms=True)
    assert abs(fcc[0] - np.log(np.exp(f[0]).sum(1)).sum()) < 1e-12
    g = rng.normal(size=(C, C))
    # one label: the only alignment repeats it
    _, _, _, _, fal = oracle.asg(f, g, [[3]], [T], [1], want_terms=True)
    assert abs(fal[0] - (f[0, :, 3].sum() + (T - 1) * g[3, 3])) < 1e-12
    # as many labels as frames: the only alignment advances every frame
    y = rng.integers(0, C, size=T)
    _, _, _, _, fal = oracle.asg(f, g, [y], [T], [T], want_terms=True)
    want = sum(f[0, t, y[t]] for t in range(T)) + sum(g[y[t], y[t - 1]] for t in range(1, T))
    assert abs(fal[0] - want) < 1e-12
    # a single class: both lattices hold the same single path
    f1 = rng.normal(size=(1, 6, 1))
    loss, ge, gt = oracle.asg(f1, np.array([[0.7]]), [[0, 0]], [6], [2])
    # C(5,1) = 5 alignments of two equal labels over six frames all spell the same labelling
    assert abs(loss[0] + math.log(5.0)) < 1e-12
    # transitions that are log-probabilities of a Markov chain and emissions that are per-frame
    # log-likelihoods: FCC is the chain's total likelihood with a flat start, by matrix products
    A = rng.random((C, C)); A /= A.sum(0, keepdims=True)         # A[i, j] = P(i | j)
    e = rng.random((T, C))
    v = e[0].copy()
    for t in range(1, T):
        v = e[t] * (A @ v)
    _, _, _, fcc, _ = oracle.asg(np.log(e)[None], np.log(A), [[0]], [T], [1], want_terms=True)
    assert abs(fcc[0] - math.log(v.sum())) < 1e-12


def test_asg_finite_differences():
    rng = np.random.default_rng(5)
    B, Tp, C = 2, 7, 4
    f = rng.normal(size=(B, Tp, C))
    g = rng.normal(size=(C, C))
    tg, Ts, Ls = np.array([[1, 3, 3, 0], [2, 0, 0, 0]], dtype=np.int32), [7, 5], [4, 2]
    total = lambda ff, gg: oracle.asg(ff, gg, tg, Ts, Ls)[0].sum()
    _, ge, gt = oracle.asg(f, g, tg, Ts, Ls)
    h = 1e-6
    for idx in [(0, 0, 1), (0, 3, 3), (0, 6, 0), (1, 2, 2), (1, 4, 0), (1, 5, 1), (1, 6, 3)]:
        fp, fm = f.copy(), f.copy()
        fp[idx] += h
        fm[idx] -= h
        assert abs((total(fp, g) - total(fm, g)) / (2 * h) - ge[idx]) < 1e-7
    for i in range(C):
        for j in range(C):
            gp, gm = g.copy(), g.copy()
            gp[i, j] += h
            gm[i, j] -= h
            assert abs((total(f, gp) - total(f, gm)) / (2 * h) - gt[i, j]) < 1e-7


def test_asg_invariants():
    rng = np.random.default_rng(9)
    B, Tp, C, Lmax = 3, 40, 6, 12
    f = rng.normal(scale=2.0, size=(B, Tp, C))
    g = rng.normal(size=(C, C))
    tg = rng.integers(0, C, size=(B, Lmax)).astype(np.int32)
    Ts, Ls = np.array([40, 33, 12]), np.array([12, 5, 12])
    loss, ge, gt = oracle.asg(f, g, tg, Ts, Ls)
    assert np.all(loss >= -1e-12)                                   # alignments are a subset of labellings
    for b in range(B):
        assert np.allclose(ge[b, :Ts[b]].sum(1), 0, atol=1e-12)     # both occupancies sum to 1 per frame
        assert np.all(ge[b, Ts[b]:] == 0)
    assert abs(gt.sum()) < 1e-10                                    # both use T-1 edges per utterance
    # a per-frame constant on the emissions, or a constant on all transitions, cancels in FCC - FAL
    shift = rng.normal(size=(B, Tp, 1))
    loss2, ge2, gt2 = oracle.asg(f + shift, g + 0.37, tg, Ts, Ls)
    assert np.allclose(loss2, loss, atol=1e-9) and np.allclose(ge2, ge, atol=1e-10) and np.allclose(gt2, gt, atol=1e-10)
    # relabelling the classes permutes everything consistently
    perm = rng.permutation(C)
    inv = np.argsort(perm)
    loss3, ge3, gt3 = oracle.asg(f[:, :, inv], g[np.ix_(inv, inv)], perm[tg].astype(np.int32), Ts, Ls)
    assert np.allclose(loss3, loss, atol=1e-9)
    assert np.allclose(ge3[:, :, perm], ge, atol=1e-10) and np.allclose(gt3[np.ix_(perm, perm)], gt, atol=1e-10)


def test_asg_degenerate_cases():
    C = 3
    f = np.zeros((4, 5, C))
    g = np.zeros((C, C))
    tg = np.array([[0, 1, 2, 0, 1, 2], [0] * 6, [1] * 6, [2, 1, 0, 0, 0, 0]], dtype=np.int32)
    loss, ge, gt = oracle.asg(f, g, tg, [5, 0, 5, 0], [6, 0, 0, 3])
    assert np.isposinf(loss[0]) and loss[1] == 0 and np.isposinf(loss[2]) and np.isposinf(loss[3])
    assert np.all(ge == 0) and np.all(gt == 0)
    # flat scores: FCC = T log C, FAL = log(number of alignments)
    loss, _, _ = oracle.asg(np.zeros((1, 5, C)), g, [[0, 1, 2]], [5], [3])
    assert abs(loss[0] - (5 * math.log(3) - math.log(math.comb(4, 2)))) < 1e-12
    with pytest.raises(ValueError):
        oracle.asg(f, g, np.full((4, 6), 3, dtype=np.int32), [5] * 4, [1] * 4)
    with pytest.raises(ValueError):
        oracle.asg(f, g, tg, [6, 5, 5, 5], [1] * 4)

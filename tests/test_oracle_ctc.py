"""Pins of the oracle's CTC (paper Sec. 2.3, the CTC criterion of Graves et al. 2006).

The paper prints no worked value, so the oracle is tied to the mathematics:
  * brute force: sum the probability of every frame labelling that collapses to the
    target (merge repeats, then drop blanks), for tiny T and C;
  * closed forms: single-alignment case, empty target, uniform scores;
  * finite differences for the gradient; per-frame invariants of the posteriors.
"""
import itertools
import math

import numpy as np
import pytest

import oracle


def collapse(path, blank):
    out, prev = [], None
    for c in path:
        if c != prev and c != blank:
            out.append(c)
        prev = c
    return tuple(out)


def brute_force(lp, target, blank=0):
    """(P(target), dP/dlp summed over alignments -> per (t,c) posterior mass)."""
    T, Cc = lp.shape
    tot = 0.0
    mass = np.zeros((T, Cc))
    for path in itertools.product(range(Cc), repeat=T):
        if collapse(path, blank) != tuple(target):
            continue
        p = math.exp(sum(lp[t, c] for t, c in enumerate(path)))
        tot += p
        for t, c in enumerate(path):
            mass[t, c] += p
    return tot, mass


def rand_lp(rng, B, T, Cc, scale=1.5):
    z = rng.standard_normal((B, T, Cc)) * scale
    return z - np.log(np.exp(z).sum(-1, keepdims=True))


CASES = [
    (4, 3, [1]), (5, 3, [1, 2]), (6, 3, [1, 1]), (6, 4, [2, 3, 2]), (7, 3, [1, 2, 2]),
    (8, 3, [1, 1, 2]), (8, 4, [3, 1, 3]), (3, 3, [1, 2, 1]), (5, 4, []), (6, 3, [2, 2, 2]),
    (1, 3, [2]), (1, 3, []), (2, 4, [3, 3][:1]),
]


@pytest.mark.parametrize("T,Cc,target", CASES)
def test_loss_and_gradient_match_enumeration(T, Cc, target):
    rng = np.random.default_rng(100 + T * 7 + Cc + len(target))
    lp = rand_lp(rng, 1, T, Cc)
    Lmax = max(1, len(target))
    tg = np.zeros((1, Lmax), dtype=np.int32)
    tg[0, :len(target)] = target
    loss, grad = oracle.ctc(lp, tg, [T], [len(target)])
    P, mass = brute_force(lp[0], target)
    assert P > 0
    assert abs(math.exp(-loss[0]) - P) <= 1e-12 * P
    # d(-log P)/dlp[t,c] = -(sum of alignment probabilities through (t,c)) / P
    np.testing.assert_allclose(grad[0], -mass / P, rtol=0, atol=1e-12)


@pytest.mark.parametrize("T,Cc,target,blank", [(5, 3, [0, 1], 2), (6, 4, [3, 0, 3], 1)])
def test_blank_index_other_than_zero(T, Cc, target, blank):
    rng = np.random.default_rng(5)
    lp = rand_lp(rng, 1, T, Cc)
    tg = np.array([target], dtype=np.int32)
    loss, grad = oracle.ctc(lp, tg, [T], [len(target)], blank=blank)
    P, mass = brute_force(lp[0], target, blank=blank)
    assert abs(math.exp(-loss[0]) - P) <= 1e-12 * P
    np.testing.assert_allclose(grad[0], -mass / P, atol=1e-12)


def test_infeasible_is_infinite_with_zero_gradient():
    rng = np.random.default_rng(1)
    lp = rand_lp(rng, 2, 4, 3)
    # needs 3 labels + 2 separating blanks = 5 frames > 4 ; second one is fine
    tg = np.array([[1, 1, 1], [1, 2, 0]], dtype=np.int32)
    loss, grad = oracle.ctc(lp, tg, [4, 4], [3, 2])
    assert np.isinf(loss[0]) and loss[0] > 0
    assert np.all(grad[0] == 0)
    assert np.isfinite(loss[1]) and np.all(np.isfinite(grad))
    P, _ = brute_force(lp[0], [1, 1, 1])
    assert P == 0.0


def test_single_alignment_closed_form():
    # T = L, no adjacent repeats: exactly one alignment, loss = -sum_t lp[t, l_t]
    rng = np.random.default_rng(2)
    T, Cc = 9, 6
    lab = np.array([1, 2, 3, 4, 5, 1, 2, 3, 4], dtype=np.int32)
    lp = rand_lp(rng, 1, T, Cc)
    loss, grad = oracle.ctc(lp, lab[None], [T], [T])
    assert abs(loss[0] + sum(lp[0, t, lab[t]] for t in range(T))) < 1e-12
    expect = np.zeros((T, Cc))
    expect[np.arange(T), lab] = -1.0
    np.testing.assert_allclose(grad[0], expect, atol=1e-12)


def test_empty_target_closed_form():
    rng = np.random.default_rng(3)
    lp = rand_lp(rng, 1, 11, 5)
    loss, grad = oracle.ctc(lp, np.zeros((1, 1), np.int32), [11], [0])
    assert abs(loss[0] + lp[0, :, 0].sum()) < 1e-12
    expect = np.zeros((11, 5))
    expect[:, 0] = -1.0
    np.testing.assert_allclose(grad[0], expect, atol=1e-12)


@pytest.mark.parametrize("T,L", [(5, 2), (12, 3), (30, 7), (40, 1), (9, 9)])
def test_uniform_scores_count_alignments(T, L):
    # every labelling has probability C^-T; a target with no adjacent repeats has
    # binom(T+L, 2L) alignments
    Cc = 29
    lab = (np.arange(L) % 2 + 1).astype(np.int32)  # 1,2,1,2,... no adjacent repeats
    lp = np.full((1, T, Cc), -math.log(Cc))
    loss, _ = oracle.ctc(lp, lab[None], [T], [L])
    expect = T * math.log(Cc) - math.log(math.comb(T + L, 2 * L))
    assert abs(loss[0] - expect) < 1e-10 * max(1.0, abs(expect))


def test_alpha_beta_consistency_every_frame():
    # lse_s( alpha_t(s) + beta_t(s) - lp[t, l'_s] ) = log P at every t
    rng = np.random.default_rng(4)
    B, T, Cc, Lmax = 3, 40, 8, 9
    lp = rand_lp(rng, B, T, Cc)
    tl = np.array([9, 4, 0], dtype=np.int32)
    il = np.array([40, 33, 17], dtype=np.int32)
    tg = rng.integers(1, Cc, size=(B, Lmax)).astype(np.int32)
    loss, grad, al, be = oracle.ctc(lp, tg, il, tl, want_lattice=True)
    for b in range(B):
        S = 2 * tl[b] + 1
        ext = [0 if s % 2 == 0 else tg[b, (s - 1) // 2] for s in range(S)]
        for t in range(il[b]):
            u = al[b, t, :S] + be[b, t, :S] - lp[b, t, ext]
            u = u[np.isfinite(u)]
            lse = u.max() + math.log(np.exp(u - u.max()).sum())
            assert abs(lse + loss[b]) < 1e-10 * max(1.0, abs(loss[b]))
        assert np.all(np.isneginf(al[b, il[b]:])) and np.all(np.isneginf(be[b, il[b]:]))


def test_posterior_invariants_and_masking():
    rng = np.random.default_rng(6)
    B, T, Cc, Lmax = 4, 60, 29, 12
    lp = rand_lp(rng, B, T, Cc, scale=1.4)
    tl = np.array([12, 5, 1, 8], dtype=np.int32)
    il = np.array([60, 41, 30, 55], dtype=np.int32)
    tg = rng.integers(1, 6, size=(B, Lmax)).astype(np.int32)  # few classes -> repeats occur
    loss, grad = oracle.ctc(lp, tg, il, tl)
    G = -grad
    for b in range(B):
        np.testing.assert_allclose(G[b, :il[b]].sum(-1), 1.0, atol=1e-10)
        assert np.all(G[b, il[b]:] == 0)
        assert G[b].min() >= 0
        present = set([0]) | set(tg[b, :tl[b]].tolist())
        absent = [c for c in range(Cc) if c not in present]
        assert np.all(G[b][:, absent] == 0)


def test_gradient_finite_differences_lp_and_logits():
    rng = np.random.default_rng(7)
    B, T, Cc, Lmax = 2, 14, 6, 5
    z = rng.standard_normal((B, T, Cc))
    tl = np.array([5, 3], dtype=np.int32)
    il = np.array([14, 11], dtype=np.int32)
    tg = np.array([[1, 1, 2, 3, 3], [4, 5, 4, 0, 0]], dtype=np.int32)
    lp = oracle.logsoftmax_fwd(z)
    _, g_lp = oracle.ctc(lp, tg, il, tl)
    _, _, g_z = oracle.ctc_from_logits(z, tg, il, tl, grad_scale=0.5)
    h = 1e-6
    for _ in range(40):
        b, t, c = rng.integers(B), rng.integers(T), rng.integers(Cc)
        d = np.zeros_like(z)
        d[b, t, c] = h
        lp_p, lp_m = lp + d, lp - d
        fd = (oracle.ctc(lp_p, tg, il, tl)[0].sum() - oracle.ctc(lp_m, tg, il, tl)[0].sum()) / (2 * h)
        assert abs(fd - g_lp[b, t, c]) < 1e-7 * max(1.0, abs(fd))
        fz = (oracle.ctc_from_logits(z + d, tg, il, tl)[0].sum()
              - oracle.ctc_from_logits(z - d, tg, il, tl)[0].sum()) / (2 * h)
        assert abs(0.5 * fz - g_z[b, t, c]) < 1e-7 * max(1.0, abs(fz))
    # gradient wrt logits sums to zero over classes on valid frames, is zero beyond
    for b in range(B):
        np.testing.assert_allclose(g_z[b, :il[b]].sum(-1), 0.0, atol=1e-12)
        assert np.all(g_z[b, il[b]:] == 0)


def test_zero_frames():
    lp = np.full((2, 3, 4), -math.log(4))
    loss, grad = oracle.ctc(lp, np.array([[1], [1]], np.int32), [0, 0], [0, 1])
    assert loss[0] == 0.0 and np.isinf(loss[1])
    assert np.all(grad == 0)


def test_rejects_bad_labels():
    lp = np.full((1, 3, 4), -math.log(4))
    for bad in ([0], [4], [-1]):
        with pytest.raises(ValueError):
            oracle.ctc(lp, np.array([bad], np.int32), [3], [1])
    with pytest.raises(ValueError):
        oracle.ctc(lp, np.array([[1]], np.int32), [4], [1])

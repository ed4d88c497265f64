"""Pins of the oracle's truncated-support functions (Section "Top-k, Nucleus Sampling, and Masking"):
top-k by a full sort, the nucleus rule on k candidates, the truncated draw, and Gumbel-top-k.
Each is checked against something other than itself: numpy's sort, a brute-force cumulative softmax,
the already pinned masked sampler, the plain sampler, and the closed-form laws by chi-square."""
import numpy as np
import pytest
from scipy import stats

import fs_workloads as wl

TRUNC, GUMBEL = 0, 1


def _case(B=3, D=64, V=300, seed=11, scale=3.0):
    H, W = wl.make_small(D=D, V=V, B=B, data_seed=seed, w_row_scale=scale)
    return H, W


def test_topk_row_equals_numpy_sort_and_breaks_ties_by_lower_id(orc):
    rng = np.random.default_rng(1)
    for V, k in [(1, 1), (5, 3), (300, 64), (300, 300), (40, 64)]:
        key = rng.normal(size=V)
        key[rng.integers(0, V, size=max(1, V // 5))] = 0.25          # planted ties
        if V > 8:
            key[3] = np.nan                                          # NaN counts as -inf
        ok, oi, nxt = orc.topk_row(key, k, vocab_offset=1000)
        clean = np.where(np.isnan(key), -np.inf, key)
        order = np.lexsort((np.arange(V), -clean))                   # key descending, id ascending
        m = min(k, V)
        assert np.array_equal(oi[:m], order[:m] + 1000)
        assert np.array_equal(ok[:m], clean[order[:m]])
        assert np.all(oi[m:] == -1) and np.all(ok[m:] == -np.inf)
        assert nxt == (clean[order[k]] if k < V else -np.inf)


def test_top_p_cut_equals_brute_force_cumulative_softmax(orc):
    rng = np.random.default_rng(2)
    for trial in range(200):
        k = int(rng.integers(1, 65))
        z = np.sort(rng.normal(scale=rng.uniform(0.2, 4.0), size=k))[::-1].copy()
        pad = int(rng.integers(0, 4))
        zp = np.concatenate([z, np.full(pad, -np.inf)])
        p = float(rng.choice([0.05, 0.3, 0.5, 0.9, 0.95, 0.999, 1.0]))
        q = np.exp(z - z.max())
        q /= q.sum()
        cum = np.cumsum(q)
        want = k if p >= 1.0 else int(np.argmax(cum >= p)) + 1 if np.any(cum >= p) else k
        n, before = orc.top_p_cut(zp, p)
        assert n == want, (trial, k, p)
        assert abs(before - (cum[n - 2] if n >= 2 else 0.0)) < 1e-12
    assert orc.top_p_cut(np.array([-np.inf, -np.inf]), 0.9)[0] == 0     # nothing has mass
    assert orc.top_p_cut(np.array([2.0]), 1e-9)[0] == 1                 # at least one candidate
    # an exact boundary: masses 0.5, 0.25, 0.25 -> p = 0.5 keeps one, p just above keeps two
    z = np.log(np.array([0.5, 0.25, 0.25]))
    assert orc.top_p_cut(z, 0.5)[0] == 1 and orc.top_p_cut(z, 0.5000001)[0] == 2


def test_truncated_draw_is_the_masked_draw_on_the_kept_set(orc):
    # pathwise: mask everything outside the kept candidates and run the (pinned) masked sampler
    H, W = _case(B=6, V=500)
    tau = np.linspace(0.5, 1.5, 6).astype(np.float32)
    for k, p in [(1, 1.0), (8, 1.0), (50, 0.9), (64, 0.5), (500, 0.8), (600, 1.0)]:
        r = orc.sample_topk(H, W, tau, k, top_p=p, mode=TRUNC, seed=9, row_offset=4)
        Y = orc.logits(H, W)
        for b in range(6):
            z = Y[b] / float(tau[b])
            order = np.lexsort((np.arange(500), -z))[:min(k, 500)]
            assert np.array_equal(r["top_id"][b, :len(order)], order)
            kept = order[:r["n_kept"][b]]
            allowed = np.zeros((1, 500), dtype=bool)
            allowed[0, kept] = True
            ref = orc.sample_full(H[b:b + 1], W, tau[b:b + 1], seed=9, row_ids=np.array([4 + b]),
                                  allowed_words=orc.pack_allowed(allowed))
            assert ref["idx"][0] == r["idx"][b] and ref["top1"][0] == r["top1"][b], (k, p, b)
    # k >= V and p = 1: nothing is cut, the draw is the plain sampler's
    r = orc.sample_topk(H, W, tau, 500, top_p=1.0, mode=TRUNC, seed=9)
    plain = orc.sample(H, W, tau, seed=9)
    assert np.array_equal(r["idx"], plain["idx"]) and np.array_equal(r["top1"], plain["top1"])


def test_gumbel_topk_first_element_is_the_plain_sample_and_order_is_a_full_sort(orc):
    H, W = _case(B=5, V=400)
    tau = np.full(5, 0.8, dtype=np.float32)
    plain = orc.sample(H, W, tau, seed=3, row_offset=10, vocab_offset=128)
    r1 = orc.sample_topk(H, W, tau, 1, mode=GUMBEL, seed=3, row_offset=10, vocab_offset=128)
    assert np.array_equal(r1["idx"], plain["idx"]) and np.array_equal(r1["top1"], plain["top1"])
    r = orc.sample_topk(H, W, tau, 37, mode=GUMBEL, seed=3, row_offset=10, vocab_offset=128)
    Y = orc.logits(H, W)
    for b in range(5):
        g, _ = orc.gumbel_from_words(orc.random_words(3, 10 + b, 128, 400))
        s = Y[b] / 0.8 + g          # float32(0.8) vs 0.8: compare by order, and values loosely
        s = Y[b] / float(tau[b]) + g
        order = np.argsort(-s, kind="stable")[:37]
        assert np.array_equal(r["top_id"][b], order + 128)
        assert np.allclose(r["top_key"][b], s[order], rtol=0, atol=1e-12)
        assert r["idx"][b] == order[0] + 128 and r["top2"][b] == r["top_key"][b, 1]


def _chi2(counts, expected):
    e, c = np.asarray(expected, float), np.asarray(counts, float)
    keep = e >= 5
    e2 = np.append(e[keep], e[~keep].sum())
    c2 = np.append(c[keep], c[~keep].sum())
    if e2[-1] == 0:
        e2, c2 = e2[:-1], c2[:-1]
    return ((c2 - e2) ** 2 / e2).sum(), stats.chi2.ppf(0.999, len(e2) - 1)


def test_truncated_draw_follows_the_renormalised_softmax_chi_square(orc):
    # same hidden row repeated: rows differ in the row word of the noise only
    V, k, p, n = 24, 8, 0.8, 60_000
    H1, W = wl.make_small(D=32, V=V, B=1, data_seed=5, w_row_scale=4.0)
    tau = 0.9
    z = orc.logits(H1, W)[0] / np.float32(tau).astype(np.float64)
    order = np.lexsort((np.arange(V), -z))[:k]
    q = np.exp(z[order] - z[order].max())
    q /= q.sum()
    nk = int(np.argmax(np.cumsum(q) >= p)) + 1
    target = np.zeros(V)
    target[order[:nk]] = q[:nk] / q[:nk].sum()
    Hn = np.repeat(H1, n, axis=0)
    r = orc.sample_topk(Hn, W, np.full(n, tau, np.float32), k, top_p=p, mode=TRUNC, seed=77)
    assert np.all(r["n_kept"] == nk)
    counts = np.bincount(r["idx"], minlength=V)
    assert counts[target == 0].sum() == 0                      # never outside the nucleus
    chi2, crit = _chi2(counts, target * n)
    assert chi2 < crit, (chi2, crit)
    # a planted mistake (nucleus applied to the full softmax instead of the k candidates) is told apart
    qf = np.exp(z - z.max()); qf /= qf.sum()
    nk_wrong = int(np.argmax(np.cumsum(qf[order]) >= p)) + 1
    if nk_wrong != nk:
        wrong = np.zeros(V); wrong[order[:nk_wrong]] = q[:nk_wrong] / q[:nk_wrong].sum()
        assert counts[wrong == 0].sum() > 0 or _chi2(counts, wrong * n)[0] > _chi2(counts, wrong * n)[1]


def test_gumbel_topk_is_sampling_without_replacement_chi_square(orc):
    # P(first two = (a, b)) = p_a p_b / (1 - p_a)  (the law of the Gumbel-top-k trick)
    V, n = 6, 80_000
    H1, W = wl.make_small(D=16, V=V, B=1, data_seed=8, w_row_scale=2.0)
    z = orc.logits(H1, W)[0]
    pr = np.exp(z - z.max()); pr /= pr.sum()
    r = orc.sample_topk(np.repeat(H1, n, axis=0), W, np.ones(n, np.float32), 2, mode=GUMBEL, seed=5)
    a, b = r["top_id"][:, 0], r["top_id"][:, 1]
    assert np.all(a != b)
    counts = np.zeros((V, V))
    np.add.at(counts, (a, b), 1)
    expect = np.outer(pr, pr) / (1.0 - pr)[:, None]
    np.fill_diagonal(expect, 0.0)
    off = ~np.eye(V, dtype=bool)
    chi2, crit = _chi2(counts[off], expect[off] * n)
    assert chi2 < crit, (chi2, crit)
    # with replacement (p_a p_b) would be rejected
    wr = np.outer(pr, pr)[off]
    assert _chi2(counts[off], wr / wr.sum() * n)[0] > crit

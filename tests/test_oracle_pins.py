"""Pins for the CPU oracle: everything here checks ``oracle/`` against something other than
itself -- published known answers, closed forms, library routines, an independent pure-Python
implementation, or brute force on tiny inputs.  No GPU, no product code.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import fs_workloads as wl
from tests import bruteforce as bf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
EULER_GAMMA = 0.5772156649015329


# ----------------------------------------------------------------------------- Philox

def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    assert len(rows) == 3
    return rows


@pytest.mark.parametrize("ctr,key,expect", _kat_rows())
def test_philox_known_answers(orc, ctr, key, expect):
    assert [int(v) for v in orc.philox4x32_10(ctr, key)] == expect
    assert bf.philox4x32_10(ctr, key) == expect          # the second implementation too


def test_philox_c_equals_python_on_random_counters(orc):
    rng = np.random.default_rng(7)
    for _ in range(300):
        ctr = [int(v) for v in rng.integers(0, 1 << 32, size=4)]
        key = [int(v) for v in rng.integers(0, 1 << 32, size=2)]
        assert [int(v) for v in orc.philox4x32_10(ctr, key)] == bf.philox4x32_10(ctr, key)


def test_philox_is_injective_on_a_counter_sweep(orc):
    # Philox is a bijection of the 128-bit counter for a fixed key: distinct counters
    # must give distinct 128-bit outputs.
    seen = set()
    for c0 in range(4096):
        out = orc.philox4x32_10([c0, c0 % 7, 0, 0], [123, 456])
        seen.add(tuple(int(v) for v in out))
    assert len(seen) == 4096


def test_random_word_counter_and_key_layout(orc):
    # counter = (vocab_id >> 2, row, 0, 0), key = (lo32(seed), hi32(seed)), word = vocab_id & 3
    seed = (0xDEADBEEF << 32) | 0x01234567
    for row, vid in [(0, 0), (0, 1), (0, 3), (0, 4), (5, 6), (17, 128255), (511, 152063),
                     (3, (1 << 31) + 5)]:
        block = orc.philox4x32_10([vid >> 2, row, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert orc.random_word(seed, row, vid) == int(block[vid & 3])
        assert orc.random_word(seed, row, vid) == bf.random_word(seed, row, vid)
    # four consecutive ids of one aligned group share one Philox block; the next group does not
    words = orc.random_words(seed, 9, 8, 8)
    assert [int(v) for v in words[:4]] == bf.philox4x32_10([2, 9, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
    assert [int(v) for v in words[4:]] == bf.philox4x32_10([3, 9, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])


def test_random_words_are_uniform(orc):
    n = 1 << 20
    words = orc.random_words(42, 3, 0, n)
    # chi-square on the top byte and on the low byte
    for shift in (24, 0):
        counts = np.bincount((words >> np.uint32(shift)) & np.uint32(0xFF), minlength=256)
        chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < stats.chi2.ppf(0.9999, 255)
    # rows and seeds give different streams
    assert not np.array_equal(words[:64], orc.random_words(42, 4, 0, 64))
    assert not np.array_equal(words[:64], orc.random_words(43, 3, 0, 64))


# ----------------------------------------------------------------------------- uniform, Gumbel

EDGE_WORDS = [0, 1, 2, 127, 128, 255, 256, (1 << 31) - 1, 1 << 31, (1 << 32) - 257,
              (1 << 32) - 129, (1 << 32) - 128, (1 << 32) - 2, (1 << 32) - 1]


def test_uniform_is_in_open_interval_and_matches_rational_model(orc):
    for r in EDGE_WORDS:
        x = orc.uniform_x(r)
        assert 0.0 < x < 1.0
        assert x == bf.uniform_x(r)
        assert np.float32(x) == x                    # an fp32 value
        assert 0.0 < 1.0 - x < 1.0                   # u strictly inside (0,1)
    assert orc.uniform_x(0) == 2.0 ** -33
    assert orc.uniform_x((1 << 32) - 1) == 1.0 - 2.0 ** -24
    rng = np.random.default_rng(11)
    rs = np.sort(rng.integers(0, 1 << 32, size=20000, dtype=np.uint64)).astype(np.uint32)
    g, x = orc.gumbel_from_words(rs)
    assert np.all(np.diff(x) >= 0)                   # monotone in r
    assert np.all(np.diff(g) <= 0)                   # u = 1 - x falls as r grows, and so does g
    for r in rs[::997]:
        assert orc.uniform_x(int(r)) == bf.uniform_x(int(r))
    # mid-point rule: x is (r + 1/2) / 2^32 up to the two fp32 roundings (of r, then of the fma)
    exact = (rs.astype(np.float64) + 0.5) / 2.0 ** 32
    assert np.all(np.abs(x.astype(np.float64) - exact) <= 2.0 ** -23 * np.maximum(exact, 2.0 ** -9))


def test_gumbel_is_finite_and_inverts_its_cdf(orc):
    words = np.array(EDGE_WORDS + list(np.random.default_rng(5).integers(0, 1 << 32, size=5000)),
                     dtype=np.uint32)
    g, x = orc.gumbel_from_words(words)
    assert np.all(np.isfinite(g))
    assert g.min() > -2.82 and g.max() < 22.95       # u in [2^-24, 1 - 2^-33]
    # The Gumbel(0,1) CDF is F(t) = exp(-exp(-t)); g = F^{-1}(u) with u = 1 - x, so F(g) = u.
    u = -np.expm1(-np.exp(-g))                       # = 1 - exp(-exp(-g)) = 1 - F(g) = x
    assert np.allclose(u, x.astype(np.float64), rtol=1e-12, atol=0)
    for r in EDGE_WORDS:
        assert math.isclose(orc.gumbel_from_word(r), bf.gumbel_from_word(r), rel_tol=1e-14)


def test_gumbel_moments_and_distribution(orc):
    n = 2_000_000
    g, _ = orc.gumbel_from_words(orc.random_words(2024, 0, 0, n))
    # mean = Euler gamma, variance = pi^2 / 6 (standard Gumbel)
    assert abs(g.mean() - EULER_GAMMA) < 5 * math.sqrt(math.pi ** 2 / 6 / n)
    assert abs(g.var() - math.pi ** 2 / 6) < 0.01
    ks = stats.kstest(g[:200_000], stats.gumbel_r.cdf)
    assert ks.pvalue > 1e-3


# ----------------------------------------------------------------------------- logits

def test_logits_equal_a_library_matmul(orc):
    import torch
    H, W = wl.make_small(D=192, V=333, B=5, data_seed=31)
    Y = orc.logits(H, W)
    Hf = torch.from_numpy(wl.bf16_bits_to_f32(H)).double()
    Wf = torch.from_numpy(wl.bf16_bits_to_f32(W)).double()
    ref = (Hf @ Wf.T).numpy()
    assert np.allclose(Y, ref, rtol=0, atol=1e-12)
    assert Y.shape == (5, 333)
    # a transposed operand or a swapped index would be caught by the asymmetric shape above;
    # single-element entry point agrees with the bulk one
    assert orc.logit(H, W, 3, 17) == Y[3, 17]


def test_logits_equal_exact_rational_dot_products(orc):
    H, W = wl.make_small(D=24, V=9, B=2, data_seed=32)
    Y = orc.logits(H, W)
    for b in range(2):
        for i in range(9):
            assert math.isclose(Y[b, i], bf.logit(H[b], W[i]), rel_tol=1e-13, abs_tol=1e-15)


# ----------------------------------------------------------------------------- sampling law

def _chi2_ok(counts, p, n, q=0.999):
    exp = p * n
    order = np.argsort(exp)
    # pool the smallest cells until every expected count is >= 5
    e_sorted, c_sorted = exp[order], counts[order]
    cells_e, cells_c, acc_e, acc_c = [], [], 0.0, 0
    for e, c in zip(e_sorted, c_sorted):
        acc_e += e
        acc_c += c
        if acc_e >= 5:
            cells_e.append(acc_e)
            cells_c.append(acc_c)
            acc_e, acc_c = 0.0, 0
    if acc_e > 0:
        cells_e[-1] += acc_e
        cells_c[-1] += acc_c
    cells_e, cells_c = np.array(cells_e), np.array(cells_c)
    chi2 = ((cells_c - cells_e) ** 2 / cells_e).sum()
    return chi2, stats.chi2.ppf(q, len(cells_e) - 1)


def _np_softmax(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


@pytest.mark.parametrize("tau", [1.0, 0.5, 2.0])
def test_chi_square_against_brute_force_softmax(orc, tau):
    # 10^6 seeded draws on a tiny vocabulary vs brute-force softmax probabilities
    # (the paper's kernel-level check uses V=512 and 10^4 draws; same test, more draws).
    rng = np.random.default_rng(100)
    y = rng.normal(0, 1.5, size=64)
    p = _np_softmax(y / tau)
    n = 1_000_000
    counts = orc.draw_counts(y, tau, seed=1234, ndraws=n, by_row=True)
    assert counts.sum() == n
    chi2, crit = _chi2_ok(counts, p, n)
    assert chi2 < crit, (chi2, crit)
    # the oracle's own softmax helper is the same brute force
    p2, lse = orc.softmax(y, tau)
    assert np.allclose(p2, p, rtol=1e-12)
    assert math.isclose(lse, float(np.log(np.exp(y / tau).sum())), rel_tol=1e-12)


def test_chi_square_over_seeds_v512(orc):
    # draws indexed by seed instead of by row, V = 512 as in the paper's check
    rng = np.random.default_rng(101)
    y = rng.normal(0, 2.0, size=512)
    p = _np_softmax(y)
    n = 300_000
    counts = orc.draw_counts(y, 1.0, seed=10_000, ndraws=n, by_row=False)
    chi2, crit = _chi2_ok(counts, p, n)
    assert chi2 < crit, (chi2, crit)


def test_wrong_distribution_is_rejected_by_the_same_chi_square(orc):
    # sensitivity of the pin: the same counts tested against softmax(y / 1.15) must fail
    rng = np.random.default_rng(100)
    y = rng.normal(0, 1.5, size=64)
    n = 1_000_000
    counts = orc.draw_counts(y, 1.0, seed=1234, ndraws=n, by_row=True)
    chi2, crit = _chi2_ok(counts, _np_softmax(y / 1.15), n)
    assert chi2 > 10 * crit


def test_max_value_is_gumbel_with_location_lse(orc):
    # Lemma "Gumbel max-stability under grouping": max_i (l_i + g_i) ~ Gumbel(lse(l), 1)
    rng = np.random.default_rng(102)
    y = rng.normal(0, 1.0, size=200)
    tau = 0.8
    n = 200_000
    _, vals = orc.draw_counts(y, tau, seed=77, ndraws=n, by_row=True, return_vals=True)
    lse = float(np.log(np.exp(y / tau).sum()))
    d = vals - lse
    assert abs(d.mean() - EULER_GAMMA) < 5 * math.sqrt(math.pi ** 2 / 6 / n)
    assert abs(d.var() - math.pi ** 2 / 6) < 0.03
    assert stats.kstest(d, stats.gumbel_r.cdf).pvalue > 1e-3


def test_two_categories_follow_the_logistic_law(orc):
    # P(0) = sigmoid(z0 - z1)
    y = np.array([0.3, -0.9])
    n = 400_000
    counts = orc.draw_counts(y, 1.0, seed=5, ndraws=n, by_row=True)
    p0 = 1.0 / (1.0 + math.exp(-(y[0] - y[1])))
    sd = math.sqrt(p0 * (1 - p0) / n)
    assert abs(counts[0] / n - p0) < 4.5 * sd


def test_temperature_limits(orc):
    rng = np.random.default_rng(103)
    y = rng.normal(0, 1.0, size=300)
    # tau -> 0: plain argmax (top-two raw gap far above 26 * tau)
    srt = np.sort(y)
    assert srt[-1] - srt[-2] > 26 * 1e-4
    for row in range(50):
        i1, _, _, _ = orc.gumbel_max_row(y, 1e-4, seed=9, row=row)
        assert i1 == int(np.argmax(y))
    # tau -> infinity: uniform
    n = 300_000
    counts = orc.draw_counts(y, 1e9, seed=6, ndraws=n, by_row=True)
    chi2, crit = _chi2_ok(counts, np.full(300, 1 / 300), n)
    assert chi2 < crit


def test_special_cases(orc):
    # V = 1
    assert orc.gumbel_max_row(np.array([0.123]), 1.0, 0, 0)[0] == 0
    # one logit far above the rest always wins (gap 40 >> the 25.8 range of g)
    y = np.zeros(1000)
    y[777] = 40.0
    for row in range(200):
        assert orc.gumbel_max_row(y, 1.0, 3, row)[0] == 777
    # -inf entries never win; NaN never wins; a row with nothing finite gives idx -1, val -inf
    y = np.full(16, -np.inf)
    y[5] = 0.0
    assert orc.gumbel_max_row(y, 1.0, 0, 0)[0] == 5
    y2 = np.full(16, np.nan)
    y2[9] = -3.0
    assert orc.gumbel_max_row(y2, 1.0, 0, 0)[0] == 9
    i1, m1, i2, m2 = orc.gumbel_max_row(np.full(4, -np.inf), 1.0, 0, 0)
    assert i1 == -1 and m1 == -np.inf and i2 == -1
    # exact ties go to the lowest index: identical huge logits, noise rounded away
    y3 = np.full(8, 1e300)
    assert orc.gumbel_max_row(y3, 1.0, 0, 0)[0] == 0
    # runner-up bookkeeping
    y4 = np.array([0.0, 100.0, 50.0, -5.0])
    i1, m1, i2, m2 = orc.gumbel_max_row(y4, 1.0, 0, 0)
    assert (i1, i2) == (1, 2) and m1 > m2


# ----------------------------------------------------------------------------- full path

def test_full_path_equals_pure_python_brute_force(orc):
    H, W = wl.make_small(D=16, V=45, B=3, data_seed=33)
    tau = np.array([1.0, 0.6, 1.7], dtype=np.float32)
    seeds = np.array([11, (7 << 32) + 5, 13], dtype=np.uint64)
    r = orc.sample(H, W, tau, row_seeds=seeds, row_offset=4, vocab_offset=1000)
    for b in range(3):
        i1, m1, scores = bf.sample_row(H[b], W, float(tau[b]), int(seeds[b]), 4 + b, 1000)
        assert r["idx"][b] == i1
        assert math.isclose(r["top1"][b], m1, rel_tol=1e-12)
        assert r["val"][b] == np.float32(m1)
        second = sorted(scores)[-2]
        assert math.isclose(r["top2"][b], second, rel_tol=1e-12)
        # single-score entry point
        s = orc.score_at(H, W, b, 7, float(tau[b]), int(seeds[b]), 4 + b, 1007)
        assert math.isclose(s, scores[7], rel_tol=1e-12)


def test_full_path_composes_logits_and_row_sampler(orc):
    H, W = wl.make_small(D=64, V=700, B=4, data_seed=34)
    tau = np.array([0.7, 1.0, 1.3, 2.0], dtype=np.float32)
    Y = orc.logits(H, W)
    r = orc.sample(H, W, tau, seed=99)
    for b in range(4):
        i1, m1, i2, m2 = orc.gumbel_max_row(Y[b], float(tau[b]), 99, b)
        assert (r["idx"][b], r["idx2"][b]) == (i1, i2)
        assert (r["top1"][b], r["top2"][b]) == (m1, m2)
    # and the sampled index is the argmax of z + g assembled from the vectorised pieces
    for b in range(4):
        g, _ = orc.gumbel_from_words(orc.random_words(99, b, 0, 700))
        s = Y[b] / np.float64(tau[b]) + g
        assert r["idx"][b] == int(np.argmax(s))


def test_tile_partition_invariance(orc):
    # Lemma "Max over vocabulary tiles": the result is the same for every tile size,
    # including ragged last tiles and tiles of one element.
    H, W = wl.make_small(D=32, V=257, B=3, data_seed=35)
    tau = np.array([1.0, 0.5, 1.5], dtype=np.float32)
    full = orc.sample(H, W, tau, seed=2)
    for tile in list(range(1, 40)) + [64, 100, 128, 129, 256, 257, 300]:
        t = orc.sample_tiled(H, W, tau, tile, seed=2)
        assert np.array_equal(t["idx"], full["idx"]), tile
        assert np.array_equal(t["val"], full["val"]), tile
        T = (257 + tile - 1) // tile
        assert t["cand_idx"].shape == (3, T)
        lo = np.arange(T) * tile
        assert np.all(t["cand_idx"] >= lo[None, :]) and np.all(t["cand_idx"] < lo[None, :] + tile)


def test_vocab_and_row_sharding_reproduce_the_unsharded_sample(orc):
    H, W = wl.make_small(D=32, V=300, B=6, data_seed=36)
    tau = np.full(6, 0.9, dtype=np.float32)
    full = orc.sample(H, W, tau, seed=8)
    # vocabulary shards with global ids
    best_v = np.full(6, -np.inf)
    best_i = np.full(6, -1)
    for lo, hi in [(0, 100), (100, 228), (228, 300)]:
        r = orc.sample(H, W[lo:hi].copy(), tau, seed=8, vocab_offset=lo)
        upd = r["top1"] > best_v
        best_v = np.where(upd, r["top1"], best_v)
        best_i = np.where(upd, r["idx"], best_i)
    assert np.array_equal(best_i, full["idx"])
    # row shards via row_offset and via explicit row ids
    r2 = orc.sample(H[2:5].copy(), W, tau[2:5], seed=8, row_offset=2)
    assert np.array_equal(r2["idx"], full["idx"][2:5])
    rows = np.array([5, 0, 3], dtype=np.int64)
    r3 = orc.sample(H[rows].copy(), W, tau[rows], seed=8, row_ids=rows)
    assert np.array_equal(r3["idx"], full["idx"][rows])


def test_per_row_seeds_equal_single_seed_calls(orc):
    H, W = wl.make_small(D=32, V=200, B=4, data_seed=37)
    tau = np.ones(4, dtype=np.float32)
    seeds = np.array([0, 1, 2, 3], dtype=np.uint64)
    r = orc.sample(H, W, tau, row_seeds=seeds)
    for b in range(4):
        one = orc.sample(H[b:b + 1].copy(), W, tau[b:b + 1], seed=int(seeds[b]), row_offset=b)
        assert one["idx"][0] == r["idx"][b]


def test_config_c1_runs_and_is_deterministic(orc):
    c1 = wl.WORKLOADS["C1"]
    H, W = wl.make_hidden(c1, 1), wl.make_weights(c1)
    assert H.shape == (1, 256) and W.shape == (4096, 256)
    a = orc.sample(H, W, wl.make_temperature(c1, 1), seed=c1.seed)
    b = orc.sample(H, W, wl.make_temperature(c1, 1), seed=c1.seed)
    assert a["idx"][0] == b["idx"][0] and 0 <= a["idx"][0] < 4096
    t = orc.sample_tiled(H, W, wl.make_temperature(c1, 1), c1.vocab_tile, seed=c1.seed)
    assert t["cand_val"].shape == (1, 32) and t["idx"][0] == a["idx"][0]

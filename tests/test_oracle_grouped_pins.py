"""Pins for the oracle's grouped variants (parallel and online Group-Gumbel-Max): the group
factorisation and binary-merge lemmas as closed forms, the sampling law by chi-square against a
softmax written out here, special cases that reduce to the already pinned plain sampler, and a
pure-Python replay of both group choices on a tiny input.  No GPU."""
import math

import numpy as np
from scipy import special

import fs_workloads as wl
from tests import bruteforce as bf
from tests.test_oracle_pins import _chi2_ok

PAR, ONL = 0, 1


def _row(V=40, seed=300, masked=()):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 1.7, size=V)
    for lo, hi in masked:
        z[lo:hi] = -np.inf
    return z


def _softmax(z):
    e = np.exp(z - z[np.isfinite(z)].max())
    return e / e.sum()


def test_group_words_use_their_own_philox_stream(orc):
    seed, row = 0x1234_5678_9ABC_DEF0, 77
    for k in (0, 1, 2, 3, 4, 5, 1001, (1 << 20) + 3):
        # stream 0 is the per-id noise of the main path (already pinned by the known-answer test)
        assert orc.group_word(seed, row, k, 0) == orc.random_word(seed, row, k)
        for stream in (1, 2):
            ref = bf.philox4x32_10([k >> 2, row, stream, 0], [seed & bf.M32, seed >> 32])[k & 3]
            assert orc.group_word(seed, row, k, stream) == ref
    words = {orc.group_word(seed, row, 5, s) for s in (0, 1, 2)}
    assert len(words) == 3


def test_group_log_masses_factorise_the_softmax(orc):
    # Lemma "Exact group factorization": P(K=k) P(I=i | K=k) = softmax_i, groups of unequal size
    z = _row(V=23, masked=[(8, 12)])            # group 2 (ids 8..11) has zero mass
    g = 4                                        # last group has 3 ids
    st = orc.group_stats(z, g, seed=1, row=0)
    m = (z.size + g - 1) // g
    assert st["L"].shape == (m,)
    p = _softmax(z)
    lse = special.logsumexp(z)
    for k in range(m):
        ids = np.arange(k * g, min(z.size, (k + 1) * g))
        if k == 2:
            assert st["L"][k] == -np.inf and st["zk"][k] == -1
            continue
        assert math.isclose(st["L"][k], special.logsumexp(z[ids]), rel_tol=1e-13)
        pk = math.exp(st["L"][k] - lse)
        assert math.isclose(pk, p[ids].sum(), rel_tol=1e-12)
        within = np.exp(z[ids] - st["L"][k])
        assert np.allclose(pk * within, p[ids], rtol=1e-12)
    assert math.isclose(orc.log_sum_exp(st["L"]), lse, rel_tol=1e-13)


def test_local_samples_are_the_plain_sampler_restricted_to_the_group(orc):
    z = _row(V=50, seed=301)
    g, seed, row, voff = 16, 9, 4, 64
    st = orc.group_stats(z, g, seed=seed, row=row, vocab_offset=voff)
    for k in range(4):
        lo, hi = k * g, min(50, (k + 1) * g)
        i1, m1, i2, m2 = orc.gumbel_max_transformed(z[lo:hi], seed, row, vocab_offset=voff + lo)
        assert (st["zk"][k], st["s1"][k], st["s2"][k]) == (i1, m1, m2)
    # pathwise: the best local sample over all groups is the plain sampler's pick (tile-max lemma)
    i_all, m_all, _, _ = orc.gumbel_max_transformed(z, seed, row, vocab_offset=voff)
    kbest = int(np.argmax(st["s1"]))
    assert st["zk"][kbest] == i_all and st["s1"][kbest] == m_all


def test_one_group_reduces_to_the_plain_sampler(orc):
    z = _row(V=37, seed=302, masked=[(3, 9)])
    for mode in (PAR, ONL):
        for row in range(50):
            i1, _, _, _ = orc.gumbel_max_transformed(z, 5, row)
            counts = orc.grouped_draw_counts(z, 37, mode, seed=5, ndraws=1, row0=row)
            assert counts[i1] == 1 and counts.sum() == 1


def test_parallel_choice_replayed_in_pure_python(orc):
    seed, row, goff = 42, 6, 8
    L = np.array([0.3, -np.inf, 1.9, 0.1, 2.2, -0.7])
    k, score = orc.group_choose_parallel(L, seed, row, group_offset=goff)
    ref = []
    for j, Lj in enumerate(L):
        if Lj == -np.inf:
            ref.append(-math.inf)
            continue
        kk = goff + j
        r = bf.philox4x32_10([kk >> 2, row, 1, 0], [seed, 0])[kk & 3]
        ref.append(Lj + bf.gumbel_from_word(r))
    assert np.allclose(score, ref, rtol=1e-14)
    assert k == max(range(len(ref)), key=lambda j: (ref[j], -j))
    assert score[1] == -np.inf
    assert orc.group_choose_parallel(np.full(5, -np.inf), seed, row)[0] == -1


def test_online_choice_replayed_in_pure_python(orc):
    seed, goff = 43, 4
    L = np.array([-np.inf, 0.3, 1.9, -np.inf, 0.1, 2.2, -0.7])
    replaced_late = 0
    for row in range(200):
        k, u, p, lse = orc.group_choose_online(L, seed, row, group_offset=goff)
        mass, kref = 0.0, -1
        for j, Lj in enumerate(L):
            if Lj == -np.inf:
                assert math.isnan(u[j]) and math.isnan(p[j])
                continue
            kk = goff + j
            r = bf.philox4x32_10([kk >> 2, row, 2, 0], [seed, 0])[kk & 3]
            uj = bf.uniform_x(r)
            mass_new = mass + math.exp(Lj)
            pj = math.exp(Lj) / mass_new           # the merge rule as a plain ratio of masses
            assert uj == u[j] and math.isclose(pj, p[j], rel_tol=1e-12)
            if uj < pj:
                kref = j
            mass = mass_new
        assert k == kref
        assert math.isclose(lse, math.log(mass), rel_tol=1e-13)
        assert p[1] == 1.0                          # first nonzero-mass group initialises the state
        replaced_late += k > 1
    assert replaced_late > 100                      # later groups do take over
    k, _, _, lse = orc.group_choose_online(np.full(4, -np.inf), seed, 0)
    assert k == -1 and lse == -np.inf


def test_binary_merge_probability(orc):
    # Lemma "binary merge": with two groups the second one wins with e^L1 / (e^L0 + e^L1)
    z = np.array([0.4, -0.9])                       # groups of one id: L_k = z_k
    n = 200_000
    counts = orc.grouped_draw_counts(z, 1, ONL, seed=11, ndraws=n)
    p1 = math.exp(-0.9) / (math.exp(0.4) + math.exp(-0.9))
    sd = math.sqrt(n * p1 * (1 - p1))
    assert counts.sum() == n and abs(counts[1] - n * p1) < 4.5 * sd


def test_both_variants_sample_the_softmax(orc):
    n = 400_000
    z = _row(V=61, seed=303, masked=[(16, 24), (40, 43)])      # one whole zero-mass group at g = 8
    p = _softmax(z)
    for mode in (PAR, ONL):
        for g in (1, 8, 7, 61, 100):
            counts = orc.grouped_draw_counts(z, g, mode, seed=1000 + g, ndraws=n)
            assert counts.sum() == n
            assert counts[~np.isfinite(z)].sum() == 0
            chi2, crit = _chi2_ok(counts, p, n)
            assert chi2 < crit, (mode, g, chi2, crit)


def test_the_law_test_has_teeth(orc):
    # A planted mistake (CPU only): feeding the online chooser log-masses with the wrong sign of
    # the exponent, i.e. replacing with probability e^{-L_k} / sum, must fail the same chi-square.
    n = 100_000
    z = _row(V=16, seed=304)
    p = _softmax(z)
    counts = np.zeros(16, dtype=np.int64)
    for row in range(0, n, 50):                      # 2000 draws are plenty for a gross error
        st = orc.group_stats(z, 4, seed=21, row=row)
        k, _, _, _ = orc.group_choose_online(-st["L"], 21, row)
        counts[st["zk"][k]] += 1
    chi2, crit = _chi2_ok(counts, p, counts.sum())
    assert chi2 > crit


def test_full_grouped_path_on_a_small_problem(orc):
    H, W = wl.make_small(D=64, V=300, B=6, data_seed=77)
    tau = np.array([0.5, 1.0, 1.5, 0.8, 1.0, 2.0], dtype=np.float32)
    rng = np.random.default_rng(5)
    bias = rng.normal(0, 1, 300).astype(np.float32)
    allowed = rng.random((6, 300)) < 0.7
    allowed[3, :] = False                                       # a row with no mass at all
    allowed[4, 128:256] = False                                 # a zero-mass group at g = 128
    aw = orc.pack_allowed(allowed)
    full = orc.sample_full(H, W, tau, seed=3, bias=bias, allowed_words=aw)
    for mode in (PAR, ONL):
        r = orc.sample_grouped(H, W, tau, 128, mode, seed=3, bias=bias, allowed_words=aw)
        assert r["zk"].shape == (6, 3)
        assert r["idx"][3] == -1 and r["lse"][3] == -np.inf
        assert r["zk"][4, 1] == -1 and r["L"][4, 1] == -np.inf
        ok = [0, 1, 2, 4, 5]
        assert np.allclose(r["lse"][ok], full["lse"][ok], rtol=1e-13)
        for b in ok:
            assert allowed[b, r["idx"][b]]
            assert r["idx"][b] in r["zk"][b]
            # the main path's pick is the local sample of the group with the best local score
            kbest = int(np.argmax(r["s1"][b]))
            assert r["zk"][b, kbest] == full["idx"][b]

"""Pins for the CPU oracle: each check uses something other than the oracle itself.

Published known-answer vectors, exact rational arithmetic, NumPy's stable argsort as brute
force, the dense special case of the update rule, conservation and hand-built cases.  A wrong
sign, index, operand order, tie rule or dropped term in ``oracle/slimdp_oracle.c`` fails at
least one of these.  No GPU is needed.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------------------
# helpers that do exact arithmetic (not the oracle's formula retyped in binary32)
# ----------------------------------------------------------------------------------------
def f32_exact(x: np.float32) -> Fraction:
    return Fraction(float(np.float32(x)))


def round_to_f32(q: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 of an exact rational."""
    approx = np.float32(float(q))
    cands = {approx, np.nextafter(approx, np.float32(np.inf)), np.nextafter(approx, np.float32(-np.inf))}
    best = None
    for c in cands:
        if not np.isfinite(c):
            continue
        err = abs(Fraction(float(c)) - q)
        even = (int(np.float32(c).view(np.uint32)) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, c)
    return np.float32(best[1])


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


# ----------------------------------------------------------------------------------------
# Philox4x32-10
# ----------------------------------------------------------------------------------------
def _kat():
    rows = []
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == out


def test_philox_is_a_bijection_on_a_counter_range():
    seen = set()
    for c0 in range(64):
        for c1 in range(8):
            out = tuple(int(x) for x in oracle.philox4x32_10([c0, c1, 0, 0], [5, 9]))
            seen.add(out)
    assert len(seen) == 64 * 8


def test_explore_word_counter_layout_matches_known_answer():
    # counter = (i div 4, worker, iteration low, iteration high), key = (seed low, seed high),
    # word = i mod 4: feed the third known-answer vector through that layout.
    ctr, key, out = _kat()[2]
    seed = key[0] | (key[1] << 32)
    iteration = ctr[2] | (ctr[3] << 32)
    worker = ctr[1]
    i0 = ctr[0] << 2
    assert i0 < 2 ** 32
    words = oracle.explore_words(seed, iteration, worker, i0, 4)
    assert [int(x) for x in words] == out
    # unaligned start: words continue into the next block
    w2 = oracle.explore_words(seed, iteration, worker, i0 + 2, 4)
    nxt = oracle.philox4x32_10([ctr[0] + 1, ctr[1], ctr[2], ctr[3]], key)
    assert [int(x) for x in w2] == [out[2], out[3], int(nxt[0]), int(nxt[1])]


def test_explore_words_are_uniform_bits():
    words = oracle.explore_words(0, 3, 1, 0, 1 << 16)
    ones = np.unpackbits(words.view(np.uint8)).reshape(-1, 8).sum()
    total = words.size * 32
    assert abs(ones / total - 0.5) < 0.005
    # top byte histogram, chi-square with 255 dof: mean 255, sd ~22.6
    h = np.bincount(words >> 24, minlength=256)
    chi2 = ((h - words.size / 256) ** 2 / (words.size / 256)).sum()
    assert chi2 < 255 + 6 * 22.6


# ----------------------------------------------------------------------------------------
# Significance, equation (1)
# ----------------------------------------------------------------------------------------
def test_score_exact_rational_closed_form():
    rng = np.random.default_rng(11)
    n, W = 257, 3
    w = rng.standard_normal(n).astype(np.float32)
    g = [rng.standard_normal(n).astype(np.float32) * np.float32(1e-2) for _ in range(W)]
    c = np.float32(1.0 + 2.0 ** -12)          # makes c*|g| inexact so fused != unfused
    S = oracle.score(w, g, float(c))
    n_fused_differs = 0
    for i in range(n):
        gi = g[0][i]
        for k in range(1, W):                 # binary32 adds in worker order, each correctly rounded
            gi = round_to_f32(f32_exact(gi) + f32_exact(g[k][i]))
        exact = abs(f32_exact(w[i])) + f32_exact(c) * abs(f32_exact(gi))
        want = round_to_f32(exact)
        assert bits(S[i:i + 1])[0] == bits(np.array([want]))[0], i
        unfused = np.float32(np.float32(c * np.abs(gi)) + np.abs(w[i]))
        n_fused_differs += int(unfused != want)
    assert n_fused_differs > 0                # the test can tell one rounding from two


def test_score_sums_workers_left_to_right():
    w = np.zeros(1, np.float32)
    g = [np.array([1e8], np.float32), np.array([-1e8], np.float32), np.array([1.0], np.float32)]
    assert oracle.score(w, g, 1.0)[0] == np.float32(1.0)       # (1e8 + -1e8) + 1
    g2 = [g[0], g[2], g[1]]
    assert oracle.score(w, g2, 1.0)[0] == np.float32(0.0)      # (1e8 + 1) + -1e8
    # magnitude of the summed update, not the sum of magnitudes
    g3 = [np.array([2.0], np.float32), np.array([-2.0], np.float32)]
    assert oracle.score(np.array([0.5], np.float32), g3, 1.0)[0] == np.float32(0.5)


def test_score_special_cases():
    rng = np.random.default_rng(5)
    w = rng.standard_normal(1000).astype(np.float32)
    g = rng.standard_normal(1000).astype(np.float32)
    # c = 0: magnitude pruning, S = |w|
    assert np.array_equal(bits(oracle.score(w, [g], 0.0)), bits(np.abs(w)))
    # w = 0, c = 1: S = |g| ; W = 1
    assert np.array_equal(bits(oracle.score(np.zeros_like(w), [g], 1.0)), bits(np.abs(g)))
    # signs do not matter
    assert np.array_equal(bits(oracle.score(-w, [-g], 1.5)), bits(oracle.score(w, [g], 1.5)))
    # never negative, never -0
    assert (bits(oracle.score(w, [g], 1.5)) >> 31).max() == 0
    assert bits(oracle.score(np.array([-0.0], np.float32), [np.array([-0.0], np.float32)], 1.0))[0] == 0
    # NaN in, canonical quiet NaN out; infinity stays infinity
    s = oracle.score(np.array([np.nan, np.inf, 1.0], np.float32),
                     [np.array([0.0, 0.0, -np.nan], np.float32)], 1.0)
    assert list(bits(s)) == [0x7FC00000, 0x7F800000, 0x7FC00000]


# ----------------------------------------------------------------------------------------
# Core selection
# ----------------------------------------------------------------------------------------
def brute_topk(S, base, ln, k):
    key = bits(S[base:base + ln]).astype(np.int64)
    order = np.argsort(-key, kind="stable")      # key descending, position ascending on ties
    return np.sort(order[:k] + base).astype(np.uint32)


@pytest.mark.parametrize("n,k,levels", [(1, 1, 0), (10, 3, 0), (1000, 100, 0), (4097, 410, 0),
                                        (10000, 1000, 7), (10000, 9999, 3), (5000, 2500, 2)])
def test_select_core_matches_stable_argsort(n, k, levels):
    rng = np.random.default_rng(n + k)
    S = np.abs(rng.standard_normal(n)).astype(np.float32)
    if levels:                                    # few distinct values: many ties
        S = (np.floor(S * levels) / levels).astype(np.float32)
    got = oracle.select_core(S, k)
    assert np.array_equal(got, brute_topk(S, 0, n, k))
    # invariants: size, ascending and distinct, threshold property, tie rule
    assert got.size == k and np.all(np.diff(got.astype(np.int64)) > 0)
    if 0 < k < n:
        mask = np.zeros(n, bool)
        mask[got] = True
        tau = S[mask].min()
        assert tau >= S[~mask].max()
        tie_in = np.flatnonzero(mask & (S == tau))
        tie_out = np.flatnonzero(~mask & (S == tau))
        if tie_in.size and tie_out.size:
            assert tie_in.max() < tie_out.min()


def test_select_core_edges():
    S = np.full(100, 0.25, np.float32)
    assert np.array_equal(oracle.select_core(S, 7), np.arange(7, dtype=np.uint32))   # all equal
    assert oracle.select_core(S, 0).size == 0
    assert np.array_equal(oracle.select_core(S, 100), np.arange(100, dtype=np.uint32))
    # descending means LARGEST first
    S2 = np.arange(10, dtype=np.float32)
    assert list(oracle.select_core(S2, 3)) == [7, 8, 9]
    # NaN above infinity above finite (bit-pattern order)
    S3 = np.array([1.0, np.inf, 3.0, np.nan, 2.0], np.float32)
    S3[3] = np.array([0x7FC00000], np.uint32).view(np.float32)[0]
    assert list(oracle.select_core(S3, 2)) == [1, 3]
    with pytest.raises(ValueError):
        oracle.select_core(S2, 11)


def test_select_core_segmented():
    rng = np.random.default_rng(3)
    S = np.abs(rng.standard_normal(3000)).astype(np.float32)
    S = (np.floor(S * 20) / 20).astype(np.float32)
    off = [0, 17, 1000, 1001, 3000]
    ks = [5, 98, 1, 0]
    got = oracle.select_core(S, ks, off)
    want = np.concatenate([brute_topk(S, off[s], off[s + 1] - off[s], ks[s]) for s in range(4)])
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------------------
# Exploration
# ----------------------------------------------------------------------------------------
def brute_explore(n, core_idx, seed, t, worker, m, base=0, ln=None):
    ln = n - base if ln is None else ln
    r = oracle.explore_words(seed, t, worker, 0, n)          # words pinned by the tests above
    mask = np.zeros(n, bool)
    mask[core_idx] = True
    rest = np.array([i for i in range(base, base + ln) if not mask[i]], dtype=np.int64)
    order = np.argsort(r[rest].astype(np.int64), kind="stable")   # word asc, index asc on ties
    return np.sort(rest[order[:m]]).astype(np.uint32)


@pytest.mark.parametrize("n,k,m", [(100, 10, 5), (1000, 100, 18), (4099, 409, 73), (64, 0, 64),
                                   (64, 64, 0), (50, 10, 40)])
def test_sample_explore_matches_brute_force(n, k, m):
    rng = np.random.default_rng(n)
    core = np.sort(rng.choice(n, size=k, replace=False)).astype(np.uint32)
    for worker, t in [(0, 0), (3, 0), (0, 7), (2, 2 ** 33 + 5)]:
        got = oracle.sample_explore(n, core, 1234, t, worker, m)
        assert np.array_equal(got, brute_explore(n, core, 1234, t, worker, m))
        assert got.size == m and np.all(np.diff(got.astype(np.int64)) > 0)
        assert np.intersect1d(got, core).size == 0


def test_sample_explore_ties_take_lower_index():
    # Equal 32-bit words do occur among 2^20 draws (about n^2 / 2^33 = 128 pairs).  Take one
    # such pair i < j with word v and ask for exactly (number of words below v) + 1 indices:
    # the set must then contain i and not j.
    n = 1 << 20
    r = oracle.explore_words(9, 0, 0, 0, n)
    order = np.argsort(r, kind="stable")
    rs = r[order]
    dup = np.flatnonzero(rs[1:] == rs[:-1])
    assert dup.size > 0
    core = np.zeros(0, np.uint32)
    for d in dup[:3]:
        v = rs[d]
        tied = np.sort(order[rs == v])
        below = int((r < v).sum())
        got = oracle.sample_explore(n, core, 9, 0, 0, below + 1)
        assert tied[0] in got and tied[1] not in got
        assert np.all(r[got] <= v)


def test_sample_explore_depends_on_worker_iteration_seed():
    n, k, m = 5000, 500, 90
    core = np.arange(0, n, 10, dtype=np.uint32)[:k]
    a = oracle.sample_explore(n, core, 0, 0, 0, m)
    assert np.array_equal(a, oracle.sample_explore(n, core, 0, 0, 0, m))
    assert not np.array_equal(a, oracle.sample_explore(n, core, 0, 0, 1, m))
    assert not np.array_equal(a, oracle.sample_explore(n, core, 0, 1, 0, m))
    assert not np.array_equal(a, oracle.sample_explore(n, core, 1, 0, 0, m))
    with pytest.raises(ValueError):
        oracle.sample_explore(n, core, 0, 0, 0, n - k + 1)


def test_sample_explore_is_uniform_over_the_complement():
    n, k, m, T = 400, 40, 36, 1500
    core = np.arange(0, n, 10, dtype=np.uint32)
    hits = np.zeros(n)
    for t in range(T):
        hits[oracle.sample_explore(n, core, 77, t, 1, m)] += 1
    assert hits[core].sum() == 0
    rest = np.setdiff1d(np.arange(n), core)
    p = m / (n - k)
    expect = T * p
    z = (hits[rest] - expect) / np.sqrt(T * p * (1 - p))
    assert np.abs(z).max() < 5.0
    # no dependence on position: first and second half of the index range hit equally often
    half = rest.size // 2
    assert abs(hits[rest[:half]].sum() - hits[rest[half:]].sum()) < 6 * np.sqrt(T * m)


def test_sample_explore_segmented():
    n = 3000
    off = [0, 17, 1000, 1001, 3000]
    core = oracle.select_core(np.abs(np.random.default_rng(1).standard_normal(n)).astype(np.float32),
                              [2, 98, 0, 200], off)
    ms = [3, 17, 1, 36]
    got = oracle.sample_explore(n, core, 5, 4, 2, ms, off)
    want = np.concatenate([brute_explore(n, core, 5, 4, 2, ms[s], off[s], off[s + 1] - off[s])
                           for s in range(4)])
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------------------
# Pack / wire size
# ----------------------------------------------------------------------------------------
def test_pack_is_a_bit_copy():
    rng = np.random.default_rng(2)
    g = rng.standard_normal(1000).astype(np.float32)
    g[5] = -0.0
    g[6] = np.array([0x7FA00001], np.uint32).view(np.float32)[0]     # signalling NaN payload
    core = np.array([0, 5, 6, 999], np.uint32)
    expl = np.array([1, 7, 500], np.uint32)
    cv, ev = oracle.pack(g, core, expl)
    assert np.array_equal(bits(cv), bits(g)[core]) and np.array_equal(bits(ev), bits(g)[expl])


def test_wire_words_formula_against_table_1():
    # section 3.5: core costs beta*n words (cached keys), explorer 2(alpha-beta)n, total
    # (2 alpha - beta) n.  With k = beta n and m = (alpha - beta) n the pack above holds
    # k + 2m words.  Table 1's measured Slim/Plump ratios agree with that count.
    for line in open(os.path.join(GOLDEN, "paper_table1_comm_hours.txt")):
        if line.startswith("#") or not line.strip():
            continue
        model, K, alpha, beta, plump, slim = line.split()
        alpha, beta, plump, slim = float(alpha), float(beta), float(plump), float(slim)
        n = 1_000_000
        k, m = round(beta * n), round((alpha - beta) * n)
        assert k + 2 * m == round((2 * alpha - beta) * n)
        assert abs(slim / plump - (k + 2 * m) / n) < 0.03, (model, K)


# ----------------------------------------------------------------------------------------
# Merge (server update)
# ----------------------------------------------------------------------------------------
def test_merge_dense_special_case_is_plump_dp():
    # k = n, m = 0: every worker sends everything; values chosen dyadic so that every
    # operation is exact and the NumPy expression w - lr * sum_k g_k has no rounding at all.
    rng = np.random.default_rng(8)
    n, W = 513, 4
    w = (rng.integers(-1024, 1024, n) / 64.0).astype(np.float32)
    g = [(rng.integers(-256, 256, n) / 16.0).astype(np.float32) for _ in range(W)]
    lr = 0.25
    core = np.arange(n, dtype=np.uint32)
    empty_i = [np.zeros(0, np.uint32)] * W
    empty_v = [np.zeros(0, np.float32)] * W
    got = oracle.merge(w, lr, core, g, empty_i, empty_v)
    want = w.astype(np.float64) - lr * np.sum(np.stack(g).astype(np.float64), axis=0)
    assert np.array_equal(got.astype(np.float64), want)


def test_merge_hand_built_collisions_and_order():
    n = 16
    w = np.arange(n, dtype=np.float32)
    w[3] = -0.0
    w[4] = np.array([0x7FA00001], np.uint32).view(np.float32)[0]
    core = np.array([1, 8], np.uint32)
    cv = [np.array([1.0, 2.0], np.float32), np.array([0.5, 0.25], np.float32),
          np.array([0.0, 0.0], np.float32)]
    # index 10 is sent by all three workers with values whose sum depends on the order;
    # index 12 by workers 0 and 2; index 2 only by worker 1
    ei = [np.array([10, 12], np.uint32), np.array([2, 10], np.uint32), np.array([10, 12], np.uint32)]
    ev = [np.array([1e8, 3.0], np.float32), np.array([7.0, -1e8], np.float32),
          np.array([1.0, 4.0], np.float32)]
    got = oracle.merge(w, 0.5, core, cv, ei, ev)
    want = w.copy()
    want[1] = 1.0 - 0.5 * 1.5
    want[8] = 8.0 - 0.5 * 2.25
    want[2] = 2.0 - 0.5 * 7.0
    want[10] = 10.0 - 0.5 * 1.0            # (1e8 + -1e8) + 1 = 1 in worker order
    want[12] = 12.0 - 0.5 * 7.0
    assert np.array_equal(bits(got), bits(want))     # untouched: -0.0 and the NaN payload survive
    # one worker
    got1 = oracle.merge(w, 0.5, core, cv[:1], ei[:1], ev[:1])
    want1 = w.copy()
    want1[1], want1[8], want1[10], want1[12] = 0.5, 7.0, 10.0 - 0.5e8, 12.0 - 1.5
    assert np.array_equal(bits(got1), bits(want1))


def test_merge_single_fma_rounding_and_sign():
    # w - lr*acc with one rounding: compare with exact rationals
    rng = np.random.default_rng(21)
    n = 300
    w = rng.standard_normal(n).astype(np.float32)
    v = rng.standard_normal(n).astype(np.float32)
    lr = np.float32(0.01)
    core = np.arange(n, dtype=np.uint32)
    got = oracle.merge(w, float(lr), core, [v], [np.zeros(0, np.uint32)], [np.zeros(0, np.float32)])
    differs = 0
    for i in range(n):
        want = round_to_f32(f32_exact(w[i]) - f32_exact(lr) * f32_exact(v[i]))
        assert bits(got[i:i + 1])[0] == bits(np.array([want]))[0]
        differs += int(np.float32(w[i] - np.float32(lr * v[i])) != want)
    assert differs > 0


def test_merge_conservation_and_f64_tolerance():
    rng = np.random.default_rng(4)
    n, W, k, m = 20000, 4, 2000, 360
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(W)]
    S = oracle.score(w, g, 1.0)
    core = oracle.select_core(S, k)
    ei = [oracle.sample_explore(n, core, 0, 0, kk, m) for kk in range(W)]
    packs = [oracle.pack(g[kk], core, ei[kk]) for kk in range(W)]
    cv = [p[0] for p in packs]
    ev = [p[1] for p in packs]
    lr = 0.01
    got = oracle.merge(w, lr, core, cv, ei, ev)
    truth = oracle.merge_f64(w, lr, core, cv, ei, ev)
    # conservation: total change equals lr times everything that was sent
    sent = sum(float(np.sum(x.astype(np.float64))) for x in cv + ev)
    assert abs((w.astype(np.float64) - truth).sum() - lr * sent) <= 1e-9 * max(1.0, abs(lr * sent))
    assert np.all(np.abs(got - truth) <= 1e-6 * np.abs(truth) + 1e-12)
    # untouched entries are bit-identical
    touched = np.zeros(n, bool)
    touched[core] = True
    for x in ei:
        touched[x] = True
    assert np.array_equal(bits(got)[~touched], bits(w)[~touched])
    assert np.any(bits(got)[touched] != bits(w)[touched])


# ----------------------------------------------------------------------------------------
# Pull and local merge
# ----------------------------------------------------------------------------------------
# ----------------------------------------------------------------------------------------
# Dense update + significance of the new model (algorithm 1, the iteration before a reselection)
# ----------------------------------------------------------------------------------------
def test_dense_update_score_exact_rational_closed_form():
    rng = np.random.default_rng(21)
    n, W = 193, 3
    w = rng.standard_normal(n).astype(np.float32)
    g = [rng.standard_normal(n).astype(np.float32) * np.float32(1e-2) for _ in range(W)]
    lr = np.float32(0.01)
    c = np.float32(1.0 + 2.0 ** -12)
    w_before = w.copy()
    w_new, S = oracle.dense_update_score(w, g, float(lr), float(c))
    assert np.array_equal(bits(w), bits(w_before))                           # the input is not modified
    for i in range(n):
        acc = np.float32(0.0)
        for k in range(W):                    # from +0, worker order, each add correctly rounded
            acc = round_to_f32(f32_exact(acc) + f32_exact(g[k][i]))
        want_w = round_to_f32(f32_exact(w[i]) - f32_exact(lr) * f32_exact(acc))            # one rounding
        assert bits(w_new[i:i + 1])[0] == bits(np.array([want_w]))[0], i
        want_s = round_to_f32(abs(f32_exact(want_w)) + f32_exact(c) * abs(f32_exact(acc)))  # of the NEW model
        assert bits(S[i:i + 1])[0] == bits(np.array([want_s]))[0], i
    # the old model would have given other scores: the test can tell the two apart
    assert not np.array_equal(bits(S), bits(oracle.score(w, g, float(c))))


def test_dense_update_score_reduces_to_known_cases():
    rng = np.random.default_rng(22)
    n, W = 1000, 4
    w = rng.standard_normal(n).astype(np.float32)
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    # lr = 0: the model keeps its bits and the significance is equation (1) on it
    w0, S0 = oracle.dense_update_score(w, g, 0.0, 0.5)
    assert np.array_equal(bits(w0), bits(w))
    assert np.array_equal(bits(S0), bits(oracle.score(w, g, 0.5)))
    # the model part is the merge with every index sent by every worker (the Plump-DP update)
    core = np.arange(n, dtype=np.uint32)
    none_i, none_v = [np.zeros(0, np.uint32)] * W, [np.zeros(0, np.float32)] * W
    w1, S1 = oracle.dense_update_score(w, g, 0.125, 1.0)
    assert np.array_equal(bits(w1), bits(oracle.merge(w, 0.125, core, g, none_i, none_v)))
    # ... and the significance is equation (1) evaluated on that new model
    assert np.array_equal(bits(S1), bits(oracle.score(w1, g, 1.0)))
    # c = 0: magnitude of the new model alone
    w2, S2 = oracle.dense_update_score(w, g, 0.125, 0.0)
    assert np.array_equal(bits(S2), bits(np.abs(w2)))
    # dyadic values: no rounding anywhere, plain NumPy in binary64 is exact
    wd = (rng.integers(-1024, 1024, n) / 64.0).astype(np.float32)
    gd = [(rng.integers(-256, 256, n) / 16.0).astype(np.float32) for _ in range(W)]
    w3, S3 = oracle.dense_update_score(wd, gd, 0.25, 2.0)
    gsum = np.sum(np.stack(gd).astype(np.float64), axis=0)
    assert np.array_equal(w3.astype(np.float64), wd.astype(np.float64) - 0.25 * gsum)
    assert np.array_equal(S3.astype(np.float64), np.abs(w3.astype(np.float64)) + 2.0 * np.abs(gsum))
    # order of the sum and sign of zero: (+0 + -0) is +0, so a model value of -0 stays -0 only through the fma
    wz = np.array([-0.0, 1.0], np.float32)
    gz = [np.array([-0.0, 1e8], np.float32), np.array([-0.0, -1e8], np.float32), np.array([-0.0, 1.0], np.float32)]
    w4, S4 = oracle.dense_update_score(wz, gz, 1.0, 1.0)
    assert bits(w4)[0] == 0x80000000 and w4[1] == np.float32(0.0) and S4[1] == np.float32(1.0)


def test_core_signature_mix_known_answers_and_definition():
    gamma, mask = 0x9E3779B97F4A7C15, (1 << 64) - 1
    for line in open(os.path.join(GOLDEN, "splitmix64_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        state = int(tok[0], 0)
        for want in tok[1:]:                     # the generator's n-th output is mix(seed + (n - 1) gamma)
            assert oracle.splitmix64_mix(state) == int(want, 0)
            state = (state + gamma) & mask
    # the signature against the definition in Python integers; order matters, the empty list gives 0
    rng = np.random.default_rng(5)
    idx = np.sort(rng.choice(1 << 20, 1000, replace=False)).astype(np.uint32)
    want = sum(oracle.splitmix64_mix(int(i) + (j << 32)) for j, i in enumerate(idx)) & mask
    assert oracle.core_signature(idx) == want
    assert oracle.core_signature(np.zeros(0, np.uint32)) == 0
    swapped = idx.copy()
    swapped[[3, 4]] = swapped[[4, 3]]
    assert oracle.core_signature(swapped) != want
    changed = idx.copy()
    changed[500] += 1
    assert oracle.core_signature(changed) != want


def test_pull_reads_and_overwrites_only_the_communication_set():
    rng = np.random.default_rng(6)
    w = rng.standard_normal(100).astype(np.float32)
    wl = rng.standard_normal(100).astype(np.float32)
    core = np.array([3, 50, 99], np.uint32)
    expl = np.array([0, 51], np.uint32)
    co, eo, new_local = oracle.pull(w, core, expl, wl)
    assert np.array_equal(bits(co), bits(w)[core]) and np.array_equal(bits(eo), bits(w)[expl])
    want = wl.copy()
    want[core] = w[core]
    want[expl] = w[expl]
    assert np.array_equal(bits(new_local), bits(want))
    assert oracle.pull(w, core, expl)[2] is None


# ----------------------------------------------------------------------------------------
# Worker side: local step and accumulation (section 3.3 step 1)
# ----------------------------------------------------------------------------------------
def test_local_step_exact_rational_and_accumulation_order():
    rng = np.random.default_rng(11)
    n = 257
    w = rng.standard_normal(n).astype(np.float32)
    eta = np.float32(0.3)
    g = [(rng.standard_normal(n) * 10.0 ** rng.integers(-3, 4, n)).astype(np.float32) for _ in range(3)]
    w1, d1 = oracle.local_step(w, None, g[0], eta)
    # one rounding for the model: the exact rational w - eta * g, rounded once
    for i in range(n):
        assert w1[i] == round_to_f32(f32_exact(w[i]) - f32_exact(eta) * f32_exact(g[0][i])), i
    assert np.array_equal(bits(d1), bits(g[0]))                 # a new accumulation starts with the first update itself
    w2, d2 = oracle.local_step(w1, d1, g[1], eta)
    w3, d3 = oracle.local_step(w2, d2, g[2], eta)
    # accumulated in binary32 in mini-batch order: (g1 + g2) + g3, each sum rounded
    for i in range(n):
        s12 = round_to_f32(f32_exact(g[0][i]) + f32_exact(g[1][i]))
        assert d2[i] == s12 and d3[i] == round_to_f32(f32_exact(s12) + f32_exact(g[2][i])), i
    # an order-sensitive triple: (1e8 + -1e8) + 1 = 1, not 1e8 + (-1e8 + 1) = 0
    a = [np.array([1e8], np.float32), np.array([-1e8], np.float32), np.array([1.0], np.float32)]
    _, d = oracle.local_step(np.zeros(1, np.float32), None, a[0], 0.0)
    _, d = oracle.local_step(np.zeros(1, np.float32), d, a[1], 0.0)
    _, d = oracle.local_step(np.zeros(1, np.float32), d, a[2], 0.0)
    assert d[0] == np.float32(1.0)
    # inputs are not modified; dyadic closed form: p equal steps of 2^-3 with eta = 2^-1
    w0 = np.full(5, 1.0, np.float32)
    gg = np.full(5, 0.125, np.float32)
    ww, dd = w0, None
    for _ in range(4):
        ww, dd = oracle.local_step(ww, dd, gg, 0.5)
    assert np.all(ww == np.float32(1.0 - 4 * 0.0625)) and np.all(dd == np.float32(0.5)) and np.all(w0 == 1.0)
    # the sign: a positive gradient lowers the parameter
    wn, _ = oracle.local_step(np.zeros(1, np.float32), None, np.ones(1, np.float32), 0.25)
    assert wn[0] == np.float32(-0.25)


# ----------------------------------------------------------------------------------------
# Quantised wire values (section 2.2 end; section 4.2: 8 bits, buckets of 512)
# ----------------------------------------------------------------------------------------
def test_quant_word_counter_layout_through_a_known_answer():
    # counter (j div 4, worker, iteration low, iteration high), key (seed low ^ 0x51534744, seed high ^ kind),
    # word j mod 4: the third Philox known answer fed through that layout
    ctr, key, out = _kat()[2]
    for kind in (0, 1):
        seed = (key[0] ^ 0x51534744) | ((key[1] ^ kind) << 32)
        iteration = ctr[2] | (ctr[3] << 32)
        for c in range(4):
            assert oracle.quant_word(seed, iteration, ctr[1], kind, 4 * ctr[0] + c) == out[c]
    # kind, worker and iteration each change the stream
    base = [oracle.quant_word(7, 3, 2, 0, j) for j in range(64)]
    assert base != [oracle.quant_word(7, 3, 2, 1, j) for j in range(64)]
    assert base != [oracle.quant_word(7, 3, 1, 0, j) for j in range(64)]
    assert base != [oracle.quant_word(7, 4, 2, 0, j) for j in range(64)]


def test_quantize_grid_points_are_exact_and_signs_and_buckets():
    # scale 127 * 2^e: the grid scale * l / 127 is l * 2^e, exactly representable, so the fraction is 0, the code is
    # the level whatever the random word says, and dequantisation returns the value itself
    levels = np.arange(128, dtype=np.float32)
    v = np.concatenate([levels * 0.25, -levels * 0.25])                  # one bucket of 256 values, scale 31.75
    code, scale = oracle.quantize(v, 5, 0, 0, 0)
    assert scale.size == 1 and scale[0] == np.float32(31.75)
    assert np.array_equal(code[:128], np.arange(128, dtype=np.uint8))
    assert np.array_equal(code[129:], np.arange(129, 256, dtype=np.uint8))   # sign bit + level
    assert code[128] == 0x80                                               # -0.0 keeps its sign bit
    out = oracle.dequantize(code, scale)
    assert np.array_equal(bits(out), bits(v))
    # buckets of 512: element 512 belongs to the second bucket and is scaled by ITS maximum; a ragged last bucket;
    # a bucket of zeros
    v = np.zeros(512 * 3 + 5, np.float32)
    v[0], v[511], v[512], v[1023] = 127.0, 1.0, 254.0, -2.0
    v[1536:] = [0.5, 0.25, 0.0, -0.5, 0.125]
    code, scale = oracle.quantize(v, 1, 2, 3, 1)
    assert np.array_equal(scale, np.array([127.0, 254.0, 0.0, 0.5], np.float32))
    assert code[0] == 127 and code[511] == 1 and code[512] == 127 and code[1023] == 0x80 | 1
    assert not code[1024:1536].any()
    assert code[1536] == 127 and code[1539] == 0x80 | 127 and code[1538] == 0
    assert np.array_equal(oracle.dequantize(code, scale)[[0, 511, 512, 1023]], np.array([127.0, 1.0, 254.0, -2.0], np.float32))


def test_quantize_rounds_up_exactly_when_the_word_says_so():
    """Between two grid points the code is the lower level plus (u < fraction), with u the top 24 bits of the
    element's random word as a fraction of 2^24; checked in exact rationals with words from the pinned Philox."""
    rng = np.random.default_rng(3)
    n = 700
    v = rng.standard_normal(n).astype(np.float32)
    seed, it, worker, kind = 12345, 9, 4, 1
    code, scale = oracle.quantize(v, seed, it, worker, kind)
    ups = 0
    for j in range(n):
        s = np.float32(np.max(np.abs(v[(j // 512) * 512:(j // 512 + 1) * 512])))
        assert scale[j // 512] == s
        r = round_to_f32(abs(f32_exact(v[j])) / f32_exact(s))              # binary32 quotient
        y = round_to_f32(f32_exact(r) * 127)                               # binary32 product
        lvl = int(np.floor(float(y)))
        frac = f32_exact(y) - lvl                                          # exact in binary32
        block = oracle.philox4x32_10([j >> 2, worker, it, 0], [seed ^ 0x51534744, kind])
        u = Fraction(int(block[j & 3]) >> 8, 1 << 24)
        up = 1 if u < frac else 0
        ups += up
        assert int(code[j]) == (0x80 if v[j] < 0 else 0) | (lvl + up), j
    assert 0.3 * n < ups < 0.7 * n                                          # both branches are taken
    # dequantisation: two roundings, product then quotient
    out = oracle.dequantize(code, scale)
    for j in range(n):
        lvl = int(code[j]) & 0x7F
        mag = round_to_f32(f32_exact(round_to_f32(f32_exact(scale[j // 512]) * lvl)) / 127)
        assert out[j] == (-mag if code[j] & 0x80 else mag), j


def test_quantize_is_unbiased_and_bounded():
    """Expectation over the random words equals the value (the property that makes the scheme usable for gradients),
    and a dequantised value never leaves the two grid points around it."""
    rng = np.random.default_rng(8)
    n = 512
    v = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    acc = np.zeros(n, np.float64)
    reps = 400
    step = float(np.max(np.abs(v))) / 127.0
    for it in range(reps):
        code, scale = oracle.quantize(v, 77, it, 0, 0)
        out = oracle.dequantize(code, scale).astype(np.float64)
        assert np.all(np.abs(out - v) <= step * (1 + 1e-6))
        acc += out
    mean = acc / reps
    # the error of one draw is at most one step with variance <= step^2 / 4: 6 standard errors
    assert np.all(np.abs(mean - v) <= 6 * 0.5 * step / np.sqrt(reps) + 1e-12)


def test_wire_bytes_against_section_3_5():
    n, alpha, beta = 1_000_000, 0.2, 0.1
    k, m = int(beta * n), int((alpha - beta) * n)
    assert oracle.wire_bytes(k, m, False) == round(4 * (2 * alpha - beta) * n)     # (2 alpha - beta) n words
    q = oracle.wire_bytes(k, m, True)
    nb = lambda c: -(-c // 512)
    assert q == k + m + 4 * m + 4 * (nb(k) + nb(m))
    assert q < 0.6 * oracle.wire_bytes(k, m, False)            # values shrink fourfold, the explorer's keys do not

"""GPU parity: every call of the C ABI against the CPU oracle on the same seeded inputs.

Bar: bit-exact scores, index sets, tile offsets, packs, pulls and random words; merged
binary32 parameters within 1e-6 relative (+1e-12) of the oracle and of the binary64 truth
(they are in fact expected to be bit-identical, and the test reports if they are not).
Sizes span several 4096-parameter tiles and a ragged tail.
"""
import numpy as np
import pytest

import oracle
from paper_1709_09393_amd import binding, workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev():
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but torch.cuda.is_available() is False")
    return torch.device("cuda:0")


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(dev())


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def f32bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def host_tile_offsets(idx, tile_start):
    return np.searchsorted(idx.astype(np.int64), tile_start.astype(np.int64), side="left").astype(np.uint32)


def run_iteration(wl, iteration=0, w_h=None, sd=None, force_fallback=False, check=True, hint=False, per_tile_tail=False,
                  clobber_after_select=False, hint_mode=0, as_scored=True, refill_before_pack=False, explore_async=0):
    """One reselect iteration on the GPU and in the oracle; returns both results."""
    seg_off = [int(x) for x in wl.segment_offsets()]
    ks, ms = [int(x) for x in wl.k_seg()], [int(x) for x in wl.m_seg()]
    w_h = wl.weights() if w_h is None else w_h
    g_h = wl.gradients(iteration)
    own = sd is None
    if own:
        sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    sd.set_option("explore_force_fallback", int(force_fallback))
    sd.set_option("explore_per_tile_tail", int(per_tile_tail))      # 1: never the short-list explorer path
    w = to_dev(w_h)
    g = [to_dev(x) for x in g_h]
    sd.set_option("explore_hint_mode", hint_mode)
    sd.set_option("explore_async", explore_async)
    if hint:        # the explorer zones are drawn ahead: on the library's side stream (1) or inside the scoring kernel (0)
        sd.explore_hint(ks, iteration, ms, 0, wl.W)
    S = sd.score(w, g, wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, ks, reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, ks, iteration, ms, 0, wl.W)
    if clobber_after_select:        # probe: values that can then only come from what the scoring pass kept
        for x in g:
            x.zero_()
    if refill_before_pack:          # the same buffers get the next updates: the pack (no flag) must extract those
        g_h = wl.gradients(iteration + 1000)
        for x, y in zip(g, g_h):
            x.copy_(to_dev(y))
    core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=as_scored)
    sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
    core_out, expl_out = sd.pull(w, epoch, core_idx, core_off, expl_idx, expl_off)
    sd.synchronize()
    got = dict(S=S.cpu().numpy(), core_idx=u32(core_idx), core_bits=u32(core_bits), core_off=u32(core_off),
               expl_idx=[u32(x) for x in expl_idx], expl_off=[u32(x) for x in expl_off],
               core_val=[x.cpu().numpy() for x in core_val], expl_val=[x.cpu().numpy() for x in expl_val],
               w=w.cpu().numpy(), core_out=[x.cpu().numpy() for x in core_out],
               expl_out=[x.cpu().numpy() for x in expl_out], tile_start=sd.tile_starts())
    if own:
        sd.close()
    if not check:
        return got, None
    so = None if wl.n_seg == 1 and wl.seg_off is None else seg_off
    S_o = oracle.score(w_h, wl.gradients(iteration), wl.c)
    core_o = oracle.select_core(S_o, ks, so)
    ei_o = [oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, iteration, q, ms, so) for q in range(wl.W)]
    packs = [oracle.pack(g_h[q], core_o, ei_o[q]) for q in range(wl.W)]
    w_o = oracle.merge(w_h, wl.lr, core_o, [p[0] for p in packs], ei_o, [p[1] for p in packs])
    w_t = oracle.merge_f64(w_h, wl.lr, core_o, [p[0] for p in packs], ei_o, [p[1] for p in packs])
    # sum of |value| sent to each index: the scale of the binary32 summation error
    sent = oracle.merge_f64(np.zeros_like(w_h), -1.0, core_o, [np.abs(p[0]) for p in packs], ei_o,
                            [np.abs(p[1]) for p in packs])
    want = dict(S=S_o, core_idx=core_o, expl_idx=ei_o, packs=packs, w=w_o, w_truth=w_t, sent=sent, lr=wl.lr)
    return got, want


def assert_iteration_matches(wl, got, want):
    ts = got["tile_start"]
    assert np.array_equal(f32bits(got["S"]), f32bits(want["S"])), "score bits"
    assert np.array_equal(got["core_idx"], want["core_idx"]), "core index set"
    assert np.array_equal(got["core_bits"], oracle.core_bits(wl.n, want["core_idx"])), "core bitmap"
    assert np.array_equal(got["core_off"], host_tile_offsets(want["core_idx"], ts)), "core tile offsets"
    for q in range(wl.W):
        assert np.array_equal(got["expl_idx"][q], want["expl_idx"][q]), "explorer %d" % q
        assert np.array_equal(got["expl_off"][q], host_tile_offsets(want["expl_idx"][q], ts))
        assert np.array_equal(f32bits(got["core_val"][q]), f32bits(want["packs"][q][0])), "core_val %d" % q
        assert np.array_equal(f32bits(got["expl_val"][q]), f32bits(want["packs"][q][1])), "expl_val %d" % q
    w_g, w_o, w_t = got["w"], want["w"], want["w_truth"]
    assert np.all(np.abs(w_g - w_o) <= 1e-6 * np.abs(w_o) + 1e-12), "merge vs oracle"
    # against exact arithmetic: 1e-6 relative to the result plus 1e-6 of the update's own scale
    # (a sum of up to W binary32 values carries about W * 2^-24 of sum|v|, scaled by lr)
    tol = 1e-6 * (np.abs(w_t) + want["lr"] * want["sent"]) + 1e-12
    assert np.all(np.abs(w_g.astype(np.float64) - w_t) <= tol), "merge vs binary64"
    nbad = int((f32bits(w_g) != f32bits(w_o)).sum())
    assert nbad == 0, "merged parameters differ from the oracle in %d places (within tolerance)" % nbad
    for q in range(wl.W):
        assert np.array_equal(f32bits(got["core_out"][q]), f32bits(w_o[want["core_idx"]])), "pull core"
        assert np.array_equal(f32bits(got["expl_out"][q]), f32bits(w_o[want["expl_idx"][q]])), "pull explorer"


# ----------------------------------------------------------------------------------------
def test_philox_words_match_oracle():
    sd = binding.SlimDP(100_000, 2, seed=0x299F31D0A4093822)
    for it, worker, i0, cnt in [(0, 0, 0, 10_000), (2 ** 33 + 7, 5, 3, 4099), (1, 31, 99_000, 1000)]:
        got = u32(sd.debug_philox(it, worker, i0, cnt))
        assert np.array_equal(got, oracle.explore_words(0x299F31D0A4093822, it, worker, i0, cnt))
    sd.close()


@pytest.mark.parametrize("n", [1, 5, 4096, 4097, 50_001, 200_003])
def test_flat_iteration_sizes(n):
    wl = workloads.TINY.scaled(n)
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("W", [4, 16])
def test_score_with_several_tiles_per_persistent_block(W):
    """More tiles than the scoring kernel has blocks, so that every wave walks through several tiles (the smaller
    cases give each block one tile at most); with and without the announced draw and the capture."""
    wl = workloads.TINY.scaled(6_000_003, W=W)
    w_h, g_h = wl.weights(), wl.gradients(0)
    S_o = oracle.score(w_h, g_h, wl.c)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    w, g = to_dev(w_h), [to_dev(x) for x in g_h]
    assert sd.T > 1024
    S = sd.score(w, g, wl.c)
    sd.synchronize()
    assert np.array_equal(f32bits(S.cpu().numpy()), f32bits(S_o)), "plain"
    sd.set_option("speculative_pack", 1)
    for t in range(2):
        sd.explore_hint([wl.k], t, [wl.m], 0, wl.W)
        sd.score(w, g, wl.c, out=S)
        core_idx, core_bits, core_off, epoch = sd.select_core(S, [wl.k], reuse_histogram=True)
        sd.synchronize()
        assert np.array_equal(f32bits(S.cpu().numpy()), f32bits(S_o)), "hinted, capturing (%d)" % t
    w2 = to_dev(w_h)
    sd.dense_update_score(w2, g, wl.lr, wl.c, out=S)
    sd.synchronize()
    w_o, S2_o = oracle.dense_update_score(w_h, g_h, wl.lr, wl.c)
    assert np.array_equal(f32bits(w2.cpu().numpy()), f32bits(w_o)) and np.array_equal(f32bits(S.cpu().numpy()), f32bits(S2_o))
    sd.close()


@pytest.mark.parametrize("W", [1, 2, 3, 8, 16, 32])          # 32: the most the interface takes
def test_worker_counts(W):
    wl = workloads.TINY.scaled(30_011, W=W)
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


def test_tiny_config_full_size():
    wl = workloads.TINY
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


def test_segmented_googlenet_recipe_scaled():
    wl = workloads.GOOGLENET.scaled(700_001)
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


def test_segmented_googlenet_config_full_size_as_benched():
    """The GoogLeNet-sized configuration at full size (6,998,552 parameters in 57 segments, W = 4) the way
    bench.py drives it: speculative packing on, the draw announced ahead, two iterations on one context."""
    wl = workloads.GOOGLENET
    seg_off = [int(x) for x in wl.segment_offsets()]
    sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    for t in range(2):
        got, want = run_iteration(wl, iteration=t, sd=sd, hint=True)
        assert_iteration_matches(wl, got, want)
    sd.close()


def test_segments_with_awkward_boundaries():
    n = 30_000
    wl = workloads.TINY.scaled(n, seg_off=(0, 1, 18, 4114, 4115, 12_307, 29_999, n), n_seg=7)
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("pack_kernel,nbuf", [(1, 2), (0, 1), (0, 2)])
def test_general_pack_kernels(pack_kernel, nbuf):
    """The pack that scans the update vectors, in its forms (loading and storing waves apart; one set of waves with
    one or two tiles in LDS): flat with a ragged last tile and three workers, segmented, and an explorer so full that
    a tile holds more of its entries than a block has threads."""
    cases = [workloads.TINY.scaled(200_003, W=3), workloads.GOOGLENET.scaled(300_001),
             workloads.TINY.scaled(50_000, W=2, core_pct=5, explore_pct=40), workloads.TINY.scaled(5, W=1)]
    for wl in cases:
        seg_off = [int(x) for x in wl.segment_offsets()]
        sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
        sd.set_option("pack_kernel", pack_kernel)
        sd.set_option("pack_nbuf", nbuf)
        got, want = run_iteration(wl, sd=sd, as_scored=False)
        assert_iteration_matches(wl, got, want)
        sd.close()


def test_many_small_segments():
    """1,500 segments of 1 to 200 parameters (most tiles hold a few dozen parameters, many segments get k = 0 or m = 0):
    per-segment rankings, the explorer's per-tile tail (such zones are not narrow) and every list's tile offsets."""
    rng = np.random.default_rng(3)
    sizes = rng.integers(1, 201, 1500)
    seg_off = tuple(int(x) for x in np.concatenate([[0], np.cumsum(sizes)]))
    wl = workloads.TINY.scaled(seg_off[-1], W=2, seg_off=seg_off, n_seg=len(sizes), core_pct=10, explore_pct=20)
    for hint in (False, True):
        got, want = run_iteration(wl, hint=hint)
        assert_iteration_matches(wl, got, want)


def test_tie_heavy_stress_recipe_scaled():
    wl = workloads.STRESS.scaled(300_007)
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("mode", [1, 2])          # 1: too few candidates; 2: the sure zone alone exceeds the demand
@pytest.mark.parametrize("hint", [False, True])
@pytest.mark.parametrize("per_tile_tail", [False, True])
def test_explore_exact_rerun_gives_the_same_sets(mode, hint, per_tile_tail):
    wl = workloads.TINY.scaled(100_003)
    got, want = run_iteration(wl, force_fallback=mode, hint=hint, per_tile_tail=per_tile_tail)
    assert_iteration_matches(wl, got, want)
    wl = workloads.GOOGLENET.scaled(300_001)
    got, want = run_iteration(wl, force_fallback=mode, hint=hint, per_tile_tail=per_tile_tail)
    assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("hint", [False, True])
def test_explore_per_tile_tail_with_narrow_zones(hint):
    """The general explorer tail (the one that also serves wide zones) on workloads that would take the short list."""
    for wl in (workloads.TINY.scaled(200_003), workloads.GOOGLENET.scaled(300_001),
               workloads.STRESS.scaled(150_001, W=5), workloads.TINY.scaled(20_005, core_pct=10, explore_pct=60)):
        got, want = run_iteration(wl, hint=hint, per_tile_tail=True)
        assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("hint_mode", [0, 1])
@pytest.mark.parametrize("n,W", [(5, 1), (4097, 3), (200_003, 4), (150_001, 8)])
def test_hinted_draw_matches(n, W, hint_mode):
    wl = workloads.TINY.scaled(n, W=W)
    got, want = run_iteration(wl, iteration=3, hint=True, hint_mode=hint_mode)
    assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("hint_mode", [0, 1])
def test_hinted_draw_segmented_and_stress_and_rerun(hint_mode):
    wl = workloads.GOOGLENET.scaled(300_001)
    got, want = run_iteration(wl, hint=True, hint_mode=hint_mode)
    assert_iteration_matches(wl, got, want)
    wl = workloads.TINY.scaled(30_000, seg_off=(0, 1, 18, 4114, 4115, 12_307, 29_999, 30_000), n_seg=7)
    got, want = run_iteration(wl, hint=True, hint_mode=hint_mode)
    assert_iteration_matches(wl, got, want)
    wl = workloads.STRESS.scaled(100_003)
    got, want = run_iteration(wl, hint=True, hint_mode=hint_mode)
    assert_iteration_matches(wl, got, want)
    wl = workloads.TINY.scaled(100_003)                       # narrow bound too small: exact rerun
    got, want = run_iteration(wl, hint=True, force_fallback=True, hint_mode=hint_mode)
    assert_iteration_matches(wl, got, want)
    for core_pct, explore_pct in [(0, 2), (10, 0), (50, 100), (10, 60)]:
        wl = workloads.TINY.scaled(20_005, core_pct=core_pct, explore_pct=explore_pct)
        got, want = run_iteration(wl, hint=True, hint_mode=hint_mode)
        assert_iteration_matches(wl, got, want)


@pytest.mark.parametrize("per_tile_tail", [False, True])
def test_explorer_ties_at_the_threshold_take_the_lower_index(per_tile_tail):
    """Two equal Philox words exactly at the threshold, the demand covering one of them: both explorer tails
    must hand it to the lower index.  Pairs early in the ranking go through the short list, late ones through
    the per-tile tail with a wide zone."""
    n, seed = 1 << 20, 9
    r = oracle.explore_words(seed, 0, 0, 0, n)
    order = np.argsort(r, kind="stable")
    rs = r[order]
    dup = np.flatnonzero(rs[1:] == rs[:-1])
    early, late = dup[dup < n // 8], dup[dup > n // 2]
    assert early.size and late.size
    sd = binding.SlimDP(n, 1, seed=seed)
    sd.set_option("explore_per_tile_tail", int(per_tile_tail))
    core_bits = torch.zeros((n + 31) // 32, dtype=torch.int32, device=dev())
    core = np.zeros(0, np.uint32)
    for d in (early[0], early[-1], late[0]):
        m = int(d) + 1                      # the words below the pair, plus one
        want = oracle.sample_explore(n, core, seed, 0, 0, m)
        tied = np.sort(order[rs == rs[d]])
        assert tied[0] in want and tied[1] not in want
        expl_idx, expl_off = sd.sample_explore(core_bits, [0], 0, [m], 0, 1)
        sd.synchronize()
        assert np.array_equal(u32(expl_idx[0]), want)
    sd.close()


@pytest.mark.parametrize("hint", [False, True])
def test_speculative_pack_over_iterations(hint):
    """With speculative packing on, the scoring pass keeps the update values of the likely core (from the second
    iteration on, once a threshold is known) and the pack takes them from there; everything stays bit-exact.
    Flat, segmented (tiles that are never captured), and a changing core size (threshold below the capture bound)."""
    for wl in (workloads.TINY.scaled(200_003), workloads.GOOGLENET.scaled(300_001), workloads.STRESS.scaled(150_001, W=8),
               workloads.GOOGLENET.scaled(300_001, core_pct=40)):       # more captured per sub-tile than is kept
        seg_off = [int(x) for x in wl.segment_offsets()]
        sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
        sd.set_option("speculative_pack", 1)
        for t in range(3):
            got, want = run_iteration(wl, iteration=t, sd=sd, hint=hint)
            assert_iteration_matches(wl, got, want)
        wl2 = workloads.TINY.scaled(wl.n, W=wl.W, core_pct=25) if wl.n_seg == 1 else None
        if wl2 is not None:                 # a much larger core: its threshold lies below what was captured
            got, want = run_iteration(wl2, iteration=3, sd=sd, hint=hint)
            assert_iteration_matches(wl2, got, want)
            got, want = run_iteration(wl2, iteration=4, sd=sd, hint=hint)
            assert_iteration_matches(wl2, got, want)
        sd.close()


@pytest.mark.parametrize("W", [1, 2, 3, 16])
def test_speculative_pack_worker_counts(W):
    """Entry widths of 1, 2 and 16 values (W = 3 is never captured: the pack then gathers); several tiles per block."""
    wl = workloads.TINY.scaled(4_500_007, W=W)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    k, m = wl.k, wl.m
    w_h = wl.weights()
    w = to_dev(w_h)
    for t in range(2):
        g_h = wl.gradients(t)
        g = [to_dev(x) for x in g_h]
        sd.explore_hint([k], t, [m], 0, W)
        S = sd.score(w, g, wl.c)
        core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
        expl_idx, expl_off = sd.sample_explore(core_bits, [k], t, [m], 0, W)
        core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=True)
        sd.synchronize()
        core_o = oracle.select_core(oracle.score(w_h, g_h, wl.c), k)
        assert np.array_equal(u32(core_idx), core_o), t
        for q in range(W):
            ei_o = oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, t, q, m)
            assert np.array_equal(u32(expl_idx[q]), ei_o), (t, q)
            cv_o, ev_o = oracle.pack(g_h[q], core_o, ei_o)
            assert np.array_equal(f32bits(core_val[q].cpu().numpy()), f32bits(cv_o)), (t, q)
            assert np.array_equal(f32bits(expl_val[q].cpu().numpy()), f32bits(ev_o)), (t, q)
    sd.close()


def test_speculative_pack_really_uses_the_captured_values():
    """White-box probe: zero the update vectors after the selection.  Core values of captured tiles must still be
    the original ones (they can only come from the capture); from the third pack on nothing is captured any more
    (one capture serves one pack) and the same pack call reads the zeroed vectors."""
    wl = workloads.TINY.scaled(200_000)            # whole tiles except the last one
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    run_iteration(wl, iteration=0, sd=sd, check=False)
    got, want = run_iteration(wl, iteration=1, sd=sd, clobber_after_select=True)
    ts = got["tile_start"]
    full = int(ts[-2])                              # parameters below this index lie in whole tiles
    core = want["core_idx"]
    inside = core < full
    assert inside.sum() > 1000
    for q in range(wl.W):
        assert np.array_equal(f32bits(got["core_val"][q][inside]), f32bits(want["packs"][q][0][inside]))
        assert not np.any(got["core_val"][q][~inside])       # the ragged last tile is gathered: zeros
        assert not np.any(got["expl_val"][q])                # explorer values are gathered: zeros
    sd.close()


def test_pack_from_the_capture_with_lists_of_any_origin():
    """A pack that states its updates are the scored ones takes the core values from what the scoring pass kept and
    the explorer values by index: lists from another draw than the announced one, of another length, hand-made
    lists, and a fuller explorer (10 % of the rest) all get the right values."""
    wl = workloads.TINY.scaled(300_001, W=4)
    ks, ms = [wl.k], [wl.m]
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    w_h = wl.weights()
    w = to_dev(w_h)
    rng = np.random.default_rng(11)
    for t, (it_hint, it_req, m_req) in enumerate([(0, 0, wl.m), (5, 6, wl.m), (7, 7, wl.m // 3), (8, 8, None)]):
        g_h = wl.gradients(t)
        g = [to_dev(x) for x in g_h]
        sd.explore_hint(ks, it_hint, ms, 0, wl.W)
        S = sd.score(w, g, wl.c)
        core_idx, core_bits, core_off, epoch = sd.select_core(S, ks, reuse_histogram=True)
        core_o = oracle.select_core(oracle.score(w_h, g_h, wl.c), ks[0])
        if m_req is None:       # hand-made lists: random non-core indices, another length per worker
            rest = np.setdiff1d(np.arange(wl.n, dtype=np.uint32), core_o)
            ei_h = [np.sort(rng.choice(rest, size=1000 + 777 * q, replace=False)).astype(np.uint32) for q in range(wl.W)]
            expl_idx = [to_dev(x) for x in ei_h]
            expl_off = [sd.tile_offsets(x) for x in expl_idx]
        else:
            expl_idx, expl_off = sd.sample_explore(core_bits, ks, it_req, [m_req], 0, wl.W)
            ei_h = [oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, it_req, q, m_req) for q in range(wl.W)]
        core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=True)
        sd.synchronize()
        for q in range(wl.W):
            assert np.array_equal(u32(expl_idx[q]), ei_h[q]), (t, q)
            cv_o, ev_o = oracle.pack(g_h[q], core_o, ei_h[q])
            assert np.array_equal(f32bits(core_val[q].cpu().numpy()), f32bits(cv_o)), (t, q)
            assert np.array_equal(f32bits(expl_val[q].cpu().numpy()), f32bits(ev_o)), (t, q)
    sd.close()
    # a fuller explorer
    wl = workloads.TINY.scaled(150_000, W=8, explore_pct=10)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    for t in range(2):
        got, want = run_iteration(wl, iteration=t, sd=sd, hint=True)
        assert_iteration_matches(wl, got, want)
    sd.close()


@pytest.mark.parametrize("bias", [0, 1 << 22, -(1 << 20), -(1 << 22)])
@pytest.mark.parametrize("announced", [False, True])
def test_first_iteration_captures_under_a_sampled_bound(bias, announced):
    """No selection has run yet: the scoring pass estimates the coming threshold from a sample of its own
    significances.  Estimate as it is, forced far too high (the selection's verdict rejects the capture: the pack
    gathers), too low (a larger capture) and far too low (more parameters qualify than a sub-tile keeps: the pack
    gathers the rest): the same bits in every case; the white-box probe (updates zeroed after the selection) shows
    which source the pack used."""
    wl = workloads.TINY.scaled(700_000)             # 170 whole tiles and a ragged one
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    sd.set_option("capture_estimate_bias", bias)
    if not announced:
        sd.set_option("expected_core", wl.k)
    got, want = run_iteration(wl, iteration=0, sd=sd, hint=announced)
    assert_iteration_matches(wl, got, want)
    sd.close()
    if bias == 0 or bias == -(1 << 22):
        return
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    sd.set_option("capture_estimate_bias", bias)
    if not announced:
        sd.set_option("expected_core", wl.k)
    got, want = run_iteration(wl, iteration=0, sd=sd, hint=announced, clobber_after_select=True)
    full = int(got["tile_start"][-2])
    inside = want["core_idx"] < full
    for q in range(wl.W):
        if bias < 0:        # every core parameter of a whole tile was kept by the scoring pass
            assert np.array_equal(f32bits(got["core_val"][q][inside]), f32bits(want["packs"][q][0][inside]))
        else:               # rejected capture: the pack read the (zeroed) vectors
            assert not np.any(got["core_val"][q])
    sd.close()


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_selection_with_the_scoring_pass_classifying_against_a_predicted_bin(mode):
    """Flat models: the scoring pass sorts whole tiles against the previous selection's threshold bin and the selection
    skips its own pass over the scores when the histogram confirms the bin.  mode 1 as shipped (iterations 1.. predict
    from the iteration before; a much larger core in between moves the bin, so the prediction fails there), 0 never,
    2 always a wrong bin: the same sets in every case.  Also through the dense update + score call."""
    wl = workloads.TINY.scaled(500_003)                 # 122 whole tiles and a ragged one
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("core_predict", mode)
    sd.set_option("speculative_pack", 1)
    for t, pct in enumerate([10, 10, 30, 30, 1, 10]):
        wl2 = workloads.TINY.scaled(wl.n, core_pct=pct)
        got, want = run_iteration(wl2, iteration=t, sd=sd, hint=(t % 2 == 0))
        assert_iteration_matches(wl2, got, want)
    w_h, g_h = wl.weights(), wl.gradients(9)
    w, g = to_dev(w_h), [to_dev(x) for x in g_h]
    for rep in range(2):                                # the second call predicts from the first one's selection
        w_h, S_o = oracle.dense_update_score(w_h, g_h, wl.lr, wl.c)
        S = sd.dense_update_score(w, g, wl.lr, wl.c)
        core_idx, core_bits, core_off, epoch = sd.select_core(S, [wl.k], reuse_histogram=True)
        sd.synchronize()
        core_o = oracle.select_core(S_o, wl.k)
        assert np.array_equal(u32(core_idx), core_o), rep
        assert np.array_equal(u32(core_bits), oracle.core_bits(wl.n, core_o)), rep
    sd.close()


@pytest.mark.parametrize("hint_mode", [0, 1])
@pytest.mark.parametrize("spec", [0, 1])
def test_asynchronous_explorer_requests(hint_mode, spec):
    """Option explore_async: the explorer request runs on the library's side stream; pack (after extracting the core
    values from what the scoring pass kept, if it did), merge and pull wait for it.  Flat, segmented, wide zones,
    forced exact rerun; a few iterations on one context."""
    cases = [workloads.TINY.scaled(300_007), workloads.GOOGLENET.scaled(300_001), workloads.STRESS.scaled(100_003, W=5),
             workloads.TINY.scaled(20_005, core_pct=10, explore_pct=60)]
    for wl in cases:
        sd = binding.SlimDP(wl.n, wl.W, seg_off=[int(x) for x in wl.segment_offsets()], seed=workloads.EXPLORE_SEED)
        sd.set_option("speculative_pack", spec)
        for t in range(3):
            got, want = run_iteration(wl, iteration=t, sd=sd, hint=True, hint_mode=hint_mode, explore_async=1,
                                      force_fallback=(1 if t == 2 else 0))
            assert_iteration_matches(wl, got, want)
        sd.close()


@pytest.mark.parametrize("hint_mode", [0, 1])
def test_asynchronous_explorer_one_iteration_ahead(hint_mode):
    """Steady iterations with cached core keys: the request for iteration t+1 (other output arrays) is issued before
    the pack of iteration t and runs on the side stream beside pack and merge (hint_mode 1: after its announced draw
    on the same stream; 0: nothing announced, the request draws itself).  Every set, and the model after every
    iteration, as in the oracle."""
    wl = workloads.LOOP.scaled(250_007, W=4)
    n, W, k, m = wl.n, wl.W, wl.k, wl.m
    sd = binding.SlimDP(n, W, seed=workloads.EXPLORE_SEED)
    sd.set_option("explore_async", 1)
    sd.set_option("explore_hint_mode", hint_mode)
    w_h = wl.weights()
    w = to_dev(w_h)
    g_h = wl.gradients(0)
    S = sd.score(w, [to_dev(x) for x in g_h], wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
    core_o = oracle.select_core(oracle.score(w_h, g_h, wl.c), k)
    bufs = [sd.sample_explore(core_bits, [k], 0, [m], 0, W), None]
    for t in range(8):
        g_h = wl.gradients(t)
        g = [to_dev(x) for x in g_h]
        if hint_mode == 1:
            sd.explore_hint([k], t + 1, [m], 0, W)
        nxt = bufs[(t + 1) & 1]
        expl_idx, expl_off = bufs[t & 1]

        def request_next():
            bufs[(t + 1) & 1] = sd.sample_explore(core_bits, [k], t + 1, [m], 0, W, expl_idx=None if nxt is None else nxt[0],
                                                  expl_off=None if nxt is None else nxt[1])
        request_next()
        core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch)
        sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
        core_out, expl_out = sd.pull(w, epoch, core_idx, core_off, expl_idx, expl_off)
        sd.synchronize()
        ei_o = [oracle.sample_explore(n, core_o, workloads.EXPLORE_SEED, t, q, m) for q in range(W)]
        packs = [oracle.pack(g_h[q], core_o, ei_o[q]) for q in range(W)]
        w_h = oracle.merge(w_h, wl.lr, core_o, [x[0] for x in packs], ei_o, [x[1] for x in packs])
        for q in range(W):
            assert np.array_equal(u32(expl_idx[q]), ei_o[q]), (t, q)
            assert np.array_equal(f32bits(expl_val[q].cpu().numpy()), f32bits(packs[q][1])), (t, q)
            assert np.array_equal(f32bits(expl_out[q].cpu().numpy()), f32bits(w_h[ei_o[q]])), (t, q)
        assert np.array_equal(f32bits(w.cpu().numpy()), f32bits(w_h)), t
    sd.close()


def test_pack_without_the_flag_reads_the_buffers_it_is_given():
    """The update buffers are refilled in place between the scoring pass and the pack (what a training loop that
    reuses its buffers does between two iterations): without SLIMDP_PACK_UPDATES_AS_SCORED the pack must extract the
    new contents although a capture of the old ones exists; a table of other arrays under the flag is refused."""
    wl = workloads.TINY.scaled(200_003)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    run_iteration(wl, iteration=0, sd=sd, check=False)
    got, want = run_iteration(wl, iteration=1, sd=sd, as_scored=False, refill_before_pack=True)
    assert_iteration_matches(wl, got, want)
    # the flag with a different table: an error, nothing launched
    w = to_dev(wl.weights())
    g = [to_dev(x) for x in wl.gradients(2)]
    S = sd.score(w, g, wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [wl.k], reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, [wl.k], 2, [wl.m], 0, wl.W)
    other = [x.clone() for x in g]
    with pytest.raises(binding.SlimDPError) as e:
        sd.pack(other, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=True)
    assert e.value.code == binding.ERR_INVALID_ARG
    sd.synchronize()
    sd.close()


@pytest.mark.parametrize("hint_mode", [0, 1])
def test_hint_that_does_not_match_the_request_is_ignored(hint_mode):
    wl = workloads.TINY.scaled(50_001, W=2)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    sd.set_option("explore_hint_mode", hint_mode)
    w = to_dev(wl.weights())
    g_h = wl.gradients(0)
    g = [to_dev(x) for x in g_h]
    k, m = wl.k, wl.m
    sd.explore_hint([k], 7, [m], 0, 2)                        # announced: iteration 7, workers 0..1
    S = sd.score(w, g, wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
    core_o = u32(core_idx)
    # asked for: iteration 8; then worker 1 alone; then a different m
    for (it, w0, nw, mm) in [(8, 0, 2, m), (7, 1, 1, m), (7, 0, 2, m - 5)]:
        sd.explore_hint([k], 7, [m], 0, 2)
        sd.score(w, g, wl.c, out=S)
        sd.select_core(S, [k], reuse_histogram=True, core_idx=core_idx, core_bits=core_bits, core_off=core_off)
        expl_idx, _ = sd.sample_explore(core_bits, [k], it, [mm], w0, nw)
        sd.synchronize()
        for q in range(nw):
            want = oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, it, w0 + q, mm)
            assert np.array_equal(u32(expl_idx[q]), want), (it, w0, nw, mm)
    sd.close()


@pytest.mark.parametrize("core_pct,explore_pct", [(0, 2), (10, 0), (100, 0), (0, 100), (50, 100), (0, 0)])
def test_degenerate_fractions(core_pct, explore_pct):
    # beta = 0 (pure random sampling), beta = alpha (no exploration), k = n (dense update),
    # explorer = everything outside the core
    wl = workloads.TINY.scaled(20_005, core_pct=core_pct, explore_pct=explore_pct)
    got, want = run_iteration(wl)
    assert_iteration_matches(wl, got, want)


def test_select_core_on_constructed_scores():
    n = 70_001
    sd = binding.SlimDP(n, 1)
    rng = np.random.default_rng(0)
    cases = {
        "all_equal": np.full(n, 0.125, np.float32),
        "two_values": rng.integers(0, 2, n).astype(np.float32),
        "few_levels": (rng.integers(0, 37, n) / 8.0).astype(np.float32),
        "zeros_and_denormals": (rng.integers(0, 3, n) * np.float32(1e-45)).astype(np.float32),
        "with_inf_nan": np.abs(rng.standard_normal(n)).astype(np.float32),
        "same_top_bits": (np.float32(1.0) + rng.integers(0, 64, n).astype(np.float32) * np.float32(2.0 ** -23)),
    }
    cases["with_inf_nan"][::1000] = np.inf
    cases["with_inf_nan"][5::1000] = np.array([0x7FC00000], np.uint32).view(np.float32)[0]
    for name, S_h in cases.items():
        S = to_dev(S_h)
        for k in [0, 1, n // 10, n // 2, n - 1, n]:
            core_idx, core_bits, core_off, _ = sd.select_core(S, [k])
            sd.synchronize()
            want = oracle.select_core(S_h, k)
            assert np.array_equal(u32(core_idx), want), (name, k)
            assert np.array_equal(u32(core_bits), oracle.core_bits(n, want)), (name, k)
    sd.close()


def test_merge_hand_built_collisions_and_tile_offsets():
    n = 10_000
    sd = binding.SlimDP(n, 3)
    rng = np.random.default_rng(1)
    w_h = rng.standard_normal(n).astype(np.float32)
    w_h[7] = -0.0
    S = to_dev(np.abs(w_h))
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [50])
    core_h = u32(core_idx)
    rest = np.setdiff1d(np.arange(n, dtype=np.uint32), core_h)
    # three workers, overlapping explorer lists: index rest[10] is sent by all, with values
    # whose sum depends on the order
    ei = [np.sort(np.concatenate([rest[[10, 500, 4100]], rest[6000:6100]])).astype(np.uint32),
          np.sort(np.concatenate([rest[[10, 4100]], rest[6050:6200]])).astype(np.uint32),
          np.sort(rest[[10, 11, 9000]]).astype(np.uint32)]
    ev = [rng.standard_normal(x.size).astype(np.float32) for x in ei]
    ev[0][np.searchsorted(ei[0], rest[10])] = 1e8
    ev[1][np.searchsorted(ei[1], rest[10])] = -1e8
    ev[2][np.searchsorted(ei[2], rest[10])] = 1.0
    cv = [rng.standard_normal(50).astype(np.float32) for _ in range(3)]
    d_ei = [to_dev(x) for x in ei]
    d_eo = [sd.tile_offsets(x) for x in d_ei]
    ts = sd.tile_starts()
    for q in range(3):
        assert np.array_equal(u32(d_eo[q]), host_tile_offsets(ei[q], ts))
    w = to_dev(w_h)
    sd.merge(w, 0.5, epoch, core_idx, core_off, [to_dev(x) for x in cv], d_ei, d_eo, [to_dev(x) for x in ev])
    sd.synchronize()
    want = oracle.merge(w_h, 0.5, core_h, cv, ei, ev)
    assert np.array_equal(f32bits(w.cpu().numpy()), f32bits(want))
    assert want[rest[10]] == np.float32(w_h[rest[10]] - 0.5)       # (1e8 + -1e8) + 1
    sd.close()


def test_merge_explorer_lists_that_overlap_the_core_follow_the_stated_order():
    # Invalid input (an explorer never holds a core index), but the interface states what happens: the core
    # contributions to such an index are added first, in worker order, then the explorer ones in worker order.
    # The addends are chosen so that any other order gives other bits.
    n = 3 * 4096 + 77
    W = 3
    sd = binding.SlimDP(n, W)
    rng = np.random.default_rng(5)
    w_h = rng.standard_normal(n).astype(np.float32)
    S = to_dev(np.abs(w_h))
    k = 40
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k])
    core_h = u32(core_idx)
    cv = [rng.standard_normal(k).astype(np.float32) for _ in range(W)]
    one, two, three = int(core_h[3]), int(core_h[17]), int(core_h[31])       # core indices also sent as explorers
    w_h[[one, two, three]] = [0.75, -1.25, 2.5]      # short values: the expected fma below is exact in binary64
    big = np.float32(2.0 ** 26)
    for j in (3, 31):
        cv[0][j], cv[1][j], cv[2][j] = big, np.float32(1.0), -big            # (big + 1) - big = 0 in binary32
    cv[0][17], cv[1][17], cv[2][17] = big, np.float32(1.0), np.float32(1.0)  # stays big (spacing 8 above 2^26)
    rest = np.setdiff1d(np.arange(n, dtype=np.uint32), core_h)
    ei = [np.sort(np.concatenate([rest[[5, 900]], [one, two, three]])).astype(np.uint32),
          np.sort(np.concatenate([rest[[5, 7000]], [three]])).astype(np.uint32),
          np.sort(np.concatenate([rest[[5, 12000]], [two, three]])).astype(np.uint32)]
    ev = [rng.standard_normal(x.size).astype(np.float32) for x in ei]
    sent = {one: [(0, 0.5)], two: [(0, 5.0), (2, -3.0)], three: [(0, big), (1, 5.0), (2, -big)]}
    accs = {}
    for idx, lst in sent.items():
        for q, v in lst:
            ev[q][np.searchsorted(ei[q], idx)] = np.float32(v)
    lr = np.float32(0.5)
    want = oracle.merge(w_h, float(lr), core_h, cv, [np.setdiff1d(x, core_h) for x in ei],
                        [v[~np.isin(x, core_h)] for x, v in zip(ei, ev)])    # everything outside the three indices
    for idx, lst in sent.items():
        j = int(np.searchsorted(core_h, idx))
        acc = np.float32(0.0)
        for q in range(W):
            acc = np.float32(acc + cv[q][j])
        for q, v in lst:
            acc = np.float32(acc + np.float32(v))
        accs[idx] = float(acc)
        want[idx] = np.float32(np.float64(w_h[idx]) - np.float64(lr) * np.float64(acc))   # exact product, one rounding
    # core first: 0 + 0.5; (big + 5 -> big + 8) - 3 -> big + 8 (the other order gives big); ((0 + big) + 5 -> big + 8) - big
    assert accs == {one: 0.5, two: float(big) + 8.0, three: 8.0}
    d_ei = [to_dev(x) for x in ei]
    d_eo = [sd.tile_offsets(x) for x in d_ei]
    d_cv, d_ev = [to_dev(x) for x in cv], [to_dev(x) for x in ev]
    for _ in range(3):
        w = to_dev(w_h)
        sd.merge(w, float(lr), epoch, core_idx, core_off, d_cv, d_ei, d_eo, d_ev)
        sd.synchronize()
        assert np.array_equal(f32bits(w.cpu().numpy()), f32bits(want))
    sd.close()


@pytest.mark.parametrize("pull_kernel", [1, 0])       # 1: the local models are streamed; 0: patched by scattered writes
def test_pull_overwrites_local_models_only_at_the_communication_set(pull_kernel):
    wl = workloads.TINY.scaled(25_003, W=2)
    seg_off = [0, wl.n]
    sd = binding.SlimDP(wl.n, wl.W)
    sd.set_option("pull_kernel", pull_kernel)
    w_h = wl.weights()
    g_h = wl.gradients(0)
    w = to_dev(w_h)
    g = [to_dev(x) for x in g_h]
    S = sd.score(w, g, 1.0)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [wl.k], reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, [wl.k], 3, [wl.m], 0, 2)
    rng = np.random.default_rng(2)
    wl_h = [rng.standard_normal(wl.n).astype(np.float32) for _ in range(2)]
    w_local = [to_dev(wl_h[0]), None]
    core_out, expl_out = sd.pull(w, epoch, core_idx, core_off, expl_idx, expl_off, w_local=w_local)
    sd.synchronize()
    ci = u32(core_idx)
    for q in range(2):
        eq = u32(expl_idx[q])
        co, eo, new_local = oracle.pull(w_h, ci, eq, wl_h[q] if q == 0 else None)
        assert np.array_equal(f32bits(core_out[q].cpu().numpy()), f32bits(co))
        assert np.array_equal(f32bits(expl_out[q].cpu().numpy()), f32bits(eo))
        if q == 0:
            assert np.array_equal(f32bits(w_local[0].cpu().numpy()), f32bits(new_local))
    sd.close()
    assert seg_off[-1] == wl.n


def test_same_call_twice_gives_identical_bits_and_workers_differ():
    wl = workloads.TINY.scaled(60_001)
    a, _ = run_iteration(wl, check=False)
    b, _ = run_iteration(wl, check=False)
    for key in ["core_idx", "core_bits", "core_off"]:
        assert np.array_equal(a[key], b[key])
    for q in range(wl.W):
        assert np.array_equal(a["expl_idx"][q], b["expl_idx"][q])
    assert np.array_equal(f32bits(a["w"]), f32bits(b["w"]))
    assert not np.array_equal(a["expl_idx"][0], a["expl_idx"][1])
    c, _ = run_iteration(wl, iteration=1, check=False)
    assert not np.array_equal(a["expl_idx"][0], c["expl_idx"][0])


@pytest.mark.parametrize("announce", [False, True])
def test_multi_iteration_loop_scaled(announce):
    # 20 iterations, core every 5, explorer every iteration, model carried along.  announce: every draw is announced
    # one iteration ahead; the scoring pass of a reselecting iteration carries it, otherwise the side stream
    wl = workloads.LOOP.scaled(40_009 if not announce else 300_007, W=4)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    if announce:
        sd.set_option("speculative_pack", 1)
        sd.explore_hint([wl.k], 0, [wl.m], 0, wl.W)
    w_h = wl.weights()
    w = to_dev(w_h)
    k, m = wl.k, wl.m
    core_o = None
    for t in range(wl.iterations):
        g_h = wl.gradients(t)
        g = [to_dev(x) for x in g_h]
        if t % wl.reselect_every == 0:
            S = sd.score(w, g, wl.c)
            core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
            core_o = oracle.select_core(oracle.score(w_h, g_h, wl.c), k)
            assert np.array_equal(u32(core_idx), core_o), t
        expl_idx, expl_off = sd.sample_explore(core_bits, [k], t, [m], 0, wl.W)
        if announce:
            sd.set_option("explore_hint_mode", 0 if (t + 1) % wl.reselect_every == 0 else 1)
            sd.explore_hint([k], t + 1, [m], 0, wl.W)
        # only a reselecting iteration packs the updates its scoring pass saw
        core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch,
                                     updates_as_scored=(t % wl.reselect_every == 0))
        sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
        ei_o = [oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, t, q, m) for q in range(wl.W)]
        for q in range(wl.W):
            assert np.array_equal(u32(expl_idx[q]), ei_o[q]), (t, q)
        packs = [oracle.pack(g_h[q], core_o, ei_o[q]) for q in range(wl.W)]
        w_h = oracle.merge(w_h, wl.lr, core_o, [p[0] for p in packs], ei_o, [p[1] for p in packs])
    sd.synchronize()
    w_g = w.cpu().numpy()
    assert np.all(np.abs(w_g - w_h) <= 1e-6 * np.abs(w_h) + 1e-12)
    assert np.array_equal(f32bits(w_g), f32bits(w_h))
    sd.close()


@pytest.mark.parametrize("n,W,segmented", [(5, 1, False), (4097, 3, False), (200_003, 8, False), (300_001, 4, True)])
@pytest.mark.parametrize("hint", [False, True])
def test_dense_update_score_matches_oracle(n, W, segmented, hint):
    """The iteration before a reselection: all updates applied, significance of the new model, then the selection."""
    wl = workloads.GOOGLENET.scaled(n, W=W) if segmented else workloads.TINY.scaled(n, W=W)
    seg_off = [int(x) for x in wl.segment_offsets()]
    ks, ms = [int(x) for x in wl.k_seg()], [int(x) for x in wl.m_seg()]
    sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)            # must not capture here: the next pack packs other updates
    w_h, g_h = wl.weights(), wl.gradients(4)
    w, g = to_dev(w_h), [to_dev(x) for x in g_h]
    if hint:
        sd.explore_hint(ks, 5, ms, 0, wl.W)
    S = sd.dense_update_score(w, g, wl.lr, wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, ks, reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, ks, 5, ms, 0, wl.W)
    g2_h = wl.gradients(5)                          # the next iteration's updates go through the new sets
    g2 = [to_dev(x) for x in g2_h]
    core_val, expl_val = sd.pack(g2, core_idx, core_off, expl_idx, expl_off, epoch)
    sd.synchronize()
    w_o, S_o = oracle.dense_update_score(w_h, g_h, wl.lr, wl.c)
    assert np.array_equal(f32bits(w.cpu().numpy()), f32bits(w_o)), "updated model bits"
    assert np.array_equal(f32bits(S.cpu().numpy()), f32bits(S_o)), "score bits"
    so = None if not segmented else seg_off
    core_o = oracle.select_core(S_o, ks, so)
    assert np.array_equal(u32(core_idx), core_o)
    for q in range(wl.W):
        ei_o = oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, 5, q, ms, so)
        assert np.array_equal(u32(expl_idx[q]), ei_o), q
        cv_o, ev_o = oracle.pack(g2_h[q], core_o, ei_o)
        assert np.array_equal(f32bits(core_val[q].cpu().numpy()), f32bits(cv_o)), q
        assert np.array_equal(f32bits(expl_val[q].cpu().numpy()), f32bits(ev_o)), q
    sd.close()


def test_paper_schedule_loop_scaled():
    """Algorithm 1's schedule with q = 5 over 12 iterations: sparse push/merge through the cached core, except that
    the iteration before each reselection pushes everything and the new core is ranked with the new model."""
    wl = workloads.LOOP.scaled(40_009, W=4)
    q_every = 5
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    w_h = wl.weights()
    w = to_dev(w_h)
    k, m = wl.k, wl.m
    # before the first reselection there is no core in the paper: the benchmark's start (selection at t = 0)
    g_h = wl.gradients(0)
    S = sd.score(w, [to_dev(x) for x in g_h], wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
    core_o = oracle.select_core(oracle.score(w_h, g_h, wl.c), k)
    for t in range(12):
        g_h = wl.gradients(t)
        g = [to_dev(x) for x in g_h]
        if (t + 1) % q_every == 0:
            S = sd.dense_update_score(w, g, wl.lr, wl.c)
            core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
            w_h, S_o = oracle.dense_update_score(w_h, g_h, wl.lr, wl.c)
            core_o = oracle.select_core(S_o, k)
            assert np.array_equal(u32(core_idx), core_o), t
        else:
            expl_idx, expl_off = sd.sample_explore(core_bits, [k], t, [m], 0, wl.W)
            core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch)
            sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
            ei_o = [oracle.sample_explore(wl.n, core_o, workloads.EXPLORE_SEED, t, q, m) for q in range(wl.W)]
            packs = [oracle.pack(g_h[q], core_o, ei_o[q]) for q in range(wl.W)]
            w_h = oracle.merge(w_h, wl.lr, core_o, [p[0] for p in packs], ei_o, [p[1] for p in packs])
    sd.synchronize()
    assert np.array_equal(f32bits(w.cpu().numpy()), f32bits(w_h))
    sd.close()


def test_core_signature_matches_oracle():
    wl = workloads.TINY.scaled(700_001)
    sd = binding.SlimDP(wl.n, wl.W, seed=workloads.EXPLORE_SEED)
    S = to_dev(oracle.score(wl.weights(), wl.gradients(0), wl.c))
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [wl.k])
    sig = sd.core_signature(core_idx)
    empty = sd.core_signature(core_idx[:0])
    one = sd.core_signature(core_idx[:1])
    sd.synchronize()
    core = u32(core_idx)
    assert int(sig.cpu().numpy().view(np.uint64)[0]) == oracle.core_signature(core)
    assert int(empty.cpu().numpy().view(np.uint64)[0]) == 0
    assert int(one.cpu().numpy().view(np.uint64)[0]) == oracle.core_signature(core[:1])
    sd.close()


def test_randomized_configurations():
    """Seeded sweep over sizes, worker counts, fractions, segmentations and the library's options (announced draws in
    both modes, speculative packing, the general explorer tail, forced exact reruns), a few iterations per context."""
    import random
    rnd = random.Random(20260101)
    for case in range(16):
        n = rnd.choice([rnd.randint(1, 5000), rnd.randint(5000, 300_000), rnd.randint(300_000, 900_000)])
        W = rnd.choice([1, 2, 3, 4, 5, 8, 16])
        kw = dict(W=W, core_pct=rnd.choice([0, 1, 5, 10, 30, 100]), explore_pct=rnd.choice([0, 1, 2, 10, 50, 100]))
        nseg = rnd.choice([1, 1, 1, rnd.randint(2, 40)])
        if nseg > 1 and n > 2 * nseg:
            cuts = sorted(rnd.sample(range(1, n), nseg - 1))
            kw.update(seg_off=tuple([0] + cuts + [n]), n_seg=nseg)
        wl = (workloads.TINY if rnd.random() < 0.7 else workloads.STRESS).scaled(n, **kw)
        sd = binding.SlimDP(wl.n, wl.W, seg_off=[int(x) for x in wl.segment_offsets()], seed=workloads.EXPLORE_SEED)
        if rnd.random() < 0.6:
            sd.set_option("speculative_pack", 1)
        for t in range(rnd.choice([1, 2, 3])):
            opts = dict(hint=rnd.random() < 0.6, hint_mode=rnd.choice([0, 1]), per_tile_tail=rnd.random() < 0.2,
                        force_fallback=rnd.choice([0, 0, 0, 1, 2]))
            got, want = run_iteration(wl, iteration=t, sd=sd, **opts)
            try:
                assert_iteration_matches(wl, got, want)
            except AssertionError as e:
                raise AssertionError("case %d (%s, iteration %d, %r): %s" % (case, wl, t, opts, e))
        sd.close()


def test_error_paths_launch_nothing():
    n = 10_000
    sd = binding.SlimDP(n, 2)
    S = to_dev(np.abs(np.random.default_rng(0).standard_normal(n)).astype(np.float32))
    with pytest.raises(binding.SlimDPError) as e:
        sd.select_core(S, [n + 1])
    assert e.value.code == binding.ERR_OUT_OF_RANGE
    with pytest.raises(binding.SlimDPError) as e:
        sd.select_core(S, [10], reuse_histogram=True)          # no slimdp_score before it
    assert e.value.code == binding.ERR_INVALID_ARG
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [100])
    with pytest.raises(binding.SlimDPError) as e:
        sd.sample_explore(core_bits, [100], 0, [n - 99])
    assert e.value.code == binding.ERR_OUT_OF_RANGE
    with pytest.raises(binding.SlimDPError) as e:
        sd.sample_explore(core_bits, [100], 0, [5], 0, 3)       # more workers than the context holds
    assert e.value.code == binding.ERR_INVALID_ARG
    expl_idx, expl_off = sd.sample_explore(core_bits, [100], 0, [5])
    g = [S]
    with pytest.raises(binding.SlimDPError) as e:
        sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch + 1)
    assert e.value.code == binding.ERR_STALE_CORE
    core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch)
    sd.select_core(S, [100])                                    # new core: old packs are stale
    with pytest.raises(binding.SlimDPError) as e:
        sd.merge(S, 0.1, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
    assert e.value.code == binding.ERR_STALE_CORE
    with pytest.raises(binding.SlimDPError) as e:
        sd.score(S, [S], -1.0)
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.SlimDPError) as e:
        sd.dense_update_score(S, [S], 0.1, 1.0, out=S)          # the score may not overwrite the model
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.SlimDPError) as e:
        sd.dense_update_score(S, [S], float("nan"), 1.0)
    assert e.value.code == binding.ERR_INVALID_ARG
    sd.synchronize()
    # a bitmap with more core bits than k_seg claims: the device reports the shortfall
    full = to_dev(np.full((n + 31) // 32, 0xFFFFFFFF, np.uint32))
    sd.sample_explore(full, [0], 0, [10])
    with pytest.raises(binding.SlimDPError) as e:
        sd.synchronize()
    assert e.value.code == binding.ERR_DEVICE_STATUS
    sd.synchronize()                                            # status is cleared once reported
    sd.close()


# ----------------------------------------------------------------------------------------
# Worker side: local steps, accumulated updates, pull with local overwrite (section 3.3 steps 1, 4, 5)
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,W,shift", [(1, 1, 0), (4099, 3, 0), (300_001, 4, 0), (70_000, 2, 1)])
def test_local_step_matches_oracle(n, W, shift):
    """p = 3 mini-batch steps; shift = 1 starts every array one element into its allocation (no 16-byte alignment)."""
    rng = np.random.default_rng(n)
    sd = binding.SlimDP(n, W)
    eta = 0.05
    w_h = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    d_h = [None] * W

    def dev_arr(a):
        buf = torch.full((n + shift,), float("nan"), dtype=torch.float32, device=dev())
        buf[shift:] = torch.from_numpy(a)
        return buf[shift:]
    w = [dev_arr(x) for x in w_h]
    d = [dev_arr(np.full(n, np.nan, np.float32)) for _ in range(W)]      # a first step must not read it
    for j in range(3):
        g_h = [(rng.standard_normal(n) * 10.0 ** rng.integers(-4, 3, n)).astype(np.float32) for _ in range(W)]
        g = [dev_arr(x) for x in g_h]
        sd.local_step(w, g, d, eta, first=(j == 0))
        sd.synchronize()
        for q in range(W):
            w_h[q], d_h[q] = oracle.local_step(w_h[q], d_h[q], g_h[q], eta)
            assert np.array_equal(f32bits(w[q].cpu().numpy()), f32bits(w_h[q])), (j, q)
            assert np.array_equal(f32bits(d[q].cpu().numpy()), f32bits(d_h[q])), (j, q)
    with pytest.raises(binding.SlimDPError) as e:
        sd.local_step(w, w, d, eta, first=True)                           # gradient aliases the model
    assert e.value.code == binding.ERR_INVALID_ARG
    sd.close()


@pytest.mark.parametrize("n,W,segmented,shift,nbuf", [(5, 1, False, 0, 2), (4097, 3, False, 0, 1), (200_003, 8, False, 0, 2),
                                                        (300_001, 4, True, 0, 2), (70_000, 2, False, 1, 2)])
def test_local_step_and_pack_in_one_pass(n, W, segmented, shift, nbuf):
    """The last mini-batch step before a push together with the extraction: the same local models, accumulated updates
    and packs as the oracle's local step followed by its pack, for a first step (p = 1) and for an accumulating one;
    flat and segmented, ragged tiles, arrays without 16-byte alignment, an explorer request still running on the side
    stream when the call is made."""
    wl = (workloads.GOOGLENET if segmented else workloads.TINY).scaled(n, W=W)
    seg_off = [int(x) for x in wl.segment_offsets()]
    ks, ms = [int(x) for x in wl.k_seg()], [int(x) for x in wl.m_seg()]
    so = None if wl.n_seg == 1 and wl.seg_off is None else seg_off
    rng = np.random.default_rng(n + W)
    sd = binding.SlimDP(n, W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    sd.set_option("pack_nbuf", nbuf)
    sd.set_option("explore_async", 1)
    eta = 0.05

    def dev_arr(a):
        buf = torch.full((n + shift,), float("nan"), dtype=torch.float32, device=dev())
        buf[shift:] = torch.from_numpy(a)
        return buf[shift:]
    S_h = np.abs(wl.weights())
    core_idx, core_bits, core_off, epoch = sd.select_core(to_dev(S_h), ks)
    core_o = oracle.select_core(S_h, ks, so)
    w_h = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    w = [dev_arr(x) for x in w_h]
    d = [dev_arr(np.full(n, np.nan, np.float32)) for _ in range(W)]
    d_h = [None] * W
    for t, steps in enumerate([1, 3]):                       # p = 1: the only step is the first one; p = 3: two plain steps before
        expl_idx, expl_off = sd.sample_explore(core_bits, ks, t, ms, 0, W)        # asynchronous: the call below waits for it
        ei_o = [oracle.sample_explore(n, core_o, workloads.EXPLORE_SEED, t, q, ms, so) for q in range(W)]
        d_h = [None] * W
        for j in range(steps):
            g_h = [(rng.standard_normal(n) * 10.0 ** rng.integers(-4, 3, n)).astype(np.float32) for _ in range(W)]
            g = [dev_arr(x) for x in g_h]
            if j + 1 < steps:
                sd.local_step(w, g, d, eta, first=(j == 0))
            else:
                core_val, expl_val = sd.local_step_pack(w, g, d, eta, j == 0, core_idx, core_off, expl_idx, expl_off, epoch)
            for q in range(W):
                w_h[q], d_h[q] = oracle.local_step(w_h[q], d_h[q], g_h[q], eta)
        sd.synchronize()
        for q in range(W):
            assert np.array_equal(u32(expl_idx[q]), ei_o[q]), (t, q)
            assert np.array_equal(f32bits(w[q].cpu().numpy()), f32bits(w_h[q])), (t, q)
            assert np.array_equal(f32bits(d[q].cpu().numpy()), f32bits(d_h[q])), (t, q)
            cv_o, ev_o = oracle.pack(d_h[q], core_o, ei_o[q])
            assert np.array_equal(f32bits(core_val[q].cpu().numpy()), f32bits(cv_o)), (t, q)
            assert np.array_equal(f32bits(expl_val[q].cpu().numpy()), f32bits(ev_o)), (t, q)
    with pytest.raises(binding.SlimDPError) as e:
        sd.local_step_pack(w, g, d, eta, True, core_idx, core_off, expl_idx, expl_off, epoch + 1)
    assert e.value.code == binding.ERR_STALE_CORE
    with pytest.raises(binding.SlimDPError) as e:
        sd.local_step_pack(w, w, d, eta, True, core_idx, core_off, expl_idx, expl_off, epoch)
    assert e.value.code == binding.ERR_INVALID_ARG
    sd.synchronize()
    sd.close()


@pytest.mark.parametrize("n,W,segmented,shift,explore_pct", [(5, 1, False, 0, 2), (4097, 3, False, 0, 2), (200_003, 8, False, 0, 2),
                                                               (300_001, 4, True, 0, 2), (70_000, 2, False, 1, 2),
                                                               (50_000, 2, False, 0, 40)])
def test_pull_and_local_step_in_one_pass(n, W, segmented, shift, explore_pct):
    """Pull, local merge and the first local step of the next round together: the same local models and accumulated
    updates as the oracle's pull (with local overwrite) followed by its local step, starting a new accumulation and
    continuing one; flat and segmented, ragged tiles, arrays without 16-byte alignment, an explorer so full that a tile
    holds more of its entries than a block has threads, an explorer request still running on the side stream."""
    wl = (workloads.GOOGLENET if segmented else workloads.TINY).scaled(n, W=W, explore_pct=explore_pct)
    seg_off = [int(x) for x in wl.segment_offsets()]
    ks, ms = [int(x) for x in wl.k_seg()], [int(x) for x in wl.m_seg()]
    so = None if wl.n_seg == 1 and wl.seg_off is None else seg_off
    rng = np.random.default_rng(n + 7 * W)
    sd = binding.SlimDP(n, W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    sd.set_option("explore_async", 1)
    eta = 0.05

    def dev_arr(a):
        buf = torch.full((n + shift,), float("nan"), dtype=torch.float32, device=dev())
        buf[shift:] = torch.from_numpy(a)
        return buf[shift:]
    w_h = wl.weights()
    w = dev_arr(w_h)
    core_idx, core_bits, core_off, epoch = sd.select_core(to_dev(np.abs(w_h)), ks)
    core_o = oracle.select_core(np.abs(w_h), ks, so)
    wk_h = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    wk = [dev_arr(x) for x in wk_h]
    d = [dev_arr(np.full(n, np.nan, np.float32)) for _ in range(W)]
    d_h = [None] * W
    for t, first in enumerate([True, False]):
        expl_idx, expl_off = sd.sample_explore(core_bits, ks, t, ms, 0, W)        # asynchronous: the call below waits for it
        g_h = [(rng.standard_normal(n) * 10.0 ** rng.integers(-4, 3, n)).astype(np.float32) for _ in range(W)]
        g = [dev_arr(x) for x in g_h]
        sd.pull_local_step(w, epoch, core_idx, core_off, expl_idx, expl_off, wk, g, d, eta, first=first)
        sd.synchronize()
        for q in range(W):
            ei_o = oracle.sample_explore(n, core_o, workloads.EXPLORE_SEED, t, q, ms, so)
            assert np.array_equal(u32(expl_idx[q]), ei_o), (t, q)
            _, _, pulled = oracle.pull(w_h, core_o, ei_o, wk_h[q])
            wk_h[q], d_h[q] = oracle.local_step(pulled, None if first else d_h[q], g_h[q], eta)
            assert np.array_equal(f32bits(wk[q].cpu().numpy()), f32bits(wk_h[q])), (t, q)
            assert np.array_equal(f32bits(d[q].cpu().numpy()), f32bits(d_h[q])), (t, q)
    with pytest.raises(binding.SlimDPError) as e:
        sd.pull_local_step(w, epoch + 1, core_idx, core_off, expl_idx, expl_off, wk, g, d, eta)
    assert e.value.code == binding.ERR_STALE_CORE
    with pytest.raises(binding.SlimDPError) as e:
        sd.pull_local_step(w, epoch, core_idx, core_off, expl_idx, expl_off, wk, wk, d, eta)
    assert e.value.code == binding.ERR_INVALID_ARG
    sd.synchronize()
    sd.close()


def test_worker_loop_closure_local_models_diverge_and_are_pulled_back():
    """W local models carried through the loop of algorithm 1's worker side: p = 2 local mini-batch steps accumulate
    delta_k, the communication set of delta_k is pushed and merged, the worker pulls the global values at its
    communication set and overwrites its local model there.  Global model, every local model and every set match the
    oracle at every iteration; and, as section 3.1 argues, parameters outside a worker's communication set drift away
    from the global model while those inside are equal to it right after the pull."""
    wl = workloads.LOOP.scaled(60_001, W=4)
    n, W, k, m = wl.n, wl.W, wl.k, wl.m
    p_steps, every, eta = 2, 3, 0.05
    sd = binding.SlimDP(n, W, seed=workloads.EXPLORE_SEED)
    w_h = wl.weights()
    w = to_dev(w_h)
    wk_h = [w_h.copy() for _ in range(W)]                   # first line of the worker loop: every worker pulls the whole model
    wk = [to_dev(x) for x in wk_h]
    delta = [torch.empty(n, dtype=torch.float32, device=dev()) for _ in range(W)]
    core_o = None
    for t in range(7):
        d_h = [None] * W
        for j in range(p_steps):
            g_h = wl.gradients(t * p_steps + j)
            sd.local_step(wk, [to_dev(x) for x in g_h], delta, eta, first=(j == 0))
            for q in range(W):
                wk_h[q], d_h[q] = oracle.local_step(wk_h[q], d_h[q], g_h[q], eta)
        if t % every == 0:
            S = sd.score(w, delta, wl.c)
            core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
            core_o = oracle.select_core(oracle.score(w_h, d_h, wl.c), k)
            assert np.array_equal(u32(core_idx), core_o), t
        expl_idx, expl_off = sd.sample_explore(core_bits, [k], t, [m], 0, W)
        core_val, expl_val = sd.pack(delta, core_idx, core_off, expl_idx, expl_off, epoch)
        sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
        sd.pull(w, epoch, core_idx, core_off, expl_idx, expl_off, w_local=wk)
        sd.synchronize()
        ei_o = [oracle.sample_explore(n, core_o, workloads.EXPLORE_SEED, t, q, m) for q in range(W)]
        packs = [oracle.pack(d_h[q], core_o, ei_o[q]) for q in range(W)]
        w_h = oracle.merge(w_h, wl.lr, core_o, [x[0] for x in packs], ei_o, [x[1] for x in packs])
        assert np.array_equal(f32bits(w.cpu().numpy()), f32bits(w_h)), t
        for q in range(W):
            assert np.array_equal(u32(expl_idx[q]), ei_o[q]), (t, q)
            _, _, wk_h[q] = oracle.pull(w_h, core_o, ei_o[q], wk_h[q])
            got = wk[q].cpu().numpy()
            assert np.array_equal(f32bits(got), f32bits(wk_h[q])), (t, q)
            inside = np.zeros(n, bool)
            inside[core_o] = True
            inside[ei_o[q]] = True
            assert np.array_equal(f32bits(got[inside]), f32bits(w_h[inside]))          # pulled: equal to the global model
            if t >= 2:      # never-communicated parameters have drifted: almost all of them differ from the global model
                outside = ~inside
                assert np.mean(got[outside] != w_h[outside]) > 0.95, (t, q)
    sd.close()


# ----------------------------------------------------------------------------------------
# Quantised wire values (sections 2.2 and 4.2: 8 bits, buckets of 512)
# ----------------------------------------------------------------------------------------
def test_quantized_packs_match_oracle_and_merge():
    wl = workloads.TINY.scaled(300_007)
    n, W, k, m = wl.n, wl.W, wl.k, wl.m
    it = 6
    sd = binding.SlimDP(n, W, seed=0x1234_5678_9ABC_DEF0)
    w_h, g_h = wl.weights(), wl.gradients(it)
    w, g = to_dev(w_h), [to_dev(x) for x in g_h]
    S = sd.score(w, g, wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, [k], it, [m], 0, W)
    core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch)
    c_code, c_scale = sd.quantize(core_val, 0, it)
    e_code, e_scale = sd.quantize(expl_val, 1, it)
    cv_q = sd.dequantize(c_code, c_scale)
    ev_q = sd.dequantize(e_code, e_scale)
    sd.merge(w, wl.lr, epoch, core_idx, core_off, cv_q, expl_idx, expl_off, ev_q)
    sd.synchronize()
    core_o, ei_o = u32(core_idx), [u32(x) for x in expl_idx]
    cv_o, ev_o = [], []
    for q in range(W):
        cv_h, ev_h = oracle.pack(g_h[q], core_o, ei_o[q])
        for kind, vals, code, scale, deq, keep in ((0, cv_h, c_code, c_scale, cv_q, cv_o), (1, ev_h, e_code, e_scale, ev_q, ev_o)):
            code_o, scale_o = oracle.quantize(vals, 0x1234_5678_9ABC_DEF0, it, q, kind)
            assert np.array_equal(code[q].cpu().numpy(), code_o), (q, kind)
            assert np.array_equal(f32bits(scale[q].cpu().numpy()), f32bits(scale_o)), (q, kind)
            deq_o = oracle.dequantize(code_o, scale_o)
            assert np.array_equal(f32bits(deq[q].cpu().numpy()), f32bits(deq_o)), (q, kind)
            keep.append(deq_o)
    w_o = oracle.merge(w_h, wl.lr, core_o, cv_o, ei_o, ev_o)
    w_g = w.cpu().numpy()
    assert np.all(np.abs(w_g - w_o) <= 1e-6 * np.abs(w_o) + 1e-12)
    assert np.array_equal(f32bits(w_g), f32bits(w_o))
    # the quantised update stays within one grid step of the exact one, and the bytes shrink as section 3.5 counts them
    exact = oracle.merge(w_h, wl.lr, core_o, [oracle.pack(g_h[q], core_o, ei_o[q])[0] for q in range(W)], ei_o,
                         [oracle.pack(g_h[q], core_o, ei_o[q])[1] for q in range(W)])
    step = max(float(np.max(np.abs(x))) for x in g_h) / 127.0
    assert np.max(np.abs(w_o - exact)) <= wl.lr * W * step * 1.01
    assert binding.wire_bytes(k, m, True) == oracle.wire_bytes(k, m, True) < binding.wire_bytes(k, m, False) == 4 * (k + 2 * m)
    sd.close()


@pytest.mark.parametrize("count", [1, 3, 511, 512, 513, 1024, 5001])
def test_quantize_ragged_counts_zero_buckets_and_unaligned_arrays(count):
    rng = np.random.default_rng(count)
    sd = binding.SlimDP(10_000, 3, seed=5)
    vals_h = [rng.standard_normal(count).astype(np.float32) * np.float32(10.0 ** rng.integers(-6, 3)) for _ in range(3)]
    vals_h[1][: min(count, 512)] = 0.0                                  # a bucket of zeros (incl. a negative zero)
    vals_h[1][0] = -0.0
    buf = [torch.empty(count + 1, dtype=torch.float32, device=dev()) for _ in range(3)]
    vals = []
    for q in range(3):
        view = buf[q][1:] if q == 2 else buf[q][:count]                  # worker 2: not 16-byte aligned
        view.copy_(torch.from_numpy(vals_h[q]))
        vals.append(view)
    code, scale = sd.quantize(vals, 1, 2 ** 35 + 3, worker0=0)
    out = sd.dequantize(code, scale)
    sd.synchronize()
    for q in range(3):
        code_o, scale_o = oracle.quantize(vals_h[q], 5, 2 ** 35 + 3, q, 1)
        assert np.array_equal(code[q].cpu().numpy(), code_o), q
        assert np.array_equal(f32bits(scale[q].cpu().numpy()), f32bits(scale_o)), q
        assert np.array_equal(f32bits(out[q].cpu().numpy()), f32bits(oracle.dequantize(code_o, scale_o))), q
    sd.close()


@pytest.mark.parametrize("segmented", [False, True])
def test_checkpoint_resume_gives_the_same_run(segmented):
    """20 iterations in one go against 12 iterations, a checkpoint (global model, core keys, iteration; the seed is
    configuration), a NEW context that adopts the keys, and the remaining 8: the same explorer sets at every
    iteration and the same final model bits.  The counter-based generator makes the explorers functions of
    (seed, iteration, worker, core) alone, so nothing else needs saving."""
    wl = (workloads.GOOGLENET.scaled(200_001, W=3) if segmented else workloads.LOOP.scaled(40_009, W=4))
    seg_off = [int(x) for x in wl.segment_offsets()]
    ks, ms = [int(x) for x in wl.k_seg()], [int(x) for x in wl.m_seg()]
    T_all, every, stop = 20, 5, 12

    def run(t_from, t_to, w, sd, core):
        sets = {}
        for t in range(t_from, t_to):
            g = [to_dev(x) for x in wl.gradients(t)]
            if t % every == 0:
                S = sd.score(w, g, wl.c)
                core = sd.select_core(S, ks, reuse_histogram=True)
            core_idx, core_bits, core_off, epoch = core
            expl_idx, expl_off = sd.sample_explore(core_bits, ks, t, ms, 0, wl.W)
            core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch)
            sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
            sd.synchronize()
            sets[t] = [u32(x) for x in expl_idx]
        return core, sets

    sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    w_a = to_dev(wl.weights())
    _, sets_a = run(0, T_all, w_a, sd, None)
    sd.close()

    sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    w_b = to_dev(wl.weights())
    core, sets_b = run(0, stop, w_b, sd, None)
    saved_w, saved_core = w_b.cpu().numpy().copy(), u32(core[0]).copy()          # the checkpoint
    sd.close()
    del w_b, core
    sd = binding.SlimDP(wl.n, wl.W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
    w_b = to_dev(saved_w)
    core_idx = to_dev(saved_core)
    core_bits, core_off, epoch = sd.import_core(core_idx, ks)
    sd.synchronize()
    assert np.array_equal(u32(core_bits), oracle.core_bits(wl.n, saved_core))
    assert np.array_equal(u32(core_off), host_tile_offsets(saved_core, sd.tile_starts()))
    _, sets_c = run(stop, T_all, w_b, sd, (core_idx, core_bits, core_off, epoch))
    sets_b.update(sets_c)
    for t in range(T_all):
        for q in range(wl.W):
            assert np.array_equal(sets_a[t][q], sets_b[t][q]), (t, q)
    assert np.array_equal(f32bits(w_a.cpu().numpy()), f32bits(w_b.cpu().numpy()))
    sd.close()

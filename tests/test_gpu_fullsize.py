"""Full-size parity: the VGG-16-sized workload in the launch configuration bench.py times
(flat model, n = 138,357,544, W = 8, explorer draw announced ahead and made inside the scoring pass,
speculative packing with the capture bound of an earlier selection), the multi-iteration loop at the same size, and
the tie-heavy stress workload of the same length (W = 16, values rounded through binary16).

What the oracle can do at this size it does in full (score, random words, pack, merge:
all linear time, bit-exact over every element).  The two rankings would need a full
comparison sort of 1.4e8 pairs per call, so they are checked through the property that
defines them at any size: the chosen set is {key beyond the threshold} plus the lowest
indices among the keys equal to the threshold, the threshold being the k-th key by
np.partition.  That property fixes the set uniquely, so the comparison is still exact.
"""
import time

import numpy as np
import pytest

import oracle
from paper_1709_09393_amd import binding, workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def exact_top(keys_u32: np.ndarray, eligible, count: int, largest: bool) -> np.ndarray:
    """Indices of the `count` largest (or smallest) keys among eligible positions, ties to the lower index."""
    if count == 0:
        return np.zeros(0, np.uint32)
    idx = np.arange(keys_u32.size, dtype=np.uint32) if eligible is None else np.flatnonzero(eligible).astype(np.uint32)
    k = keys_u32 if eligible is None else keys_u32[idx]
    if largest:
        tau = np.partition(k, k.size - count)[k.size - count]
        sure = k > tau
    else:
        tau = np.partition(k, count - 1)[count - 1]
        sure = k < tau
    n_sure = int(sure.sum())
    ties = np.flatnonzero(k == tau)[: count - n_sure]          # flatnonzero is ascending: lowest indices first
    chosen = np.concatenate([np.flatnonzero(sure), ties])
    chosen.sort()
    return idx[chosen]


@pytest.mark.parametrize("wl", [workloads.VGG16, workloads.STRESS], ids=lambda x: x.name)
def test_full_size_iteration_matches(wl):
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but torch.cuda.is_available() is False")
    dev = torch.device("cuda:0")
    n, W, k, m = wl.n, wl.W, wl.k, wl.m
    it = 3
    t0 = time.time()
    w_h = wl.weights()
    g_h = wl.gradients(it)
    print("inputs drawn in %.1f s" % (time.time() - t0), flush=True)

    sd = binding.SlimDP(n, W, seed=workloads.EXPLORE_SEED)
    w = torch.from_numpy(w_h).to(dev)
    g = [torch.from_numpy(x).to(dev) for x in g_h]
    sd.set_option("speculative_pack", 1)
    sd.set_option("explore_async", 1)            # as bench.py runs it: the explorer request beside the pack of the core
    S = sd.score(w, g, wl.c)                     # as bench.py's warm-up does: a first selection sets the capture bound
    sd.select_core(S, [k], reuse_histogram=True)
    sd.explore_hint([k], it, [m], 0, W)
    S = sd.score(w, g, wl.c)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, [k], it, [m], 0, W)
    core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=True)
    sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
    sd.synchronize()
    print("GPU iteration done", flush=True)

    def u32(t):
        return t.cpu().numpy().view(np.uint32)

    # score: every element, bit-exact
    S_o = oracle.score(w_h, g_h, wl.c)
    assert np.array_equal(S.cpu().numpy().view(np.uint32), S_o.view(np.uint32)), "score bits"
    print("score ok (%.1f s)" % (time.time() - t0), flush=True)

    # core: the unique set fixed by the threshold property
    core_want = exact_top(S_o.view(np.uint32), None, k, largest=True)
    core_got = u32(core_idx)
    assert core_got.size == k and np.array_equal(core_got, core_want), "core set"
    ts = sd.tile_starts()
    assert np.array_equal(u32(core_off), np.searchsorted(core_want, ts.astype(np.int64)).astype(np.uint32))
    in_core = np.zeros(n, bool)
    in_core[core_want] = True
    bits_want = np.packbits(np.concatenate([in_core, np.zeros((-n) % 32, bool)]).reshape(-1, 32), axis=1,
                            bitorder="little").view(np.uint32).reshape(-1)
    assert np.array_equal(u32(core_bits), bits_want), "core bitmap"
    print("core ok (%.1f s)" % (time.time() - t0), flush=True)

    # explorers: every worker's set in full (the host work of several workers runs side by side)
    from concurrent.futures import ThreadPoolExecutor
    ei_got = [u32(x) for x in expl_idx]

    def check_explorer(q):
        words = oracle.explore_words(workloads.EXPLORE_SEED, it, q, 0, n)
        want = exact_top(words, ~in_core, m, largest=False)
        return np.array_equal(ei_got[q], want) and np.array_equal(
            u32(expl_off[q]), np.searchsorted(want, ts.astype(np.int64)).astype(np.uint32))
    with ThreadPoolExecutor(8) as pool:
        ok = list(pool.map(check_explorer, range(W)))
    assert all(ok), "explorer sets: %r" % ok
    print("all %d explorers ok (%.1f s)" % (W, time.time() - t0), flush=True)

    # packs: bit copies, every entry
    cv = [x.cpu().numpy() for x in core_val]
    ev = [x.cpu().numpy() for x in expl_val]
    for q in range(W):
        assert np.array_equal(cv[q].view(np.uint32), g_h[q][core_want].view(np.uint32)), q
        assert np.array_equal(ev[q].view(np.uint32), g_h[q][ei_got[q]].view(np.uint32)), q
    print("packs ok (%.1f s)" % (time.time() - t0), flush=True)

    # merge: the oracle in full
    w_o = oracle.merge(w_h, wl.lr, core_want, cv, ei_got, ev)
    w_g = w.cpu().numpy()
    assert np.all(np.abs(w_g - w_o) <= 1e-6 * np.abs(w_o) + 1e-12), "merge tolerance"
    assert np.array_equal(w_g.view(np.uint32), w_o.view(np.uint32)), "merge bits"
    print("merge ok (%.1f s)" % (time.time() - t0), flush=True)

    # the exact rerun of the explorer (zones forced to miss) at this size: one block per worker, about 0.4 s
    if wl.name == "vgg16_flat":
        sd.set_option("explore_force_fallback", 1)
        expl_idx2, expl_off2 = sd.sample_explore(core_bits, [k], it, [m], 0, W)
        sd.synchronize()
        q = W - 1
        words = oracle.explore_words(workloads.EXPLORE_SEED, it, q, 0, n)
        want = exact_top(words, ~in_core, m, largest=False)
        assert np.array_equal(u32(expl_idx2[q]), want), "exact rerun, explorer %d" % q
        assert np.array_equal(u32(expl_off2[q]), np.searchsorted(want, ts.astype(np.int64)).astype(np.uint32))
        assert np.array_equal(u32(expl_idx2[0]), ei_got[0]), "exact rerun, explorer 0"
        print("exact rerun ok (%.1f s)" % (time.time() - t0), flush=True)
    sd.close()


def test_full_size_loop_steady_path_matches():
    """The multi-iteration configuration at its stated size (n = 138,357,544, W = 8; core every 5 iterations,
    explorer every iteration, fresh updates per (iteration, worker) written into the SAME device buffers), six
    iterations: t = 0 the first selection of a fresh context, t = 1..4 steady iterations (core keys cached, the pack
    scans updates no scoring pass has seen, every draw announced one iteration ahead: on the side stream, or inside
    the scoring pass before a reselection; explorer requests on the side stream, one iteration ahead while the core stays), t = 5 a reselection whose capture bound comes from t = 0's selection on
    other updates.  Checked over every element: scores, both packs of a reselecting iteration (values kept by the
    scoring pass, and the scanning pack), merge, pull (+ local overwrite), ALL W explorer sets of every iteration,
    and one dense update + significance; the rankings through the threshold property."""
    from concurrent.futures import ThreadPoolExecutor
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but torch.cuda.is_available() is False")
    dev = torch.device("cuda:0")
    wl = workloads.LOOP
    n, W, k, m = wl.n, wl.W, wl.k, wl.m
    every = wl.reselect_every
    t0 = time.time()
    pool = ThreadPoolExecutor(8)
    sd = binding.SlimDP(n, W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    sd.set_option("explore_async", 1)
    w_h = wl.weights()
    w = torch.from_numpy(w_h).to(dev)
    g = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(W)]
    ahead = None                                            # explorer lists requested one iteration ahead
    ts = sd.tile_starts().astype(np.int64)
    rng = np.random.default_rng(5)
    local_h = rng.standard_normal(n).astype(np.float32)

    def u32(t):
        return t.cpu().numpy().view(np.uint32)

    core_want = in_core = None
    sd.explore_hint([k], 0, [m], 0, W)                     # the first draw rides inside the first scoring pass
    for t in range(6):
        g_h = list(pool.map(lambda q: wl.gradient(t, q), range(W)))
        for q in range(W):
            g[q].copy_(torch.from_numpy(g_h[q]))            # refilled in place
        resel = t % every == 0
        if resel:
            S = sd.score(w, g, wl.c)
            core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
        if ahead is not None:
            expl_idx, expl_off = ahead
        else:
            expl_idx, expl_off = sd.sample_explore(core_bits, [k], t, [m], 0, W)
        sd.set_option("explore_hint_mode", 0 if (t + 1) % every == 0 else 1)
        sd.explore_hint([k], t + 1, [m], 0, W)
        # the next iteration keeps the core: its explorer request goes out now and runs beside this pack and merge
        ahead = sd.sample_explore(core_bits, [k], t + 1, [m], 0, W) if (t + 1) % every != 0 else None
        core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=resel)
        if resel:                                           # the scanning pack of the same updates gives the same bits
            cv2, ev2 = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch)
        sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
        w_local = [None] * W
        if t in (1, 5):
            w_local[W - 1] = torch.from_numpy(local_h).to(dev)
        core_out, expl_out = sd.pull(w, epoch, core_idx, core_off, expl_idx, expl_off, w_local=w_local)
        sd.synchronize()
        print("t=%d GPU done (%.1f s)" % (t, time.time() - t0), flush=True)

        if resel:
            S_o = oracle.score(w_h, g_h, wl.c)
            assert np.array_equal(S.cpu().numpy().view(np.uint32), S_o.view(np.uint32)), "score bits, t=%d" % t
            core_want = exact_top(S_o.view(np.uint32), None, k, largest=True)
            assert np.array_equal(u32(core_idx), core_want), "core set, t=%d" % t
            assert np.array_equal(u32(core_off), np.searchsorted(core_want, ts).astype(np.uint32))
            in_core = np.zeros(n, bool)
            in_core[core_want] = True
            for q in range(W):
                assert torch.equal(cv2[q].view(torch.int32), core_val[q].view(torch.int32)), (t, q)
                assert torch.equal(ev2[q].view(torch.int32), expl_val[q].view(torch.int32)), (t, q)
            del cv2, ev2, S_o
        ei_got = [u32(x) for x in expl_idx]

        def check_explorer(q):
            words = oracle.explore_words(workloads.EXPLORE_SEED, t, q, 0, n)
            want = exact_top(words, ~in_core, m, largest=False)
            return np.array_equal(ei_got[q], want) and np.array_equal(
                u32(expl_off[q]), np.searchsorted(want, ts).astype(np.uint32))
        ok = list(pool.map(check_explorer, range(W)))
        assert all(ok), "explorer sets, t=%d: %r" % (t, ok)
        cv = [x.cpu().numpy() for x in core_val]
        ev = [x.cpu().numpy() for x in expl_val]
        for q in range(W):
            assert np.array_equal(cv[q].view(np.uint32), g_h[q][core_want].view(np.uint32)), (t, q)
            assert np.array_equal(ev[q].view(np.uint32), g_h[q][ei_got[q]].view(np.uint32)), (t, q)
        w_h = oracle.merge(w_h, wl.lr, core_want, cv, ei_got, ev)
        w_g = w.cpu().numpy()
        assert np.all(np.abs(w_g - w_h) <= 1e-6 * np.abs(w_h) + 1e-12), "merge tolerance, t=%d" % t
        assert np.array_equal(w_g.view(np.uint32), w_h.view(np.uint32)), "merge bits, t=%d" % t
        for q in range(W):
            assert np.array_equal(core_out[q].cpu().numpy().view(np.uint32), w_h[core_want].view(np.uint32)), (t, q)
            assert np.array_equal(expl_out[q].cpu().numpy().view(np.uint32), w_h[ei_got[q]].view(np.uint32)), (t, q)
        if w_local[W - 1] is not None:
            _, _, want_local = oracle.pull(w_h, core_want, ei_got[W - 1], local_h)
            assert np.array_equal(w_local[W - 1].cpu().numpy().view(np.uint32), want_local.view(np.uint32)), t
        del cv, ev, w_g, core_out, expl_out, w_local
        print("t=%d checked (%.1f s)" % (t, time.time() - t0), flush=True)

    # the iteration before a reselection as algorithm 1 has it: every update applied, significance of the new model
    S2 = sd.dense_update_score(w, g, wl.lr, wl.c)
    sd.synchronize()
    w_o, S_o = oracle.dense_update_score(w_h, g_h, wl.lr, wl.c)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_o.view(np.uint32)), "dense update bits"
    assert np.array_equal(S2.cpu().numpy().view(np.uint32), S_o.view(np.uint32)), "dense score bits"
    print("dense update ok (%.1f s)" % (time.time() - t0), flush=True)
    sd.close()
    pool.shutdown()


def test_full_size_worker_side_local_steps_and_fused_pack():
    """The worker side at the VGG-16 size (two of the eight workers, to keep the host's part short): a first local
    step, then the last step before the push with the extraction in the same pass, then the pull with local overwrite.
    Local models, accumulated updates and packs are compared with the oracle over every element; the index sets are the
    library's own (their parity is the business of the tests above)."""
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but torch.cuda.is_available() is False")
    dev = torch.device("cuda:0")
    wl = workloads.VGG16
    n, W, k, m = wl.n, 2, wl.k, wl.m
    eta = 0.05
    t0 = time.time()
    w_h = wl.weights()
    sd = binding.SlimDP(n, W, seed=workloads.EXPLORE_SEED)
    sd.set_option("explore_async", 1)
    w = torch.from_numpy(w_h).to(dev)
    core_idx, core_bits, core_off, epoch = sd.select_core(w.abs(), [k])
    expl_idx, expl_off = sd.sample_explore(core_bits, [k], 0, [m], 0, W)        # runs beside the local steps
    wk_h = [w_h.copy() for _ in range(W)]
    wk = [torch.from_numpy(x).to(dev) for x in wk_h]
    delta = [torch.full((n,), float("nan"), dtype=torch.float32, device=dev) for _ in range(W)]
    d_h = [None] * W
    for j in range(2):
        g_h = [wl.gradient(j, q) for q in range(W)]
        g = [torch.from_numpy(x).to(dev) for x in g_h]
        if j == 0:
            sd.local_step(wk, g, delta, eta, first=True)
        else:
            core_val, expl_val = sd.local_step_pack(wk, g, delta, eta, False, core_idx, core_off, expl_idx, expl_off, epoch)
        for q in range(W):
            wk_h[q], d_h[q] = oracle.local_step(wk_h[q], d_h[q], g_h[q], eta)
        del g
    sd.synchronize()
    print("local steps done at %.1f s" % (time.time() - t0), flush=True)
    ci = core_idx.cpu().numpy().view(np.uint32)
    for q in range(W):
        ei = expl_idx[q].cpu().numpy().view(np.uint32)
        assert ei.size == m and np.all(ei[1:] > ei[:-1])
        assert np.array_equal(wk[q].cpu().numpy().view(np.uint32), wk_h[q].view(np.uint32)), "local model %d" % q
        assert np.array_equal(delta[q].cpu().numpy().view(np.uint32), d_h[q].view(np.uint32)), "accumulated update %d" % q
        cv_o, ev_o = oracle.pack(d_h[q], ci, ei)
        assert np.array_equal(core_val[q].cpu().numpy().view(np.uint32), cv_o.view(np.uint32)), "core_val %d" % q
        assert np.array_equal(expl_val[q].cpu().numpy().view(np.uint32), ev_o.view(np.uint32)), "expl_val %d" % q
    # push, then pull with local overwrite: inside the communication set the local model equals the global one
    sd.merge(w, wl.lr, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
    sd.pull(w, epoch, core_idx, core_off, expl_idx, expl_off, w_local=wk)
    sd.synchronize()
    w_o = oracle.merge(w_h, wl.lr, ci, [oracle.pack(d_h[q], ci, expl_idx[q].cpu().numpy().view(np.uint32))[0] for q in range(W)],
                       [expl_idx[q].cpu().numpy().view(np.uint32) for q in range(W)],
                       [oracle.pack(d_h[q], ci, expl_idx[q].cpu().numpy().view(np.uint32))[1] for q in range(W)])
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_o.view(np.uint32)), "merged model"
    for q in range(W):
        ei = expl_idx[q].cpu().numpy().view(np.uint32)
        _, _, want = oracle.pull(w_o, ci, ei, wk_h[q])
        assert np.array_equal(wk[q].cpu().numpy().view(np.uint32), want.view(np.uint32)), "pulled local model %d" % q
    print("worker side checked at %.1f s" % (time.time() - t0), flush=True)
    sd.close()


@pytest.mark.parametrize("n", [2 ** 30 - 4089, 2 ** 30 + 12293, 2 ** 31], ids=["below_2_30", "above_2_30", "largest_2_31"])
def test_sizes_around_the_32_bit_byte_offset_limit(n, capsys):
    """A flat model just below 2^30 parameters (the largest the pipelined scoring kernel takes: its byte offsets reach
    2^32 - 16 KB), just above (the general kernels with 64-bit addresses; more than 2^18 tiles), and the largest model
    the interface takes (2^31 parameters: 8.6 GB per vector), one worker: score,
    core, explorer, pack and merge against the oracle as in the full-size test above.  Inputs: uniform values with only
    2^24 levels, so every threshold falls into a group of about a hundred equal keys (ties to the lower index)."""
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but torch.cuda.is_available() is False")
    dev = torch.device("cuda:0")
    W, it = 1, 5
    k, m = n // 10, (n - n // 10) // 50
    t0 = time.time()

    def say(what):
        with capsys.disabled():
            print("  [n=%d] %s (%.1f s)" % (n, what, time.time() - t0), flush=True)
    rng = np.random.default_rng(n)
    w_h = rng.random(n, dtype=np.float32)
    w_h -= np.float32(0.5)
    g_h = rng.random(n, dtype=np.float32)
    g_h -= np.float32(0.5)
    g_h *= np.float32(0.01)
    say("inputs drawn")
    sd = binding.SlimDP(n, W, seed=workloads.EXPLORE_SEED)
    sd.set_option("speculative_pack", 1)
    w = torch.from_numpy(w_h).to(dev)
    g = [torch.from_numpy(g_h).to(dev)]
    sd.explore_hint([k], it, [m], 0, W)
    S = sd.score(w, g, 1.0)
    core_idx, core_bits, core_off, epoch = sd.select_core(S, [k], reuse_histogram=True)
    expl_idx, expl_off = sd.sample_explore(core_bits, [k], it, [m], 0, W)
    core_val, expl_val = sd.pack(g, core_idx, core_off, expl_idx, expl_off, epoch, updates_as_scored=True)
    sd.merge(w, 0.01, epoch, core_idx, core_off, core_val, expl_idx, expl_off, expl_val)
    sd.synchronize()
    say("GPU iteration done")

    def u32(t):
        return t.cpu().numpy().view(np.uint32)
    S_o = oracle.score(w_h, [g_h], 1.0)
    assert np.array_equal(u32(S), S_o.view(np.uint32)), "score bits"
    del S
    say("score ok")
    core_want = exact_top(S_o.view(np.uint32), None, k, largest=True)
    del S_o
    assert np.array_equal(u32(core_idx), core_want), "core set"
    ts = sd.tile_starts()
    assert np.array_equal(u32(core_off), np.searchsorted(core_want, ts.astype(np.int64)).astype(np.uint32))
    in_core = np.zeros(n, bool)
    in_core[core_want] = True
    bits_want = np.packbits(np.concatenate([in_core, np.zeros((-n) % 32, bool)]).reshape(-1, 32), axis=1,
                            bitorder="little").view(np.uint32).reshape(-1)
    assert np.array_equal(u32(core_bits), bits_want), "core bitmap"
    del bits_want
    say("core ok")
    words = oracle.explore_words(workloads.EXPLORE_SEED, it, 0, 0, n)
    np.logical_not(in_core, out=in_core)
    want = exact_top(words, in_core, m, largest=False)
    del words, in_core
    ei = u32(expl_idx[0])
    assert np.array_equal(ei, want), "explorer set"
    assert np.array_equal(u32(expl_off[0]), np.searchsorted(want, ts.astype(np.int64)).astype(np.uint32))
    say("explorer ok")
    cv, ev = core_val[0].cpu().numpy(), expl_val[0].cpu().numpy()
    assert np.array_equal(cv.view(np.uint32), g_h[core_want].view(np.uint32)), "core_val"
    assert np.array_equal(ev.view(np.uint32), g_h[ei].view(np.uint32)), "expl_val"
    w_o = oracle.merge(w_h, 0.01, core_want, [cv], [ei], [ev])
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_o.view(np.uint32)), "merge bits"
    say("packs and merge ok")
    sd.close()

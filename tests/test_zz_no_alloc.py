"""The allocation-free entry point slimdp_select_core_static against slimdp_select_core (context) through the C ABI:
bit-exact index list, bitmap and tile offsets, on two calls in a row, the second with a smaller input (the static
workspace keeps the first call's contents)."""
import numpy as np
import pytest

import oracle
from paper_1709_09393_amd import binding, workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def test_static_selection_matches_the_context_call_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but torch.cuda.is_available() is False")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    for n, pct, stress in [(1 << 20, 10, False), (1_000_003, 10, False), (300_001, 37, True), (4097, 50, False), (5, 40, False)]:
        wl = (workloads.STRESS if stress else workloads.TINY).scaled(n, core_pct=pct)
        k = wl.k
        S_h = oracle.score(wl.weights(), wl.gradients(0), wl.c)
        S = torch.from_numpy(S_h).to(dev)
        T = binding.num_tiles(n)
        core_idx = torch.full((k,), -1, dtype=torch.int32, device=dev)
        core_bits = torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device=dev)
        core_off = torch.full((T + 1,), -1, dtype=torch.int32, device=dev)
        before = torch.cuda.memory_allocated()
        binding.select_core_static(S, k, core_idx, core_bits, core_off)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        sd = binding.SlimDP(n, 1)
        want_idx, want_bits, want_off, _ = sd.select_core(S, [k])
        sd.synchronize()
        assert np.array_equal(u32(core_idx), u32(want_idx)), n
        assert np.array_equal(u32(core_bits), u32(want_bits)), n
        assert np.array_equal(u32(core_off), u32(want_off)), n
        assert np.array_equal(u32(core_idx), oracle.select_core(S_h, k)), n
        sd.close()
    # beyond the stated maximum: refused, nothing launched
    big = torch.zeros(binding.STATIC_MAX_N + 1, dtype=torch.float32, device=dev)
    with pytest.raises(binding.SlimDPError) as e:
        binding.select_core_static(big, 1, core_idx, core_bits, core_off)
    assert e.value.code == binding.ERR_OUT_OF_RANGE and "SLIMDP_STATIC_MAX_N" in str(e.value)
    with pytest.raises(binding.SlimDPError) as e:
        binding.select_core_static(S, S.numel() + 1, core_idx, core_bits, core_off)
    assert e.value.code == binding.ERR_OUT_OF_RANGE

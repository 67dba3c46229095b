"""pac_build_mask on weights with very many equal magnitudes, bit for bit against the oracle: the weights
a training loop really holds (Eq. 2 keeps pruned weights at exactly zero, so a fraction s of them is 0),
constant tensors, several tie values, ties that straddle tile and scope boundaries, and the cut through
the ties falling at every kind of position.  Large enough for the sampled first pass (above 4M elements
per scope) and for the exact one.  Also checks that these inputs stay on the fast code path."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


def check(pac, w, offsets, sp, expect_fast=True, label=""):
    dev = w.device
    n = w.numel()
    nseg = len(offsets) - 1
    ctx = pac.PacContext(max_elems=n, max_segments=nseg, device=0)
    try:
        mask, prefix, nnz = ctx.build_mask(w, offsets, sp)
        torch.cuda.synchronize()
        st = ctx.device_status()
        em, ep, k = oracle.build_mask(w.cpu().numpy(), offsets, sp)
        assert nnz == k
        got = mask.cpu().numpy().view(np.uint64)
        if not np.array_equal(got, em):
            bad = np.flatnonzero(got != em)
            raise AssertionError(f"{label}: {bad.size} mask words differ, first at word {bad[0]} (element {bad[0] * 64}); "
                                 f"status {st:#x}")
        assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep), f"{label}: prefix differs"
        assert st & pac.PAC_DEV_ERROR_MASK == 0, f"{label}: status {st:#x}"
        if expect_fast:
            assert st & pac.PAC_DEV_SLOW_PATH == 0, f"{label}: took the slow path (status {st:#x})"
        return st
    finally:
        ctx.close()


def gaussian(n, dev, seed):
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    return torch.randn(n, device=dev, generator=gen) * 0.02


@pytest.mark.parametrize("n", [6_000_037, 1_500_003])
@pytest.mark.parametrize("s_prev,s_now", [(0.9, 0.9), (0.5, 0.5), (0.9, 0.8), (0.8, 0.9), (0.95, 0.5)])
def test_weights_of_an_already_pruned_model(n, s_prev, s_now):
    """Prune at s_prev (pruned weights become exact zeros), then build the mask at s_now: same sparsity (the
    steady state: k equals the number of non-zeros), a lower one (the cut falls among the zeros) and a
    higher one."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    w = gaussian(n, dev, 7)
    ctx = pac.PacContext(max_elems=n, device=0)
    mask, prefix, nnz = ctx.build_mask(w, [0, n], s_prev)
    zero_grad = torch.zeros(nnz, device=dev)
    ctx.decompress_update(zero_grad, mask, prefix, 0.0, w, nnz)      # the library's own re-zeroing of pruned weights
    torch.cuda.synchronize()
    ctx.close()
    assert int((w == 0).sum().item()) == n - nnz
    check(pac, w, [0, n], [s_now], label=f"pruned {s_prev}->{s_now}")


@pytest.mark.parametrize("n", [9_000_001, 4096 * 300 + 17])
@pytest.mark.parametrize("s", [0.9, 0.5, 0.000001, 0.999999, 0.3333])
def test_one_constant_scope(n, s):
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    w = torch.full((n,), 0.02, device=dev)
    w[::3] = -0.02                                   # the sign does not matter
    check(pac, w, [0, n], [s], label=f"constant s={s}")


def test_two_tie_values_and_a_continuous_rest():
    """40 % zeros, 30 % of one magnitude, the rest Gaussian, cut at several ranks - inside either tie value
    and inside the continuous part.  Only one key can be the tie key: the other value's elements are listed
    or walked, which may be the slow path."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 7_000_003
    w = gaussian(n, dev, 21)
    gen = torch.Generator(device=dev)
    gen.manual_seed(22)
    u = torch.rand(n, device=dev, generator=gen)
    w[u < 0.4] = 0.0
    w[(u >= 0.4) & (u < 0.7)] = 0.015
    for s in (0.2, 0.45, 0.7, 0.85, 0.95):
        check(pac, w, [0, n], [s], expect_fast=False, label=f"two ties s={s}")


def test_ties_across_scope_and_tile_boundaries():
    """Per-tensor scopes whose boundaries fall inside tiles; constant, zero-heavy and continuous tensors side
    by side, small scopes between the large ones, a ragged end."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    sizes = [5_000_011, 100, 70_001, 4_500_000, 33, 40_000, 6_100_777, 2_000_003, 50_001]
    offsets = [0]
    for z in sizes:
        offsets.append(offsets[-1] + z)
    n = offsets[-1]
    w = gaussian(n, dev, 31)
    gen = torch.Generator(device=dev)
    gen.manual_seed(32)
    u = torch.rand(n, device=dev, generator=gen)
    o = offsets
    w[o[0]:o[1]][u[o[0]:o[1]] < 0.9] = 0.0              # pruned at 0.9
    w[o[1]:o[2]] = 1.0                                   # a norm vector
    w[o[3]:o[4]] = -0.5                                  # constant large scope
    w[o[6]:o[7]][u[o[6]:o[7]] < 0.5] = 0.0
    w[o[7]:o[8]] = 0.0                                   # all zero
    for sp in ([0.9, 0.9, 0.5, 0.3, 0.0, 0.8, 0.5, 0.6, 0.7], [0.5] * 9, [0.95, 0.1, 0.9, 0.999, 1.0, 0.2, 0.9, 0.0, 0.5]):
        check(pac, w, offsets, sp, label=f"boundaries {sp[0]}")


@pytest.mark.parametrize("s", [0.999999, 0.99999, 0.00001])
def test_extreme_sparsity_on_a_sampled_scope(s):
    """k of a few elements (or all but a few) in a scope large enough to be sampled: the bracket spans
    thousands of first-digit bins."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 8_000_009
    w = gaussian(n, dev, 41)
    w[12345] = 3.0e8
    w[777] = -1.0e-30
    check(pac, w, [0, n], [s], expect_fast=False, label=f"extreme s={s}")


def test_cut_at_every_kind_of_position_inside_the_ties():
    """A constant scope cut exactly at tile boundaries, word boundaries, first and last element."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 4096 * 1200
    w = torch.full((n,), 0.25, device=dev)
    ctx = pac.PacContext(max_elems=n, device=0)
    try:
        for k in (1, 63, 64, 65, 4095, 4096, 4097, 4096 * 600, 4096 * 600 + 1, n - 4096, n - 1):
            s = 1.0 - k / n
            s = round(s, 6)
            kk = pac.pac_keep_count(n, s)
            mask, prefix, nnz = ctx.build_mask(w, [0, n], s)
            assert nnz == kk
            got = mask.cpu().numpy().view(np.uint64)
            want = np.zeros(n // 64, dtype=np.uint64)
            want[:kk // 64] = np.uint64(0xFFFFFFFFFFFFFFFF)
            if kk % 64:
                want[kk // 64] = np.uint64((1 << (kk % 64)) - 1)
            assert np.array_equal(got, want), f"k={kk}"
        assert ctx.device_status() & (pac.PAC_DEV_ERROR_MASK | pac.PAC_DEV_SLOW_PATH) == 0
    finally:
        ctx.close()

"""The device status word: what only the device can see (a count that does not match the mask, metadata
that does not fit together, a bounded wait that gave up) reaches the caller through pac_device_status.
Every kernel here exits normally: the give-up is forced from the host with a spin limit of zero."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


def _ctx_and_mask(pac, n, s, dev, seed=5):
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    w = torch.randn(n, device=dev, generator=gen)
    ctx = pac.PacContext(max_elems=n, device=0)
    mask, prefix, nnz = ctx.build_mask(w, [0, n], s)
    torch.cuda.synchronize()
    return ctx, w, mask, prefix, nnz


def test_status_is_clear_after_an_ordinary_step_and_reads_are_repeatable():
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 300007
    ctx, w, mask, prefix, nnz = _ctx_and_mask(pac, n, 0.75, dev)
    try:
        g = torch.randn(n, device=dev)
        c = ctx.compress(g, mask, prefix, nnz)
        out = ctx.decompress(c, mask, prefix, n, nnz)
        ctx.decompress_update(c, mask, prefix, 0.5, w.clone(), nnz)
        assert ctx.device_status() == 0
        flags = torch.full((1,), -1, dtype=torch.int32, device=dev)
        assert pac.pac_device_status(ctx.handle, flags, to_host=False) is None
        torch.cuda.synchronize()
        assert int(flags.item()) == 0
        assert out.numel() == n
    finally:
        ctx.close()


def test_scan_give_up_is_reported_and_sticky_until_cleared():
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = (1 << 26) + 77                       # 129 scan tiles
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    w = torch.randn(n, device=dev, generator=gen)
    ctx = pac.PacContext(max_elems=n, device=0)
    try:
        pac.pac_debug_set_scan_spin_limit(ctx.handle, 0)      # a workgroup gives up instead of waiting
        ctx.build_mask(w, [0, n], 0.9)
        st = ctx.device_status()
        assert st & pac.PAC_DEV_SCAN_STALLED, f"status {st:#x}"
        # sticky: later good calls do not clear it, a clearing read does
        pac.pac_debug_set_scan_spin_limit(ctx.handle, 1 << 22)
        mask, prefix, nnz = ctx.build_mask(w, [0, n], 0.9)
        assert ctx.device_status() & pac.PAC_DEV_SCAN_STALLED
        assert ctx.device_status(clear=True) & pac.PAC_DEV_SCAN_STALLED
        assert ctx.device_status() == 0
        em, ep, k = oracle.build_mask(w.cpu().numpy(), [0, n], 0.9)
        assert k == nnz
        assert np.array_equal(mask.cpu().numpy().view(np.uint64), em)
        assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep)
    finally:
        ctx.close()


@pytest.mark.parametrize("dtype,offset", [(torch.float32, 0), (torch.bfloat16, 0), (torch.float32, 1)])
def test_a_wrong_count_is_reported(dtype, offset):
    """nnz passed != the mask's own bit count: the call cannot know on the host; the device says so."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 200003
    ctx, w, mask, prefix, nnz = _ctx_and_mask(pac, n, 0.6, dev)
    try:
        g = torch.randn(n + offset, device=dev).to(dtype)[offset:]        # offset 1: the element-wise kernels
        guard = 16
        c = torch.zeros(nnz + guard, dtype=dtype, device=dev)
        pac.pac_compress(ctx.handle, g, mask, prefix, c, nnz - 3)
        st = ctx.device_status(clear=True)
        assert st & pac.PAC_DEV_COUNT_MISMATCH, f"status {st:#x}"
        assert torch.count_nonzero(c[nnz - 3:].view(torch.int16 if dtype == torch.bfloat16 else torch.int32)) == 0
        pac.pac_compress(ctx.handle, g, mask, prefix, c, nnz)
        assert ctx.device_status(clear=True) == 0
        d = torch.empty(n + offset, dtype=dtype, device=dev)[offset:]
        pac.pac_decompress(ctx.handle, c, mask, prefix, d, nnz - 3)
        assert ctx.device_status(clear=True) & pac.PAC_DEV_COUNT_MISMATCH
        pac.pac_decompress(ctx.handle, c, mask, prefix, d, nnz)
        assert ctx.device_status(clear=True) == 0
        wts = torch.zeros(n + offset, dtype=torch.float32, device=dev)[offset:] if dtype == torch.float32 else torch.zeros(n, device=dev)
        pac.pac_decompress_update(ctx.handle, c, mask, prefix, 0.1, wts, nnz - 1)
        assert ctx.device_status(clear=True) & pac.PAC_DEV_COUNT_MISMATCH
    finally:
        ctx.close()


def test_metadata_that_does_not_fit_together_is_reported():
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 200003
    ctx, w, mask, prefix, nnz = _ctx_and_mask(pac, n, 0.6, dev)
    try:
        bad_prefix = torch.flip(prefix, dims=[0]).contiguous()            # descending: a tile ends before it starts
        g = torch.randn(n, device=dev)
        c = torch.zeros(nnz + 16, dtype=torch.float32, device=dev)
        pac.pac_compress(ctx.handle, g, mask, bad_prefix, c, nnz)
        st = ctx.device_status(clear=True)
        assert st & pac.PAC_DEV_META_MISMATCH, f"status {st:#x}"
        assert torch.count_nonzero(c[nnz:]) == 0
        d = torch.empty(n, device=dev)
        pac.pac_decompress(ctx.handle, c, mask, bad_prefix, d, nnz)
        assert ctx.device_status(clear=True) & pac.PAC_DEV_META_MISMATCH
    finally:
        ctx.close()


def test_build_mask_checks_its_own_count_on_the_device():
    """The scan's last tile compares the mask's bit count with the sum of the keep counts: clean on every
    kind of scope table (ties, empty and tiny scopes, sampled scopes)."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    n = 5_000_011
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    w = torch.randn(n, device=dev, generator=gen)
    w[1000:3000] = 1.0
    w[500000:900000] = 0.0
    offsets = [0, 0, 17, 4096, 70000, 70000, 1_000_000, n]
    sp = [0.5, 0.3, 0.9, 0.5, 0.1, 0.8, 0.9]
    ctx = pac.PacContext(max_elems=n, max_segments=len(sp), device=0)
    try:
        mask, prefix, nnz = ctx.build_mask(w, offsets, sp)
        st = ctx.device_status()
        assert st & pac.PAC_DEV_ERROR_MASK == 0, f"status {st:#x}"
        em, ep, k = oracle.build_mask(w.cpu().numpy(), offsets, sp)
        assert k == nnz and np.array_equal(mask.cpu().numpy().view(np.uint64), em)
    finally:
        ctx.close()


def _mask_equals_oracle(ctx, w, s):
    n = w.numel()
    mask, prefix, nnz = ctx.build_mask(w, [0, n], s)
    torch.cuda.synchronize()
    em, ep, k = oracle.build_mask(w.cpu().numpy(), [0, n], s)
    assert nnz == k
    assert np.array_equal(mask.cpu().numpy().view(np.uint64), em)
    assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep)


def test_informational_bits_name_the_slower_exact_path_that_ran():
    """Two inputs built to leave the fast path: magnitudes constant over each 16384-element tile (a sample of
    tiles then predicts the quantile badly: the sampled bracket misses and the full-count round runs), and two
    neighbouring magnitudes with hundreds of thousands of elements each, cut inside the one that is not the tie
    key (its elements exceed what the final selection holds in LDS, so the scope is resolved from its weights).
    The masks are the oracle's either way; the status word says which path produced them, and no error bit."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    rng = np.random.default_rng(52)
    tile, tiles = 16384, 1300
    n = tiles * tile + 77
    per_tile = (rng.random(tiles + 1) * 4.0 + 0.01).astype(np.float32)
    w = torch.from_numpy(np.repeat(per_tile, tile)[:n].copy()).to(dev)
    ctx = pac.PacContext(max_elems=n, device=0)
    try:
        seen = 0
        for s in (0.3, 0.5, 0.77):
            _mask_equals_oracle(ctx, w, s)
            seen |= ctx.device_status(clear=True)
        assert seen & pac.PAC_DEV_ERROR_MASK == 0, f"status {seen:#x}"
        assert seen & pac.PAC_DEV_RETRY_TAKEN, f"no sampled bracket missed (status {seen:#x})"
    finally:
        ctx.close()

    n = 1_000_003
    u = torch.from_numpy(rng.random(n)).to(dev)
    w = torch.full((n,), 1.0, device=dev)
    w[u < 0.4] = float(np.nextafter(np.float32(1.0), np.float32(2.0)))
    ctx = pac.PacContext(max_elems=n, device=0)
    try:
        _mask_equals_oracle(ctx, w, 0.8)            # the 200,001-st largest lies inside the 40 % group
        st = ctx.device_status(clear=True)
        assert st & pac.PAC_DEV_ERROR_MASK == 0, f"status {st:#x}"
        assert st & pac.PAC_DEV_SLOW_PATH, f"the scope was not resolved from its weights (status {st:#x})"
        assert ctx.device_status() == 0
    finally:
        ctx.close()

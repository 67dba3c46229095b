"""GPU parity of the Mask Tracker calls and of the fused decompress + weight update against the CPU
oracle: masks, prefix entries, counts and difference counts bit-exact; updated weights bit-exact
(one fp32 multiply and one fp32 subtract per kept element, no contraction on either side).
"""
import numpy as np
import pytest
import torch

import oracle
from synth import make_workload

pytestmark = pytest.mark.gpu

SPECIAL_F32 = np.array([0.0, -0.0, 1.0, -1.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 3.0e38], dtype=np.float32)


@pytest.fixture(scope="module")
def pac():
    import paper_2505_18563_amd as pac_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pac_mod


@pytest.fixture(scope="module")
def ctx(pac):
    c = pac.PacContext(max_elems=1 << 25, max_segments=64, device=0)
    yield c
    c.close()


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def same_floats(got: np.ndarray, want: np.ndarray) -> bool:
    """Bit-exact, except that a NaN only has to be a NaN: IEEE 754 leaves the sign and payload of a
    NaN produced by an arithmetic operation open, and the host and the GPU choose differently."""
    gn, wn = np.isnan(got), np.isnan(want)
    return np.array_equal(gn, wn) and np.array_equal(got.view(np.uint32)[~gn], want.view(np.uint32)[~wn])


def bf16_from_u16(u):
    return torch.from_numpy(u.view(np.int16).copy()).cuda().view(torch.bfloat16)


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def sparse_values(n, seed, dtype):
    rng = np.random.default_rng(seed)
    v = rng.standard_normal(n).astype(np.float32)
    v[rng.random(n) < 0.7] = 0.0
    v[rng.random(n) < 0.05] = -0.0
    if n >= SPECIAL_F32.size:
        v[:SPECIAL_F32.size] = SPECIAL_F32
        v[-1] = 5.0
    if dtype == "bf16":
        return oracle.f32_to_bf16(v)
    return v


# ------------------------------------------------------------------ pac_mask_from_nonzero
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 3, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 8191, 100003, 1 << 20, 3000001])
def test_mask_from_nonzero(ctx, dtype, n):
    v = sparse_values(n, 1000 + n, dtype)
    code = oracle.F32 if dtype == "f32" else oracle.BF16
    em, ep, ennz = oracle.mask_from_nonzero(v, code)
    t = dev(v) if dtype == "f32" else bf16_from_u16(v)
    mask, prefix, nnz = ctx.mask_from_nonzero(t)
    torch.cuda.synchronize()
    assert int(nnz.item()) == ennz
    assert np.array_equal(u64(mask), em)
    assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("offset", [1, 2, 3, 5])
def test_mask_from_nonzero_unaligned_pointer(ctx, dtype, offset):
    n = 70001
    v = sparse_values(n + offset, 77 + offset, dtype)
    code = oracle.F32 if dtype == "f32" else oracle.BF16
    em, ep, ennz = oracle.mask_from_nonzero(v[offset:], code)
    t = (dev(v) if dtype == "f32" else bf16_from_u16(v))[offset:]
    mask, prefix, nnz = ctx.mask_from_nonzero(t)
    assert int(nnz.item()) == ennz and np.array_equal(u64(mask), em)
    assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep)


def test_mask_from_nonzero_all_bf16_patterns(ctx):
    pat = np.arange(65536, dtype=np.uint16)
    em, ep, ennz = oracle.mask_from_nonzero(pat, oracle.BF16)
    mask, prefix, nnz = ctx.mask_from_nonzero(bf16_from_u16(pat))
    assert int(nnz.item()) == ennz == 65534 and np.array_equal(u64(mask), em)


def test_mask_from_nonzero_of_pruned_weights_is_the_prune_mask(ctx, pac):
    """Eq. 2 on a pruned model: (Weight != 0) gives back the prune mask, minus kept weights that are
    exactly zero (the workload's zero-initialised bias vectors)."""
    wl = make_workload(2, device=torch.device("cuda", 0), with_grads=False)
    sp = wl.sparsity_at(0)
    big = pac.PacContext(max_elems=wl.n, max_segments=len(sp), device=0)
    try:
        pm, pp, k = big.build_mask(wl.weights, wl.scope_offsets, sp)
        pruned = big.decompress(big.compress(wl.weights, pm, pp, k), pm, pp, wl.n, k)
        m, p, nnz = big.mask_from_nonzero(pruned)
        em, ep, ennz = oracle.mask_from_nonzero(pruned.cpu().numpy())
        assert int(nnz.item()) == ennz and np.array_equal(u64(m), em)
        assert np.array_equal(p.cpu().numpy().view(np.uint32), ep)
        assert int((m & ~pm).abs().sum()) == 0                       # a subset of the prune mask
        assert k - ennz == int((pruned == 0).sum()) - (wl.n - k)     # missing bits = kept weights equal to zero
    finally:
        big.close()


def test_mask_from_nonzero_empty_and_too_long(ctx, pac):
    mask = torch.empty(0, dtype=torch.int64, device="cuda")
    prefix = torch.empty(0, dtype=torch.int32, device="cuda")
    nnz = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    pac.pac_mask_from_nonzero(ctx.handle, torch.empty(0, device="cuda"), mask, prefix, nnz)
    assert int(nnz.item()) == 0
    small = pac.PacContext(max_elems=1000, device=0)
    try:
        with pytest.raises(pac.PacError) as e:
            small.mask_from_nonzero(torch.zeros(2000, device="cuda"))
        assert e.value.status == -3
    finally:
        small.close()


# ------------------------------------------------------------------ pac_mask_equal
@pytest.mark.parametrize("n", [1, 63, 64, 65, 1000, 70001, 1 << 22, 5000003])
def test_mask_equal(ctx, n):
    rng = np.random.default_rng(n)
    words = (n + 63) // 64
    a = rng.integers(0, 2**63, size=words, dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, size=words, dtype=np.uint64)
    b = a.copy()
    flips = rng.choice(n, size=min(n, 101), replace=False)
    for i in flips:
        b[i >> 6] ^= np.uint64(1) << np.uint64(i & 63)
    want = oracle.mask_diff(a, b, n)
    assert want == flips.size
    ta, tb = dev(a.view(np.int64)), dev(b.view(np.int64))
    assert int(ctx.mask_equal(ta, tb, n).item()) == want
    assert int(ctx.mask_equal(ta, ta, n).item()) == 0
    # garbage in the bits at and beyond n does not count
    if n % 64:
        c = b.copy()
        c[-1] |= ~((np.uint64(1) << np.uint64(n % 64)) - np.uint64(1))
        assert int(ctx.mask_equal(ta, dev(c.view(np.int64)), n).item()) == oracle.mask_diff(a, c, n) == want


# ------------------------------------------------------------------ tracker
def test_tracker_follows_the_oracle_bookkeeping(ctx, pac):
    n = 300007
    rng = np.random.default_rng(5)
    words = (n + 63) // 64
    A = rng.integers(0, 2**62, size=words, dtype=np.uint64)
    A[-1] &= (np.uint64(1) << np.uint64(n % 64)) - np.uint64(1)
    B = A.copy()
    B[words // 2] ^= np.uint64(1) << np.uint64(17)
    seq = [A, A, A, B, B, B, B, A, A]
    ref = oracle.MaskTracker(patience=2)
    tr = pac.MaskTracker(ctx, max_elems=n, patience=2)
    try:
        for m in seq:
            want = ref.update(m, n)
            got = tr.update(dev(m.view(np.int64)), n).cpu().numpy()
            assert (int(got[0]), bool(got[1])) == want
        # another length counts as a change
        want = ref.update(A[:100], 6400)
        got = tr.update(dev(A[:100].view(np.int64)), 6400).cpu().numpy()
        assert (int(got[0]), bool(got[1])) == want == (0, False)
        with pytest.raises(pac.PacError) as e:                     # longer than the tracker was sized for
            tr.update(torch.zeros(words + 1, dtype=torch.int64, device="cuda"), n + 64)
        assert e.value.status == -3
    finally:
        tr.close()


def test_dense_fallback_is_the_same_sum_over_dense_buffers(ctx):
    # unstable mask -> full synchronisation: the W-way sum over the dense gradients themselves
    n, W = 100003, 5
    rng = np.random.default_rng(9)
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
    out = ctx.reduce_local([dev(x) for x in g], n)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.reduce_local(g).view(np.uint32))


# ------------------------------------------------------------------ pac_decompress_update
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,s", [(1, 0.0), (5, 0.5), (511, 0.5), (512, 0.9), (513, 0.1), (4099, 0.9), (100003, 0.5),
                                 (1 << 20, 0.9), (3000001, 0.99), (70000, 0.0), (70000, 1.0)])
def test_decompress_update(ctx, dtype, n, s):
    rng = np.random.default_rng(n * 7 + int(s * 100))
    x = rng.standard_normal(n).astype(np.float32)
    em, ep, k = oracle.build_mask(x, [0, n], s)
    g = (rng.standard_normal(k) * 4).astype(np.float32)
    if k >= 3:
        g[0], g[1], g[2] = np.float32(np.inf), np.float32(np.nan), np.float32(-0.0)
    alpha = 0.0375
    if dtype == "bf16":
        gu = oracle.f32_to_bf16(g)
        want = oracle.decompress_update(gu, em, x, alpha, oracle.BF16)
        red = bf16_from_u16(gu)
    else:
        want = oracle.decompress_update(g, em, x, alpha, oracle.F32)
        red = dev(g)
    w = dev(x)
    ctx.decompress_update(red, dev(em.view(np.int64)), dev(ep.view(np.int32)), alpha, w, k)
    assert same_floats(w.cpu().numpy(), want)


@pytest.mark.parametrize("offset", [1, 2, 3])
def test_decompress_update_unaligned_weights(ctx, offset):
    n = 50001
    rng = np.random.default_rng(offset)
    x = rng.standard_normal(n).astype(np.float32)
    em, ep, k = oracle.build_mask(x, [0, n], 0.8)
    g = rng.standard_normal(k).astype(np.float32)
    want = oracle.decompress_update(g, em, x, 0.5)
    buf = torch.zeros(n + offset, device="cuda")
    w = buf[offset:]
    w.copy_(dev(x))
    ctx.decompress_update(dev(g), dev(em.view(np.int64)), dev(ep.view(np.int32)), 0.5, w, k)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert float(buf[:offset].abs().sum()) == 0.0


def test_update_equals_unfused_path_on_a_whole_step(ctx):
    """mask -> compress x W -> sum -> (decompress; x - alpha*g; re-mask) equals the fused call."""
    wl = make_workload(1, device=torch.device("cuda", 0))
    sp = wl.sparsity_at(0)
    mask, prefix, k = ctx.build_mask(wl.weights, wl.scope_offsets, sp)
    red = ctx.reduce_local([ctx.compress(g, mask, prefix, k) for g in wl.grads], k)
    w_np = wl.weights.cpu().numpy()
    em, ep, ek = oracle.build_mask(w_np, wl.scope_offsets, sp)
    code = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    raw = (lambda t: t.cpu().numpy()) if code == oracle.F32 else (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16))
    e_red = oracle.reduce_local([oracle.compress(raw(g), em, ek, code) for g in wl.grads], code)
    alpha = 0.01 / wl.workers
    want = oracle.decompress_update(e_red, em, w_np, alpha, code)
    w = wl.weights.clone()
    ctx.decompress_update(red, mask, prefix, alpha, w, k)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_decompress_update_error_codes(ctx, pac):
    w = torch.zeros(100, device="cuda")
    mask = torch.zeros(2, dtype=torch.int64, device="cuda")
    prefix = torch.zeros(2, dtype=torch.int32, device="cuda")
    red = torch.zeros(10, device="cuda")
    with pytest.raises(pac.PacError) as e:
        pac.pac_decompress_update(ctx.handle, torch.zeros(200, device="cuda"), mask, prefix, 1.0, w, 101)
    assert e.value.status == -4
    with pytest.raises(TypeError):
        pac.pac_decompress_update(ctx.handle, red, mask, prefix, 1.0, w.to(torch.bfloat16), 10)

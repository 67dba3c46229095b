"""GPU parity of the ternary payload calls (Sec. III-D) against the CPU oracle: the scale bit-exact, every
2-bit code equal (both sides draw from the same counter-based generator and take the keep decision in
single precision), the scaled integer sum bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from synth import make_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pac():
    import paper_2505_18563_amd as pac_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pac_mod


@pytest.fixture(scope="module")
def ctx(pac):
    c = pac.PacContext(max_elems=1 << 22, max_segments=4, device=0)
    yield c
    c.close()


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def bf16_from_u16(u):
    return torch.from_numpy(u.view(np.int16).copy()).cuda().view(torch.bfloat16)


def values(count, seed, dtype):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(count) * 0.01).astype(np.float32)
    g[rng.random(count) < 0.1] = 0.0
    if count >= 8:
        g[1], g[2], g[3], g[5] = np.float32(np.nan), np.float32(-0.0), np.float32(0.2), np.float32(-0.2)
    if dtype == "bf16":
        return oracle.f32_to_bf16(g)
    return g


def to_dev(v, dtype):
    return dev(v) if dtype == "f32" else bf16_from_u16(v)


SIZES = [1, 3, 4, 5, 7, 8, 9, 255, 256, 1023, 1025, 100003, (1 << 20) + 5]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("count", SIZES)
def test_absmax_and_ternarize(pac, ctx, dtype, count):
    code = oracle.F32 if dtype == "f32" else oracle.BF16
    v = values(count, 31 * count + 7, dtype)
    t = to_dev(v, dtype)
    scale = torch.full((1,), -5.0, device="cuda")
    pac.pac_absmax(ctx.handle, t, scale)
    want_scale = oracle.absmax(v, code)
    assert np.float32(scale.item()).view(np.uint32) == np.float32(want_scale).view(np.uint32)
    packed = torch.full(((count + 3) // 4,), 0xFF, dtype=torch.uint8, device="cuda")
    seed, stream_id = 0xA5A5A5A512345678, 3 + count
    pac.pac_ternarize(ctx.handle, t, scale, seed, stream_id, packed)
    want = oracle.ternarize(v, want_scale, seed, stream_id, code)
    assert np.array_equal(packed.cpu().numpy(), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("offset", [1, 2, 3])
def test_absmax_and_ternarize_unaligned_input(pac, ctx, dtype, offset):
    count = 5003
    code = oracle.F32 if dtype == "f32" else oracle.BF16
    v = values(count + offset, 5 + offset, dtype)
    t = to_dev(v, dtype)[offset:]
    scale = torch.zeros(1, device="cuda")
    pac.pac_absmax(ctx.handle, t, scale)
    want_scale = oracle.absmax(v[offset:], code)
    assert float(scale.item()) == want_scale
    packed = torch.empty((count + 3) // 4, dtype=torch.uint8, device="cuda")
    pac.pac_ternarize(ctx.handle, t, scale, 11, 22, packed)
    assert np.array_equal(packed.cpu().numpy(), oracle.ternarize(v[offset:], want_scale, 11, 22, code))


def test_absmax_accumulates_the_shared_scale(pac, ctx):
    rng = np.random.default_rng(2)
    bufs = [(rng.standard_normal(10007) * (w + 1)).astype(np.float32) for w in range(4)]
    scale = torch.zeros(1, device="cuda")
    want = 0.0
    for w, b in enumerate(bufs):
        pac.pac_absmax(ctx.handle, dev(b), scale, accumulate=w > 0)
        want = oracle.absmax(b, start=want if w > 0 else None)
    assert float(scale.item()) == want == max(float(np.max(np.abs(b))) for b in bufs)
    pac.pac_absmax(ctx.handle, torch.empty(0, device="cuda"), scale)     # empty buffer: zero
    assert float(scale.item()) == 0.0


@pytest.mark.parametrize("s", [0.0, -1.0, float("inf"), float("nan")])
def test_ternarize_unusable_scale(pac, ctx, s):
    g = values(1000, 3, "f32")
    packed = torch.full((250,), 0xFF, dtype=torch.uint8, device="cuda")
    pac.pac_ternarize(ctx.handle, dev(g), torch.tensor([s], device="cuda"), 1, 2, packed)
    assert int(packed.sum()) == 0


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("W,count", [(1, 1), (2, 5), (3, 8), (8, 1001), (16, 100003), (64, 4099)])
def test_ternary_reduce(pac, ctx, out_dtype, W, count):
    rng = np.random.default_rng(W * 7919 + count)
    g = [values(count, 1000 * w + count, "f32") for w in range(W)]
    s = 0.0
    for x in g:
        s = oracle.absmax(x, start=s)
    packed = [oracle.ternarize(g[w], s, 77, w) for w in range(W)]
    code = oracle.F32 if out_dtype == "f32" else oracle.BF16
    want = oracle.ternary_reduce(packed, count, s, code)
    out = torch.empty(count, dtype=torch.float32 if out_dtype == "f32" else torch.bfloat16, device="cuda")
    scale = torch.tensor([s], dtype=torch.float32, device="cuda")
    pac.pac_ternary_reduce_local(ctx.handle, [dev(p) for p in packed], scale, out, count)
    got = out.cpu().numpy().view(np.uint32) if out_dtype == "f32" else out.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want.view(got.dtype))


def test_ternary_step_on_workload_1(pac, ctx):
    """mask -> compress -> shared scale -> ternarize per worker -> integer sum -> decompress, against the oracle."""
    wl = make_workload(1, device=torch.device("cuda", 0))
    sp = wl.sparsity_at(0)
    mask, prefix, k = ctx.build_mask(wl.weights, wl.scope_offsets, sp)
    compact = [ctx.compress(g, mask, prefix, k) for g in wl.grads]
    scale = torch.zeros(1, device="cuda")
    for w, c in enumerate(compact):
        pac.pac_absmax(ctx.handle, c, scale, accumulate=w > 0)
    packed = [torch.empty((k + 3) // 4, dtype=torch.uint8, device="cuda") for _ in compact]
    for w, c in enumerate(compact):
        pac.pac_ternarize(ctx.handle, c, scale, 2024, w, packed[w])
    red = torch.empty(k, device="cuda")
    pac.pac_ternary_reduce_local(ctx.handle, packed, scale, red, k)
    dense = ctx.decompress(red, mask, prefix, wl.n, k)

    em, ep, ek = oracle.build_mask(wl.weights.cpu().numpy(), wl.scope_offsets, sp)
    e_compact = [oracle.compress(g.cpu().numpy(), em, ek) for g in wl.grads]
    s = 0.0
    for c in e_compact:
        s = oracle.absmax(c, start=s)
    e_packed = [oracle.ternarize(c, s, 2024, w) for w, c in enumerate(e_compact)]
    e_dense = oracle.decompress(oracle.ternary_reduce(e_packed, ek, s), em, wl.n)
    assert float(scale.item()) == s
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), e_dense.view(np.uint32))


def test_ternary_error_codes(pac, ctx):
    g = torch.zeros(100, device="cuda")
    scale = torch.ones(1, device="cuda")
    packed = torch.zeros(32, dtype=torch.uint8, device="cuda")
    with pytest.raises(pac.PacError) as e:                        # packed buffer not 4-byte aligned
        pac.pac_ternarize(ctx.handle, g, scale, 1, 1, packed[1:], count=100)
    assert e.value.status == -2
    with pytest.raises(pac.PacError) as e:
        pac.pac_ternary_reduce_local(ctx.handle, [packed] * 65, scale, g, 100)
    assert e.value.status == -3

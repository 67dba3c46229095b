"""Pins of the oracle's ternary payload (Sec. III-D): the random source against published known-answer
vectors, the quantiser against its defining properties (support, sign, saturation, unbiasedness), the
packing and the integer sum against numpy."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def unpack(packed: np.ndarray, count: int) -> np.ndarray:
    """2-bit codes -> values in {-1, 0, +1} with numpy shifts (element j: bits 2*(j%4) of byte j//4)."""
    j = np.arange(count)
    code = (packed[j >> 2] >> (2 * (j & 3)).astype(np.uint8)) & 3
    assert not np.any(code == 3)
    return np.where(code == 1, 1, np.where(code == 2, -1, 0)).astype(np.int32)


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert [int(x) for x in oracle.philox4x32_10(w[0:4], w[4:6])] == w[6:10]


def test_absmax_equals_numpy_nanmax():
    rng = np.random.default_rng(1)
    v = rng.standard_normal(1001).astype(np.float32)
    v[5] = np.nan
    v[17] = -7.5
    v[33] = -0.0
    assert oracle.absmax(v) == float(np.nanmax(np.abs(v))) == 7.5
    assert oracle.absmax(v, start=9.0) == 9.0 and oracle.absmax(v, start=1.0) == 7.5
    assert oracle.absmax(np.zeros(0, dtype=np.float32)) == 0.0
    assert oracle.absmax(np.array([np.nan, np.nan], dtype=np.float32)) == 0.0
    assert oracle.absmax(np.array([-np.inf, 1.0], dtype=np.float32)) == float("inf")
    b = torch.tensor([0.5, -3.0, 2.0]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert oracle.absmax(b, oracle.BF16) == 3.0


@pytest.mark.parametrize("count", [1, 3, 4, 5, 63, 64, 1001])
def test_ternarize_support_sign_saturation_and_layout(count):
    rng = np.random.default_rng(count)
    g = rng.standard_normal(count).astype(np.float32)
    g[rng.random(count) < 0.2] = 0.0
    s = float(np.max(np.abs(g))) if count > 1 else 2.0
    packed = oracle.ternarize(g, s, seed=0x1234567811223344, stream=7)
    assert packed.size == (count + 3) // 4
    t = unpack(packed, count)
    assert np.all(t[g == 0] == 0)                                   # zero stays zero
    assert np.all(np.sign(t[t != 0]) == np.sign(g[t != 0]))         # the sign is the gradient's
    if count > 1:
        assert np.all(t[np.abs(g) == np.float32(s)] != 0)           # |g| = s is always kept (u < 1)
    if count % 4:                                                   # unused bits of the last byte are zero
        assert packed[-1] >> (2 * (count % 4)) == 0


def test_ternarize_decision_is_u_below_p_with_the_pinned_generator():
    # u = (word >> 8) * 2^-24 from the generator pinned above, p = |g| / s in single precision.
    count, seed, stream = 1000, 0xDEADBEEF01234567, 3
    rng = np.random.default_rng(9)
    g = (rng.standard_normal(count) * 0.3).astype(np.float32)
    s = np.float32(1.25)
    t = unpack(oracle.ternarize(g, float(s), seed, stream), count)
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for blk in range(count // 4):
        r = oracle.philox4x32_10([blk, 0, stream, 0], key)
        u = (r >> 8).astype(np.float32) * np.float32(2.0 ** -24)
        p = np.abs(g[4 * blk:4 * blk + 4]) / s
        want = np.where(u < p, np.sign(g[4 * blk:4 * blk + 4]), 0).astype(np.int32)
        assert np.array_equal(t[4 * blk:4 * blk + 4], want)


def test_ternarize_is_unbiased():
    # E[s * t] = g (Eq. 3): the mean over many independent streams stays within 5 standard errors.
    g = np.array([0.9, -0.5, 0.1, -0.01, 0.0, 0.33, -1.0, 0.75], dtype=np.float32)
    s, N = 1.0, 6000
    acc = np.zeros(g.size)
    for stream in range(N):
        acc += unpack(oracle.ternarize(g, s, seed=42, stream=stream), g.size)
    mean = s * acc / N
    se = np.sqrt(np.maximum(s * np.abs(g) - g.astype(np.float64) ** 2, 1e-12) / N)
    assert np.all(np.abs(mean - g) <= 5 * se + 1e-12)
    assert mean[4] == 0.0 and mean[6] == -1.0                       # exact at the ends


def test_ternarize_streams_and_seeds_differ_and_repeat():
    g = np.full(4096, 0.5, dtype=np.float32)
    a = oracle.ternarize(g, 1.0, 1, 0)
    assert np.array_equal(a, oracle.ternarize(g, 1.0, 1, 0))
    assert not np.array_equal(a, oracle.ternarize(g, 1.0, 1, 1))
    assert not np.array_equal(a, oracle.ternarize(g, 1.0, 2, 0))
    kept = np.count_nonzero(unpack(a, g.size))
    assert abs(kept - 2048) < 5 * np.sqrt(4096 * 0.25)              # Bernoulli(1/2)


@pytest.mark.parametrize("scale", [0.0, -1.0, float("inf"), float("nan")])
def test_ternarize_unusable_scale_gives_zeros(scale):
    g = np.array([1.0, -2.0, 0.5, 3.0, -1.0], dtype=np.float32)
    assert not np.any(oracle.ternarize(g, scale, 5, 5))


def test_ternarize_nan_elements_and_clipping():
    g = np.array([np.nan, 4.0, -4.0, 0.0], dtype=np.float32)
    t = unpack(oracle.ternarize(g, 2.0, 1, 1), 4)                   # |g| above the scale: always kept
    assert list(t) == [0, 1, -1, 0]


def test_ternarize_bf16_equals_f32_of_the_widened_values():
    rng = np.random.default_rng(4)
    g = torch.from_numpy(rng.standard_normal(777).astype(np.float32)).to(torch.bfloat16)
    raw = g.view(torch.int16).numpy().view(np.uint16)
    wide = g.to(torch.float32).numpy()
    assert np.array_equal(oracle.ternarize(raw, 3.0, 8, 2, oracle.BF16), oracle.ternarize(wide, 3.0, 8, 2))


@pytest.mark.parametrize("W,count", [(1, 5), (3, 64), (8, 1001), (16, 4099)])
def test_ternary_reduce_equals_numpy_integer_sum(W, count):
    rng = np.random.default_rng(W * 1000 + count)
    codes = rng.choice(np.array([0, 1, 2], dtype=np.uint8), size=(W, count), p=[0.5, 0.25, 0.25])
    packed = []
    for w in range(W):
        pad = np.concatenate([codes[w], np.zeros((-count) % 4, dtype=np.uint8)]).reshape(-1, 4)
        packed.append((pad[:, 0] | (pad[:, 1] << 2) | (pad[:, 2] << 4) | (pad[:, 3] << 6)).astype(np.uint8))
    total = np.where(codes == 1, 1, np.where(codes == 2, -1, 0)).sum(axis=0)
    scale = np.float32(0.0123)
    want = scale * total.astype(np.float32)
    got = oracle.ternary_reduce(packed, count, float(scale))
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    got16 = oracle.ternary_reduce(packed, count, float(scale), oracle.BF16)
    want16 = torch.from_numpy(want).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got16, want16)


def test_ternary_path_estimates_the_plain_sum():
    # sum over workers of s * t_w is an unbiased estimate of the sum of the gradients
    rng = np.random.default_rng(12)
    W, count = 8, 20000
    g = [(rng.standard_normal(count) * 0.1).astype(np.float32) for _ in range(W)]
    s = 0.0
    for x in g:
        s = oracle.absmax(x, start=s)
    packed = [oracle.ternarize(g[w], s, seed=99, stream=w) for w in range(W)]
    est = oracle.ternary_reduce(packed, count, s).astype(np.float64)
    exact = np.sum(np.stack(g).astype(np.float64), axis=0)
    var = np.sum(s * np.abs(np.stack(g)).astype(np.float64) - np.stack(g).astype(np.float64) ** 2, axis=0)
    z = (est - exact) / np.sqrt(np.maximum(var, 1e-30))
    assert abs(np.mean(z)) < 5 / np.sqrt(count) and 0.9 < np.std(z) < 1.1

"""Pins of the CPU oracle against things other than itself.

The paper prints no worked input/output pair for the compression path, so the pins are: brute
force on tiny inputs, exhaustive enumeration, closed forms, invariants that characterise the
result, and library routines on the special cases where the definition reduces to them.
Each pin is chosen so that a plausible slip in the oracle (a wrong sign in the tie rule, an
off-by-one in the count, a transposed bit order, a dropped worker, a double rounding) fails it.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from synth import config_shapes, flat_size

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def bits_to_bool(mask, n):
    """Unpack uint64 words, LSB first, to a bool vector of length n (numpy's own unpackbits)."""
    b = np.unpackbits(mask.view(np.uint8), bitorder="little")
    return b[:n].astype(bool)


def key_of(w):
    return np.ascontiguousarray(w, dtype=np.float32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def brute_force_keep(w, k):
    """rank_i = #{j : key_j > key_i or (key_j == key_i and j < i)}; keep iff rank_i < k.  O(n^2)."""
    key = key_of(w).astype(np.int64)
    n = key.size
    idx = np.arange(n)
    gt = key[None, :] > key[:, None]
    eq_before = (key[None, :] == key[:, None]) & (idx[None, :] < idx[:, None])
    rank = (gt | eq_before).sum(axis=1)
    return rank < k


def exact_keep_count(n, s_text):
    """ceil((1-s) n) in exact rational arithmetic from the decimal text of s."""
    return math.ceil((1 - Fraction(s_text)) * n)


# ----------------------------------------------------------------------------- keep count
def test_keep_count_golden_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "keep_counts.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for n, s, k in rows:
        assert oracle.keep_count(int(n), float(s)) == int(k), (n, s, k)


def test_keep_count_matches_exact_rational_ceiling():
    rng = np.random.default_rng(1)
    for _ in range(2000):
        n = int(rng.integers(0, 2**32 - 1))
        ppm = int(rng.integers(0, 1000001))
        s_text = f"{ppm / 1e6:.6f}"
        assert oracle.keep_count(n, float(s_text)) == exact_keep_count(n, s_text)


def test_keep_count_does_not_inherit_double_rounding():
    # (1 - 0.7) * 10 evaluates to 3.0000000000000004 in doubles; the count is 3.
    assert oracle.keep_count(10, 0.7) == 3
    assert oracle.keep_count(109482240, 0.7) == 32844672


def test_flat_sizes_golden():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "flat_sizes.txt")) if l.strip() and not l.startswith("#")]
    for cid, tensors, n in rows:
        specs = config_shapes(int(cid))
        assert len(specs) == int(tensors)
        assert flat_size(specs) == int(n)


def test_paper_model_shapes_reach_the_published_parameter_counts():
    from synth.shapes import _resnet152, _vgg19, _vit_base_16
    assert flat_size(_vgg19(1000)) == 143667240
    assert flat_size(_resnet152(1000)) == 60192808
    assert flat_size(_vit_base_16(1000)) == 86567656


# ----------------------------------------------------------------------------- kept set
@pytest.mark.parametrize("n", [1, 2, 7, 63, 64, 65, 130, 257, 700])
def test_mask_equals_brute_force_with_heavy_ties(n):
    rng = np.random.default_rng(n)
    pool = np.array([0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 2.0, 3.5, 1e-40, -1e-40, np.inf, -np.inf], dtype=np.float32)
    for trial in range(12):
        w = rng.choice(pool, size=n) if trial % 2 == 0 else rng.standard_normal(n).astype(np.float32)
        for s in (0.0, 0.1, 0.5, 0.77, 0.9, 0.999, 1.0):
            mask, prefix, nnz = oracle.build_mask(w, None, s)
            k = exact_keep_count(n, f"{s:.6f}")
            assert nnz == k
            got = bits_to_bool(mask, n)
            assert np.array_equal(got, brute_force_keep(w, k)), (n, trial, s)
            # tail bits of the last word are zero
            assert int(np.unpackbits(mask.view(np.uint8), bitorder="little").sum()) == k


def test_mask_exhaustive_small_alphabet():
    """All weight vectors over {-1, -0, +0, 1, 2} for n <= 5, every k."""
    alphabet = np.array([-1.0, -0.0, 0.0, 1.0, 2.0], dtype=np.float32)
    for n in range(1, 6):
        for combo in itertools.product(range(5), repeat=n):
            w = alphabet[list(combo)]
            for k in range(n + 1):
                s = 1.0 if k == 0 else 1.0 - (k - 0.5) / n     # (1-s)n = k-1/2, whose ceiling is k
                mask, _, nnz = oracle.build_mask(w, None, s)
                assert nnz == k
                assert np.array_equal(bits_to_bool(mask, n), brute_force_keep(w, k))


def test_mask_all_equal_keeps_first_k_and_ramp_keeps_last_k():
    n = 1000
    for s in (0.3, 0.9):
        k = exact_keep_count(n, str(s))
        m, _, _ = oracle.build_mask(np.full(n, 1.0, np.float32), None, s)
        assert np.array_equal(np.flatnonzero(bits_to_bool(m, n)), np.arange(k))
        m, _, _ = oracle.build_mask(np.arange(n, dtype=np.float32), None, s)
        assert np.array_equal(np.flatnonzero(bits_to_bool(m, n)), np.arange(n - k, n))
        # sign must not matter
        m, _, _ = oracle.build_mask(-np.arange(n, dtype=np.float32), None, s)
        assert np.array_equal(np.flatnonzero(bits_to_bool(m, n)), np.arange(n - k, n))


def test_mask_distinct_values_equals_library_topk():
    rng = np.random.default_rng(7)
    n = 50000
    w = rng.permutation(n).astype(np.float32) - n / 2 + 0.25      # distinct magnitudes
    assert np.unique(np.abs(w)).size == n
    for s in (0.5, 0.8, 0.95):
        k = exact_keep_count(n, str(s))
        top = np.argsort(-np.abs(w), kind="stable")[:k]
        m, _, _ = oracle.build_mask(w, None, s)
        assert np.array_equal(np.flatnonzero(bits_to_bool(m, n)), np.sort(top))


def test_mask_equals_stable_argsort_on_abs_with_ties():
    rng = np.random.default_rng(8)
    n = 20000
    w = rng.integers(-20, 21, size=n).astype(np.float32)          # many ties, both signs
    for s in (0.2, 0.5, 0.9):
        k = exact_keep_count(n, str(s))
        top = np.argsort(-np.abs(w), kind="stable")[:k]            # |w| descending, index ascending
        m, _, _ = oracle.build_mask(w, None, s)
        assert np.array_equal(np.flatnonzero(bits_to_bool(m, n)), np.sort(top))


def test_mask_gaussian_threshold_matches_normal_quantile():
    """For N(0, sigma^2) weights the smallest kept |w| is sigma*z_{(1+s)/2} up to O(n^-1/2)."""
    rng = np.random.default_rng(9)
    n = 1 << 20
    sigma = 1.0 / 32.0
    w = (rng.standard_normal(n) * sigma).astype(np.float32)
    for s, z in ((0.5, 0.6745), (0.7, 1.0364), (0.8, 1.2816), (0.9, 1.6449), (0.95, 1.9600)):
        m, _, k = oracle.build_mask(w, None, s)
        kept = bits_to_bool(m, n)
        t = np.abs(w[kept]).min()
        assert abs(t / sigma - z) < 0.01, (s, t / sigma, z)
        assert np.abs(w[~kept]).max() <= t


def test_special_floats_order_by_bit_pattern():
    # magnitudes ascending by key: 0, denormal, tiny normal, 1, inf, nan
    w = np.array([np.nan, -np.inf, 1.0, 1.2e-38, -1e-45, -0.0], dtype=np.float32)
    for k in range(7):
        m, _, nnz = oracle.build_mask(w, None, 1.0 if k == 0 else 1.0 - (k - 0.5) / 6)
        assert nnz == k
        assert np.array_equal(np.flatnonzero(bits_to_bool(m, 6)), np.arange(k))


def test_segmented_mask_equals_independent_scopes():
    rng = np.random.default_rng(10)
    sizes = [0, 5, 64, 1, 63, 0, 129, 1000, 2, 64]
    off = np.concatenate([[0], np.cumsum(sizes)])
    n = int(off[-1])
    w = rng.integers(-3, 4, size=n).astype(np.float32)
    sp = rng.choice([0.0, 0.3, 0.5, 0.9, 1.0], size=len(sizes))
    mask, prefix, nnz = oracle.build_mask(w, off, sp)
    got = bits_to_bool(mask, n)
    total = 0
    for i, sz in enumerate(sizes):
        k = exact_keep_count(sz, str(sp[i]))
        total += k
        assert np.array_equal(got[off[i]:off[i + 1]], brute_force_keep(w[off[i]:off[i + 1]], k))
    assert nnz == total


def test_invariants_characterise_the_kept_set():
    rng = np.random.default_rng(11)
    n = 200000
    w = np.round(rng.standard_normal(n) * 50).astype(np.float32)     # heavy ties
    m, _, k = oracle.build_mask(w, None, 0.8)
    kept = bits_to_bool(m, n)
    key = key_of(w)
    assert kept.sum() == k
    t = key[kept].min()
    assert key[~kept].max() <= t
    tie = np.flatnonzero(key == t)
    # among ties at the threshold every kept index precedes every pruned one
    assert kept[tie].sum() >= 1
    assert np.all(np.diff(kept[tie].astype(int)) <= 0)


# ----------------------------------------------------------------------------- prefix
def test_prefix_is_exclusive_scan_of_word_popcounts():
    rng = np.random.default_rng(12)
    n = 100003
    w = rng.standard_normal(n).astype(np.float32)
    m, p, k = oracle.build_mask(w, None, 0.6)
    pop = np.unpackbits(m.view(np.uint8), bitorder="little").reshape(-1, 64).sum(axis=1)
    assert np.array_equal(p.astype(np.int64), np.cumsum(pop) - pop)
    assert int(p[-1]) + int(pop[-1]) == k


# ----------------------------------------------------------------------------- compress / decompress
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_compress_equals_boolean_indexing_and_round_trips(dtype):
    rng = np.random.default_rng(13)
    n = 70001
    w = rng.standard_normal(n).astype(np.float32)
    m, p, k = oracle.build_mask(w, None, 0.8)
    kept = bits_to_bool(m, n)
    if dtype == oracle.F32:
        g = rng.standard_normal(n).astype(np.float32)
        g[::97] = -0.0
        g[5::1013] = np.nan
        raw = g.view(np.uint32)
    else:
        g = rng.integers(0, 65536, size=n).astype(np.uint16)
        raw = g
    c = oracle.compress(g, m, k, dtype)
    assert c.size == k
    cr = c.view(np.uint32) if dtype == oracle.F32 else c
    assert np.array_equal(cr, raw[kept])                       # bit copies, ascending flat index
    d = oracle.decompress(c, m, n, dtype)
    dr = d.view(np.uint32) if dtype == oracle.F32 else d
    assert np.array_equal(dr, np.where(kept, raw, 0))           # pruned positions are +0 patterns
    assert np.array_equal(oracle.compress(d, m, k, dtype).view(raw.dtype), cr)


def test_compress_rejects_wrong_count():
    w = np.arange(100, dtype=np.float32)
    m, _, k = oracle.build_mask(w, None, 0.5)
    with pytest.raises(ValueError):
        oracle.compress(w, m, k - 1)
    with pytest.raises(ValueError):
        oracle.decompress(np.zeros(k + 1, np.float32), m, 100)


def test_sparsity_zero_is_identity_and_one_is_all_zero():
    g = np.arange(1, 131, dtype=np.float32)
    m, _, k = oracle.build_mask(g, None, 0.0)
    assert k == 130 and np.array_equal(oracle.compress(g, m, k), g)
    assert np.array_equal(oracle.decompress(g, m, 130), g)
    m, _, k = oracle.build_mask(g, None, 1.0)
    assert k == 0 and oracle.compress(g, m, 0).size == 0
    assert np.array_equal(oracle.decompress(np.zeros(0, np.float32), m, 130).view(np.uint32), np.zeros(130, np.uint32))


# ----------------------------------------------------------------------------- sum
def test_sum_single_worker_is_identity_including_negative_zero():
    c = np.array([-0.0, 1.5, np.inf, -3.0], dtype=np.float32)
    assert np.array_equal(oracle.reduce_local([c]).view(np.uint32), c.view(np.uint32))


def test_sum_of_small_integers_is_exact():
    rng = np.random.default_rng(14)
    bufs = [rng.integers(-1000, 1000, size=5000).astype(np.float32) for _ in range(8)]
    exact = np.sum([b.astype(np.int64) for b in bufs], axis=0)
    assert np.array_equal(oracle.reduce_local(bufs).astype(np.int64), exact)


def test_sum_is_left_fold_in_single_precision():
    rng = np.random.default_rng(15)
    W, n = 16, 20000
    bufs = [(rng.standard_normal(n) * 10.0 ** rng.integers(-6, 6)).astype(np.float32) for _ in range(W)]
    acc = bufs[0].copy()
    for b in bufs[1:]:
        acc = (acc + b).astype(np.float32)                      # numpy float32 add, same order
    got = oracle.reduce_local(bufs)
    assert np.array_equal(got.view(np.uint32), acc.view(np.uint32))
    # and the order matters on this data, so a reversed fold would have been caught
    rev = bufs[-1].copy()
    for b in bufs[-2::-1]:
        rev = (rev + b).astype(np.float32)
    assert not np.array_equal(rev.view(np.uint32), acc.view(np.uint32))


def test_bf16_rounding_matches_torch_cpu_cast():
    rng = np.random.default_rng(16)
    x = np.concatenate([
        (rng.standard_normal(200000) * 10.0 ** rng.integers(-30, 30, size=200000)).astype(np.float32),
        np.array([0.0, -0.0, np.inf, -np.inf, 3.3895314e38, 1e-45, 1.0039062, 1.0117188], dtype=np.float32),
        # exact ties between two bf16 values, both parities
        (np.arange(0x3F800000, 0x3F800000 + (64 << 16), 1 << 15, dtype=np.uint32)).view(np.float32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16(x), ref)
    nan_out = oracle.f32_to_bf16(np.array([np.nan], dtype=np.float32))
    assert (nan_out[0] & 0x7F80) == 0x7F80 and (nan_out[0] & 0x007F) != 0


def test_bf16_sum_widens_adds_in_single_and_rounds_once():
    rng = np.random.default_rng(17)
    W, n = 16, 30000
    tens = [torch.from_numpy((rng.standard_normal(n) * 1e-4).astype(np.float32)).to(torch.bfloat16) for _ in range(W)]
    bufs = [t.view(torch.int16).numpy().view(np.uint16) for t in tens]
    acc = tens[0].to(torch.float32)
    for t in tens[1:]:
        acc = acc + t.to(torch.float32)
    ref = acc.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.reduce_local(bufs, oracle.BF16)
    assert np.array_equal(got, ref)
    # rounding after every add (a double-rounding slip) gives a different answer on this data
    acc2 = tens[0].clone()
    for t in tens[1:]:
        acc2 = (acc2.to(torch.float32) + t.to(torch.float32)).to(torch.bfloat16)
    assert not np.array_equal(acc2.view(torch.int16).numpy().view(np.uint16), ref)


# ----------------------------------------------------------------------------- whole path
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_pipeline_equals_masked_fold_of_dense_gradients(dtype):
    """decompress(sum_w compress(g_w)) == where(mask, fold_w g_w, +0): Eq. 2 applied to Eq. 1's sum."""
    rng = np.random.default_rng(18)
    n, W = 40007, 8
    w = rng.standard_normal(n).astype(np.float32)
    m, p, k = oracle.build_mask(w, None, 0.9)
    kept = bits_to_bool(m, n)
    gs32 = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(W)]
    if dtype == oracle.BF16:
        tens = [torch.from_numpy(g).to(torch.bfloat16) for g in gs32]
        gs = [t.view(torch.int16).numpy().view(np.uint16) for t in tens]
        acc = tens[0].to(torch.float32)
        for t in tens[1:]:
            acc = acc + t.to(torch.float32)
        dense_sum = acc.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    else:
        gs = gs32
        acc = gs32[0].copy()
        for g in gs32[1:]:
            acc = (acc + g).astype(np.float32)
        dense_sum = acc.view(np.uint32)
    red = oracle.reduce_local([oracle.compress(g, m, k, dtype) for g in gs], dtype)
    out = oracle.decompress(red, m, n, dtype)
    out_raw = out.view(np.uint32) if dtype == oracle.F32 else out
    assert np.array_equal(out_raw, np.where(kept, dense_sum, 0))


# ---- the all-core leg of the benchmark's CPU baseline: defined by the functions pinned above ----

@pytest.mark.parametrize("trial", range(24))
def test_all_core_leg_equals_the_definition_oracle(trial):
    """pac_oracle_mt.cpp (counting select, positional tie rule, word-parallel gather / sum / scatter) against
    pac_oracle.cpp (composites + nth_element, ascending walks, left fold) on random scope tables, heavy ties,
    pruned (zeroed) weights, all-equal scopes, empty scopes, s = 0 and s = 1, both payload types."""
    rng = np.random.default_rng(1000 + trial)
    n = int(rng.integers(1, 200000)) if trial % 6 else int(rng.integers(1, 130))
    w = rng.standard_normal(n).astype(np.float32)
    if trial % 3 == 0:
        w[rng.random(n) < 0.6] = 0.0
    if trial % 5 == 0:
        w[:] = np.float32(0.5)
    if trial % 7 == 0:
        w = (np.round(w * 4) / 4).astype(np.float32)
    if trial % 4 == 1 and n > 8:
        w[:4] = [np.inf, -np.inf, np.nan, -0.0]
    nseg = int(rng.integers(1, 9))
    off = [0] + sorted(int(c) for c in rng.integers(0, n + 1, size=nseg - 1)) + [n]
    sp = rng.choice([0.0, 1.0, 0.5, 0.9, 0.123456, 0.8], size=nseg)
    mask, prefix, k = oracle.build_mask(w, off, sp)
    m2, p2, k2 = oracle.build_mask_mt(w, off, sp)
    assert k == k2 and np.array_equal(mask, m2) and np.array_equal(prefix, p2)
    for dt in (oracle.F32, oracle.BF16):
        W = int(rng.integers(1, 6))
        if dt == oracle.F32:
            grads = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
        else:
            grads = [rng.integers(0, 65536, n).astype(np.uint16) for _ in range(W)]
        cs = [oracle.compress(g, mask, k, dt) for g in grads]
        cm = [oracle.compress_mt(g, mask, prefix, k, dt) for g in grads]
        assert all(np.array_equal(a.view(np.uint8), b.view(np.uint8)) for a, b in zip(cs, cm))
        r, rm = oracle.reduce_local(cs, dt), oracle.reduce_local_mt(cm, dt)
        assert np.array_equal(r.view(np.uint8), rm.view(np.uint8))
        d, dm = oracle.decompress(r, mask, n, dt), oracle.decompress_mt(rm, mask, prefix, n, dt)
        assert np.array_equal(d.view(np.uint8), dm.view(np.uint8))
    assert 1 <= oracle.mt_threads() <= 4096

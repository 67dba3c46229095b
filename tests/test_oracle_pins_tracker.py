"""Pins of the oracle's Mask Tracker and weight-update functions against numpy / torch routines and
closed forms (nothing here calls the function under test to produce its own expectation)."""
import numpy as np
import pytest
import torch

import oracle


def bits_to_bool(mask, n):
    return np.unpackbits(mask.view(np.uint8), bitorder="little")[:n].astype(bool)


def bool_to_words(b):
    n = b.size
    pad = (-n) % 64
    by = np.packbits(np.concatenate([b, np.zeros(pad, dtype=bool)]), bitorder="little")
    return by.view(np.uint64).copy()


SPECIAL_F32 = np.array([0.0, -0.0, 1.0, -1.0, np.nan, -np.nan, np.inf, -np.inf, 1e-45, -1e-45,
                        np.finfo(np.float32).tiny, 3.0e38], dtype=np.float32)


# ------------------------------------------------------------------ mask_from_nonzero
@pytest.mark.parametrize("n", [0, 1, 5, 63, 64, 65, 127, 128, 1000, 4097])
def test_from_nonzero_f32_equals_numpy_comparison_and_packbits(n):
    rng = np.random.default_rng(100 + n)
    v = rng.standard_normal(n).astype(np.float32)
    v[rng.random(n) < 0.6] = 0.0
    v[rng.random(n) < 0.1] = -0.0
    if n >= SPECIAL_F32.size:
        v[:SPECIAL_F32.size] = SPECIAL_F32
    mask, prefix, nnz = oracle.mask_from_nonzero(v)
    want = v != 0                       # numpy's IEEE comparison: -0 is zero, NaN is not
    assert nnz == int(np.count_nonzero(want))
    assert np.array_equal(mask, bool_to_words(want)[:mask.size])
    assert np.array_equal(bits_to_bool(mask, n), want)
    pop = np.array([bin(int(x)).count("1") for x in mask], dtype=np.int64)
    assert np.array_equal(prefix.astype(np.int64), np.cumsum(pop) - pop)


def test_from_nonzero_bf16_equals_torch_comparison():
    # every bf16 bit pattern once: torch's own bf16 comparison decides which are non-zero
    pat = np.arange(65536, dtype=np.uint16)
    t = torch.from_numpy(pat.view(np.int16)).view(torch.bfloat16)
    want = (t != 0).numpy()
    mask, prefix, nnz = oracle.mask_from_nonzero(pat, oracle.BF16)
    assert np.array_equal(bits_to_bool(mask, pat.size), want)
    assert nnz == 65536 - 2             # +0 and -0 are the only zeros
    assert not want[0] and not want[0x8000] and want[0x0001] and want[0x7FC0]


def test_from_nonzero_of_pruned_weights_recovers_the_prune_mask():
    # Eq. 2: the mask is (Weight != 0) of the pruned model.  With no exact zeros among the kept
    # weights this must give back the mask that build_mask (pinned elsewhere) produced.
    rng = np.random.default_rng(7)
    n = 20000
    w = rng.standard_normal(n).astype(np.float32)
    w[w == 0] = 1.0
    pm, pp, k = oracle.build_mask(w, [0, 5000, n], [0.9, 0.5])
    pruned = np.where(bits_to_bool(pm, n), w, np.float32(0))
    m, p, nnz = oracle.mask_from_nonzero(pruned)
    assert nnz == k and np.array_equal(m, pm) and np.array_equal(p, pp)


# ------------------------------------------------------------------ mask_diff
@pytest.mark.parametrize("n", [1, 64, 65, 1000, 4099])
def test_mask_diff_equals_boolean_xor_count(n):
    rng = np.random.default_rng(n)
    a = rng.random(n) < 0.3
    b = a.copy()
    flips = rng.choice(n, size=min(n, 17), replace=False)
    b[flips] = ~b[flips]
    wa, wb = bool_to_words(a), bool_to_words(b)
    assert oracle.mask_diff(wa, wb, n) == int(np.count_nonzero(a != b)) == flips.size
    assert oracle.mask_diff(wa, wa, n) == 0
    assert oracle.mask_diff(wb, wa, n) == flips.size                       # symmetric
    assert oracle.mask_diff(wa, np.zeros_like(wa), n) == int(a.sum())      # distance to the empty mask


def test_mask_diff_ignores_bits_at_and_beyond_n():
    a = np.array([0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    b = np.array([0x00000000000000FF], dtype=np.uint64)
    assert oracle.mask_diff(a, b, 8) == 0
    assert oracle.mask_diff(a, b, 9) == 1
    assert oracle.mask_diff(a, b, 64) == 56


# ------------------------------------------------------------------ tracker bookkeeping
def test_tracker_sequence_by_hand():
    # masks A A A B B B B A with patience 2: comparisons "same" at steps 1,2 | 4,5,6 |
    A = np.array([0b1011], dtype=np.uint64)
    B = np.array([0b1101], dtype=np.uint64)
    tr = oracle.MaskTracker(patience=2)
    got = [tr.update(m, 4) for m in (A, A, A, B, B, B, B, A)]
    assert got == [(0, False), (1, False), (2, True), (0, False), (1, False), (2, True), (3, True), (0, False)]


def test_tracker_length_change_counts_as_change():
    A = np.array([0b1011], dtype=np.uint64)
    tr = oracle.MaskTracker(patience=1)
    assert tr.update(A, 4) == (0, False)
    assert tr.update(A, 4) == (1, True)
    assert tr.update(A, 5) == (0, False)


# ------------------------------------------------------------------ decompress_update (Eq. 1)
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_update_equals_numpy_masked_assignment(dtype):
    rng = np.random.default_rng(11)
    n = 5000
    x = rng.standard_normal(n).astype(np.float32)
    keep = rng.random(n) < 0.2
    mask = bool_to_words(keep)
    k = int(keep.sum())
    g32 = (rng.standard_normal(k) * 3).astype(np.float32)
    if dtype == oracle.BF16:
        gb = torch.from_numpy(g32).to(torch.bfloat16)
        compact = gb.view(torch.int16).numpy().view(np.uint16)
        g32 = gb.to(torch.float32).numpy()          # exact widening, by torch
    else:
        compact = g32
    alpha = np.float32(0.0125)
    want = np.zeros(n, dtype=np.float32)
    want[keep] = x[keep] - alpha * g32               # numpy float32: multiply rounds, subtract rounds
    got = oracle.decompress_update(compact, mask, x, float(alpha), dtype)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_update_is_two_roundings_not_a_fused_multiply_add():
    # x = 1, alpha = 1 + 2^-12, g = 1 + 2^-12: alpha*g = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 in
    # single precision, so two roundings give exactly -2^-11; a fused multiply-add would keep the
    # 2^-24 and give -(2^-11 + 2^-24).
    a = np.float32(1 + 2.0 ** -12)
    mask = np.array([1], dtype=np.uint64)
    got = oracle.decompress_update(np.array([a], dtype=np.float32), mask, np.array([1.0], dtype=np.float32), float(a))
    assert got[0] == np.float32(-(2.0 ** -11))


def test_update_closed_forms():
    rng = np.random.default_rng(3)
    n = 300
    x = rng.standard_normal(n).astype(np.float32)
    keep = rng.random(n) < 0.5
    mask = bool_to_words(keep)
    k = int(keep.sum())
    g = rng.standard_normal(k).astype(np.float32)
    # alpha = 0: kept weights unchanged, pruned weights +0 (sign bit clear)
    z = oracle.decompress_update(g, mask, x, 0.0)
    assert np.array_equal(z[keep], x[keep]) and np.all(z[~keep].view(np.uint32) == 0)
    # g = 0: the same
    z = oracle.decompress_update(np.zeros(k, dtype=np.float32), mask, x, 0.5)
    assert np.array_equal(z[keep], x[keep])
    # equals "decompress, then dense update, then re-apply the mask" (the unfused path)
    dense = oracle.decompress(g, mask, n)
    unfused = np.where(keep, x - np.float32(0.25) * dense, np.float32(0))
    assert np.array_equal(oracle.decompress_update(g, mask, x, 0.25).view(np.uint32), unfused.view(np.uint32))


def test_update_rejects_wrong_count():
    mask = np.array([0b111], dtype=np.uint64)
    with pytest.raises(ValueError):
        oracle.decompress_update(np.zeros(2, dtype=np.float32), mask, np.zeros(3, dtype=np.float32), 1.0)

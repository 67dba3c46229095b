"""Seeded random sweep over pac_build_mask -> pac_compress -> pac_decompress against the oracle: random
sizes (one element to 30M, so that exact, sampled and small prune scopes all occur), random scope tables
(unaligned, word-aligned with empty scopes, many small scopes before a large one), random sparsities
including 0 and 1, and value kinds with heavy ties, tile-constant magnitudes and special floats."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


def weights_of(kind, n, rng):
    if kind == "gauss":
        return (rng.standard_normal(n) * 0.02).astype(np.float32)
    if kind == "ties":
        return (rng.integers(-8, 9, n) / 8.0).astype(np.float32)
    if kind == "equal":
        return np.full(n, 1.0, np.float32)
    if kind == "zeros_half":
        w = (rng.standard_normal(n) * 0.02).astype(np.float32)
        w[rng.random(n) < 0.5] = 0
        return w
    if kind == "tile_constant":
        per = (rng.random(n // 16384 + 2) * 4 + 0.01).astype(np.float32)
        return np.repeat(per, 16384)[:n].copy()
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)          # "special"
    idx = rng.integers(0, n, max(1, n // 1000))
    w[idx] = np.array([np.inf, -np.inf, np.nan, 0.0, -0.0, 1e-42], np.float32)[rng.integers(0, 6, idx.size)]
    return w


def scope_table(n, rng):
    nseg = min(int(rng.choice([1, 1, 2, 3, 7, 40, 300])), n)
    if nseg == 1:
        return [0, n]
    mode = int(rng.integers(0, 3))
    if mode == 0:
        cuts = np.sort(rng.integers(0, n + 1, nseg - 1))
    elif mode == 1:
        cuts = np.sort(np.minimum(n, rng.integers(0, n // 64 + 1, nseg - 1) * 64))
    else:
        cuts = np.sort(np.minimum(np.cumsum(rng.integers(1, 5000, nseg - 1)), n))
    return [0] + [int(c) for c in cuts] + [n]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_tables_and_values(seed):
    import paper_2505_18563_amd as pac
    rng = np.random.default_rng(seed)
    ctx = pac.PacContext(max_elems=1 << 25, max_segments=4096, device=0)
    try:
        for case in range(40):
            if case % 8 == 0:
                n = int(rng.integers(4_200_000, 30_000_000))
            else:
                n = int(rng.choice([rng.integers(1, 5000), rng.integers(1, 200_000), rng.integers(1, 3_000_000)]))
            kind = str(rng.choice(["gauss", "ties", "equal", "zeros_half", "tile_constant", "special"]))
            w = weights_of(kind, n, rng)
            offs = scope_table(n, rng)
            sp = [float(rng.choice([0.0, 1.0, 0.5, 0.9, 0.99, rng.random()])) for _ in range(len(offs) - 1)]
            print(f"[random] seed={seed} case={case} n={n} kind={kind} nseg={len(offs) - 1}", flush=True)
            em, ep, ennz = oracle.build_mask(w, offs, sp)
            m, p, nnz = ctx.build_mask(torch.from_numpy(w).cuda(), offs, sp)
            torch.cuda.synchronize()
            assert nnz == ennz
            gm = m.cpu().numpy().view(np.uint64)
            assert np.array_equal(gm, em), f"case {case}: mask differs"
            assert np.array_equal(p.cpu().numpy().view(np.uint32), ep), f"case {case}: prefix differs"
            g = rng.standard_normal(n).astype(np.float32)
            gt = torch.from_numpy(g).cuda()
            compact = ctx.compress(gt, m, p, nnz)
            dense = ctx.decompress(compact, m, p, n, nnz)
            torch.cuda.synchronize()
            ec = oracle.compress(g, em, ennz)
            assert np.array_equal(compact.cpu().numpy().view(np.uint32), ec.view(np.uint32)), f"case {case}: gather"
            ed = oracle.decompress(ec, em, n)
            assert np.array_equal(dense.cpu().numpy().view(np.uint32), ed.view(np.uint32)), f"case {case}: scatter"
    finally:
        ctx.close()

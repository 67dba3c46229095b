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


def _bits(t):
    if t.dtype == torch.float32:
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _device_view(a_f32, bf16, shift):
    """Device tensor with the values of a_f32 (rounded to bf16 if asked) whose data pointer lies `shift`
    elements past an aligned allocation, and the host array that the oracle gets."""
    if bf16:
        u = oracle.f32_to_bf16(a_f32)
        base = torch.zeros(u.size + 8, dtype=torch.int16, device="cuda")
        base[shift:shift + u.size] = torch.from_numpy(u.view(np.int16)).cuda()
        return base[shift:shift + u.size].view(torch.bfloat16), u
    base = torch.zeros(a_f32.size + 8, dtype=torch.float32, device="cuda")
    base[shift:shift + a_f32.size] = torch.from_numpy(a_f32).cuda()
    return base[shift:shift + a_f32.size], a_f32


@pytest.mark.parametrize("seed", [21, 22])
def test_random_payloads_and_alignments(seed):
    """mask_from_nonzero -> compress x W -> reduce_local -> decompress / decompress_update with random length,
    density, payload type, worker count and element misalignment of every buffer; guard elements around the
    outputs must keep their values."""
    import paper_2505_18563_amd as pac
    rng = np.random.default_rng(seed)
    ctx = pac.PacContext(max_elems=1 << 23, max_segments=8, device=0)
    h = ctx.handle
    try:
        for case in range(40):
            n = int(rng.choice([rng.integers(1, 300), rng.integers(1, 70_000), rng.integers(1, 3_000_000)]))
            bf16 = bool(rng.integers(0, 2))
            dt = oracle.BF16 if bf16 else oracle.F32
            dens = float(rng.choice([0.0, 1.0, 0.1, 0.5, rng.random()]))
            W = int(rng.choice([1, 2, 3, 8, 16, 33]))
            shift = int(rng.choice([0, 0, 1, 3, 4]))
            print(f"[random] seed={seed} case={case} n={n} bf16={bf16} density={dens:.3f} W={W} shift={shift}", flush=True)
            keep = rng.random(n) < dens
            vals = np.where(keep, rng.standard_normal(n).astype(np.float32) + 3.0, 0).astype(np.float32)
            vt, vhost = _device_view(vals, bf16, shift)
            em, ep, nnz = oracle.mask_from_nonzero(vhost, dt)
            words = (n + 63) // 64
            m = torch.empty(words, dtype=torch.int64, device="cuda")
            p = torch.empty(words, dtype=torch.int32, device="cuda")
            nz = torch.zeros(1, dtype=torch.int64, device="cuda")
            pac.pac_mask_from_nonzero(h, vt, m, p, nz)
            torch.cuda.synchronize()
            assert int(nz.item()) == nnz
            assert np.array_equal(m.cpu().numpy().view(np.uint64), em), f"case {case}: mask of non-zeros"
            assert np.array_equal(p.cpu().numpy().view(np.uint32), ep), f"case {case}: prefix"

            comps, ecomps = [], []
            for w in range(W):
                g = rng.standard_normal(n).astype(np.float32)
                gt, ghost = _device_view(g, bf16, int(rng.choice([0, shift])))
                guard = torch.full((nnz + 8,), 7, dtype=gt.dtype, device="cuda")
                osh = int(rng.choice([0, 1, 2]))
                out = guard[osh:osh + nnz]
                pac.pac_compress(h, gt, m, p, out, nnz)
                ec = oracle.compress(ghost, em, nnz, dt)
                torch.cuda.synchronize()
                assert np.array_equal(_bits(out), ec.view(_bits(out).dtype)), f"case {case}: gather, worker {w}"
                assert bool((guard[:osh].float() == 7).all()) and bool((guard[osh + nnz:].float() == 7).all()), \
                    f"case {case}: gather wrote outside its buffer"
                comps.append(out)
                ecomps.append(ec)

            red = torch.empty(nnz, dtype=comps[0].dtype, device="cuda")
            pac.pac_reduce_local(h, comps, red, nnz)
            er = oracle.reduce_local(ecomps, dt)
            torch.cuda.synchronize()
            assert np.array_equal(_bits(red), er.view(_bits(red).dtype)), f"case {case}: sum"

            guard = torch.full((n + 8,), 5, dtype=red.dtype, device="cuda")
            dsh = int(rng.choice([0, shift]))
            dense = guard[dsh:dsh + n]
            pac.pac_decompress(h, red, m, p, dense, nnz)
            ed = oracle.decompress(er, em, n, dt)
            torch.cuda.synchronize()
            assert np.array_equal(_bits(dense), ed.view(_bits(dense).dtype)), f"case {case}: scatter"
            assert bool((guard[:dsh].float() == 5).all()) and bool((guard[dsh + n:].float() == 5).all()), \
                f"case {case}: scatter wrote outside its buffer"

            x = rng.standard_normal(n).astype(np.float32)
            xt = torch.from_numpy(x).cuda()
            alpha = float(np.float32(rng.random() * 0.1))
            pac.pac_decompress_update(h, red, m, p, alpha, xt, nnz)
            ex = oracle.decompress_update(er, em, x, alpha, dt)
            torch.cuda.synchronize()
            assert np.array_equal(xt.cpu().numpy().view(np.uint32), ex.view(np.uint32)), f"case {case}: fused update"
    finally:
        ctx.close()

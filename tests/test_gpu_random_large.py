"""pac_build_mask on large seeded random inputs: 60 to 400 million elements, random scope tables (so that scopes
of every sampling stride, counted-in-full ones and small ones sit side by side, with cuts at arbitrary offsets),
random sparsities including 0 and 1, and the value kinds that stress the selection: continuous weights, an
already pruned model, magnitudes constant over each 16384-element tile (sampled brackets miss), a handful of
distinct values, one constant.  Mask and prefix whole against the oracle; no error bit in the status word."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

KINDS = ["gauss", "pruned", "tilec", "ties", "equal"]


def make_weights(kind, n, dev, gen, rng):
    w = torch.randn(n, device=dev, generator=gen) * 0.02
    if kind == "pruned":
        w[w.abs() < float(rng.choice([0.0135, 0.0256, 0.0329]))] = 0.0      # 50 %, 80 %, 90 % of exact zeros
    elif kind == "tilec":
        t = 16384
        per = torch.rand(n // t + 2, device=dev, generator=gen) * 4 + 0.01
        w = per.repeat_interleave(t)[:n].contiguous()
    elif kind == "ties":
        w = torch.randint(-8, 9, (n,), device=dev, generator=gen).float() / 8.0
    elif kind == "equal":
        w.fill_(0.5)
    return w


@pytest.mark.parametrize("case", range(8))
def test_large_random_scope_tables(case):
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    rng = np.random.default_rng(9100 + case)
    n = int(rng.integers(60_000_000, 400_000_000))
    kind = KINDS[case % len(KINDS)]
    nseg = int(rng.choice([1, 2, 5, 40, 300]))
    gen = torch.Generator(device=dev)
    gen.manual_seed(9200 + case)
    w = make_weights(kind, n, dev, gen, rng)
    offs = [0, n] if nseg == 1 else [0] + [int(x) for x in np.sort(rng.integers(0, n + 1, nseg - 1))] + [n]
    sp = [float(rng.choice([0.0, 0.3, 0.5, 0.8, 0.9, 0.95, 0.99, 1.0])) for _ in range(len(offs) - 1)]
    print(f"[large] case {case}: n={n} kind={kind} scopes={len(offs) - 1}", flush=True)
    ctx = pac.PacContext(max_elems=n, max_segments=len(offs) - 1, device=0)
    try:
        m, p, k = ctx.build_mask(w, offs, sp)
        torch.cuda.synchronize()
        st = ctx.device_status(clear=True)
        em, ep, ek = oracle.build_mask(w.cpu().numpy(), offs, sp)
        assert k == ek
        assert np.array_equal(m.cpu().numpy().view(np.uint64), em), f"mask words differ (status {st:#x})"
        assert np.array_equal(p.cpu().numpy().view(np.uint32), ep), "prefix differs"
        assert st & pac.PAC_DEV_ERROR_MASK == 0, f"status {st:#x}"
    finally:
        ctx.close()
        del w
        torch.cuda.empty_cache()

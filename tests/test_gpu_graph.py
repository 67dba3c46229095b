"""The whole step captured in a HIP graph: the library launches kernels only (no memset, no allocation,
no host synchronisation once the scope table is on the device), so a step can be recorded once and
replayed.  Every replay is checked against the eager result, with eager work and synchronisations of the
program's own between the replays and fresh inputs in the captured buffers."""
import numpy as np
import pytest
import torch

from synth import make_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("config_id", [1, 2])
def test_step_replays_from_a_graph(config_id):
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    wl = make_workload(config_id, device=dev)
    n, W = wl.n, wl.workers
    sp = wl.sparsity_at(0)
    nseg = len(wl.scope_offsets) - 1
    ctx = pac.PacContext(max_elems=n, max_segments=nseg, device=0)
    try:
        h = ctx.handle
        words = (n + 63) // 64
        k = sum(pac.pac_keep_count(wl.scope_offsets[i + 1] - wl.scope_offsets[i], sp[i]) for i in range(nseg))
        weights = wl.weights.clone()
        grads = [g.clone() for g in wl.grads]
        mask = torch.empty(words, dtype=torch.int64, device=dev)
        prefix = torch.empty(words, dtype=torch.int32, device=dev)
        compact = [torch.empty(k, dtype=grads[0].dtype, device=dev) for _ in range(W)]
        red = torch.empty(k, dtype=grads[0].dtype, device=dev)
        dense = torch.empty(n, dtype=grads[0].dtype, device=dev)

        def step():
            nnz = pac.pac_build_mask(h, weights, wl.scope_offsets, sp, mask, prefix)
            for w in range(W):
                pac.pac_compress(h, grads[w], mask, prefix, compact[w], nnz)
            pac.pac_reduce_local(h, compact, red, nnz)
            pac.pac_decompress(h, red, mask, prefix, dense, nnz)

        step()                                   # eager warm-up: uploads the scope table, one-time set-up
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        torch.cuda.synchronize()

        gen = torch.Generator(device=dev)
        gen.manual_seed(77)
        for replay in range(4):
            # fresh inputs in the captured buffers, written eagerly
            weights.copy_(torch.randn(n, device=dev, generator=gen) * 0.02)
            for g in grads:
                g.copy_(torch.randn(n, device=dev, generator=gen).to(g.dtype))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = (mask.clone(), prefix.clone(), red.clone(), dense.clone())
            mask.zero_(); prefix.zero_(); red.zero_(); dense.zero_()
            torch.cuda.synchronize()
            step()                               # the same step, eagerly
            torch.cuda.synchronize()
            assert torch.equal(got[0], mask) and torch.equal(got[1], prefix), f"replay {replay}: mask differs"
            assert torch.equal(got[2].view(torch.int16 if red.dtype == torch.bfloat16 else torch.int32),
                               red.view(torch.int16 if red.dtype == torch.bfloat16 else torch.int32))
            assert torch.equal(got[3].view(torch.int16 if red.dtype == torch.bfloat16 else torch.int32),
                               dense.view(torch.int16 if red.dtype == torch.bfloat16 else torch.int32))
    finally:
        ctx.close()


def test_two_contexts_on_two_streams_do_not_interfere():
    """Two contexts, each on a stream of its own, interleaved from the host: same results as one after the other."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    wls = [make_workload(2, device=dev), make_workload(1, device=dev)]
    ctxs = [pac.PacContext(max_elems=wl.n, max_segments=len(wl.scope_offsets) - 1, device=0) for wl in wls]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        def run(i, stream):
            wl, ctx = wls[i], ctxs[i]
            sp = wl.sparsity_at(0)
            mask, prefix, k = ctx.build_mask(wl.weights, wl.scope_offsets, sp, stream=stream)
            compact = [ctx.compress(g, mask, prefix, k, stream=stream) for g in wl.grads]
            red = ctx.reduce_local(compact, k, stream=stream)
            return mask, prefix, ctx.decompress(red, mask, prefix, wl.n, k, stream=stream)

        torch.cuda.synchronize()
        ref = [run(i, None) for i in range(2)]
        torch.cuda.synchronize()
        for _ in range(5):
            for s in streams:
                s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(streams[0]):
                a = run(0, streams[0])
            with torch.cuda.stream(streams[1]):
                b = run(1, streams[1])
            torch.cuda.synchronize()
            for got, want in ((a, ref[0]), (b, ref[1])):
                assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
                assert torch.equal(got[2].view(torch.int32), want[2].view(torch.int32))
    finally:
        for c in ctxs:
            c.close()



def test_cyclic_sparsity_schedule_keeps_its_tables_resident_and_replays_from_graphs():
    """The per-layer schedule of the largest workload changes the scope table every step (s = 0.5, 0.8, 0.95
    in turn).  The context keeps the last few tables on the device, so after one eager round every step of
    the cycle enqueues kernels only: each is captured in a graph of its own and replayed, twice round the
    cycle with fresh inputs, against the oracle.  A table the context has not seen is refused under capture."""
    import oracle
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    wl = make_workload(5, device=dev, reduced=True, workers=2)
    n, W = wl.n, wl.workers
    nseg = len(wl.scope_offsets) - 1
    ctx = pac.PacContext(max_elems=n, max_segments=nseg, device=0)
    try:
        h = ctx.handle
        words = (n + 63) // 64
        cycle = [wl.sparsity_at(t) for t in range(3)]
        ks = [sum(pac.pac_keep_count(wl.scope_offsets[i + 1] - wl.scope_offsets[i], sp[i]) for i in range(nseg)) for sp in cycle]
        weights = wl.weights.clone()
        grads = [g.clone() for g in wl.grads]
        mask = torch.empty(words, dtype=torch.int64, device=dev)
        prefix = torch.empty(words, dtype=torch.int32, device=dev)
        compact = [torch.empty(max(ks), dtype=torch.float32, device=dev) for _ in range(W)]
        red = torch.empty(max(ks), dtype=torch.float32, device=dev)
        dense = torch.empty(n, dtype=torch.float32, device=dev)

        def step(t):
            nnz = pac.pac_build_mask(h, weights, wl.scope_offsets, cycle[t], mask, prefix)
            for w in range(W):
                pac.pac_compress(h, grads[w], mask, prefix, compact[w], nnz)
            pac.pac_reduce_local(h, compact, red, nnz)
            pac.pac_decompress(h, red, mask, prefix, dense, nnz)

        for t in range(3):                       # one eager round: the three tables become resident
            step(t)
        torch.cuda.synchronize()
        graphs = []
        for t in range(3):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(t)
            graphs.append(g)
        torch.cuda.synchronize()

        # a table that is not resident cannot be uploaded under capture: refused, nothing enqueued
        g = torch.cuda.CUDAGraph()
        refused = None
        with torch.cuda.graph(g):
            try:
                pac.pac_build_mask(h, weights, wl.scope_offsets, [0.25] * nseg, mask, prefix)
            except pac.PacError as e:
                refused = e
        torch.cuda.synchronize()
        assert refused is not None and refused.status == -1
        del g

        gen = torch.Generator(device=dev)
        gen.manual_seed(99)
        for rnd in range(2):
            for t in range(3):
                weights.copy_(torch.randn(n, device=dev, generator=gen) * 0.02)
                for gr in grads:
                    gr.copy_(torch.randn(n, device=dev, generator=gen))
                mask.zero_(); prefix.zero_(); red.zero_(); dense.zero_()
                torch.cuda.synchronize()
                graphs[t].replay()
                torch.cuda.synchronize()
                em, ep, k = oracle.build_mask(weights.cpu().numpy(), wl.scope_offsets, cycle[t])
                assert k == ks[t]
                assert np.array_equal(mask.cpu().numpy().view(np.uint64), em), f"round {rnd} step {t}: mask"
                assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep), f"round {rnd} step {t}: prefix"
                e_red = oracle.reduce_local([oracle.compress(gr.cpu().numpy(), em, k) for gr in grads])
                assert np.array_equal(red[:k].cpu().numpy().view(np.uint32), e_red.view(np.uint32))
                e_out = oracle.decompress(e_red, em, n)
                assert np.array_equal(dense.cpu().numpy().view(np.uint32), e_out.view(np.uint32))
        assert ctx.device_status() & pac.PAC_DEV_ERROR_MASK == 0

        # more distinct tables than slots, eagerly: the oldest is replaced, results stay right
        for s in (0.1, 0.2, 0.3, 0.4, 0.6, 0.1):
            nnz = pac.pac_build_mask(h, weights, wl.scope_offsets, [s] * nseg, mask, prefix)
            torch.cuda.synchronize()
            em, ep, k = oracle.build_mask(weights.cpu().numpy(), wl.scope_offsets, [s] * nseg)
            assert k == nnz and np.array_equal(mask.cpu().numpy().view(np.uint64), em)
            assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep)
    finally:
        ctx.close()

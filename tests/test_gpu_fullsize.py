"""GPU parity at the full sizes of the measured configurations, in the launch configuration bench.py
times (same context sizing, same calls, inputs generated on the device and copied to the host for
the oracle), with every configuration's stated number of workers.  The oracle is fast enough to check
every output element at these sizes, so nothing is sampled.  To bound host memory the oracle is driven
one worker at a time: a worker's gradient is copied to the host once, gathered by the oracle for every
step of the sparsity schedule, compared with the library's compact buffer of that (step, worker), and
only the oracle's compact buffers are kept for the sum.
"""
import time

import numpy as np
import pytest
import torch

import oracle
from synth import make_workload

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1200)]


def raw_np(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.float32:
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_full(config_id: int, steps=(0,)):
    import paper_2505_18563_amd as pac
    assert torch.cuda.is_available()
    dev = torch.device("cuda", 0)
    t_start = time.perf_counter()
    wl = make_workload(config_id, device=dev)
    n, W = wl.n, wl.workers
    code = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    raw_dtype = np.uint32 if code == oracle.F32 else np.uint16
    nseg = len(wl.scope_offsets) - 1
    print(f"[full] C{config_id} {wl.name} n={n} W={W} nseg={nseg} dtype={wl.dtype}", flush=True)
    ctx = pac.PacContext(max_elems=n, max_segments=nseg, device=0)
    try:
        # the library: every step of the schedule, results kept on the device
        gpu = []
        for step in steps:
            sp = wl.sparsity_at(step)
            mask, prefix, nnz = ctx.build_mask(wl.weights, wl.scope_offsets, sp)
            compact = [ctx.compress(g, mask, prefix, nnz) for g in wl.grads]
            red = ctx.reduce_local(compact, nnz)
            out = ctx.decompress(red, mask, prefix, n, nnz)
            gpu.append((sp, mask, prefix, nnz, compact, red, out))
        torch.cuda.synchronize()
        assert ctx.device_status() == 0, "the library raised a device-side flag"
        print(f"[full]   library done for steps {list(steps)} ({time.perf_counter() - t_start:.1f} s)", flush=True)

        # the oracle's masks
        w_np = wl.weights.cpu().numpy()
        e_masks = []
        for (sp, mask, prefix, nnz, _, _, _) in gpu:
            em, ep, k = oracle.build_mask(w_np, wl.scope_offsets, sp)
            assert nnz == k
            assert np.array_equal(mask.cpu().numpy().view(np.uint64), em), "mask words differ"
            assert np.array_equal(prefix.cpu().numpy().view(np.uint32), ep), "prefix differs"
            e_masks.append((em, k))
            print(f"[full]   s={sp[0]}: mask and prefix equal, k={k} ({time.perf_counter() - t_start:.1f} s)", flush=True)
        del w_np

        # one worker at a time: gather with the oracle, compare, keep the oracle's compact buffer
        e_compact = [[] for _ in gpu]
        for w in range(W):
            g_np = raw_np(wl.grads[w])
            g_arg = g_np.view(np.float32) if code == oracle.F32 else g_np
            for si, (em, k) in enumerate(e_masks):
                ec = oracle.compress(g_arg, em, k, code)
                got = raw_np(gpu[si][4][w])
                assert np.array_equal(got, ec.view(raw_dtype)), f"step {steps[si]}: compact[{w}] differs"
                e_compact[si].append(ec)
                del got
            del g_np, g_arg
            print(f"[full]   worker {w}: compact buffers equal ({time.perf_counter() - t_start:.1f} s)", flush=True)

        # the sum over all W workers and the scatter
        for si, (em, k) in enumerate(e_masks):
            e_red = oracle.reduce_local(e_compact[si], code)
            e_compact[si] = None
            got_red = raw_np(gpu[si][5])
            assert np.array_equal(got_red, e_red.view(raw_dtype)), f"step {steps[si]}: reduced buffer differs"
            del got_red
            e_out = oracle.decompress(e_red, em, n, code)
            got_out = raw_np(gpu[si][6])
            assert np.array_equal(got_out, e_out.view(raw_dtype)), f"step {steps[si]}: dense output differs"
            del e_out, got_out, e_red
            print(f"[full]   step {steps[si]}: W={W} sum and scatter equal ({time.perf_counter() - t_start:.1f} s)", flush=True)
    finally:
        ctx.close()
        del wl
        torch.cuda.empty_cache()


def test_full_config3_bert_base_shaped_global_prune():
    run_full(3)


def test_full_config4_gpt2_medium_shaped_bf16_w16():
    """The benchmark workload: 354,823,168 elements, one prune scope (sampled bracket), 16 bf16 workers."""
    run_full(4)


def test_full_config4_mask_of_the_pruned_model_and_of_a_constant_tensor():
    """The weights a training loop holds after its first step: pruned positions set to exactly +0 by the
    library's own fused update (Eq. 1 and 2), so 90 % of the 354,823,168 elements tie at zero; re-pruned at
    the same sparsity, the same mask must come back, on the fast path.  Then one all-equal scope of the same
    length, where the tie rule alone decides.  Masks and prefixes whole against the oracle."""
    import paper_2505_18563_amd as pac
    dev = torch.device("cuda", 0)
    wl = make_workload(4, device=dev)
    n = wl.n
    sp = wl.sparsity_at(0)
    ctx = pac.PacContext(max_elems=n, max_segments=1, device=0)
    try:
        mask, prefix, nnz = ctx.build_mask(wl.weights, wl.scope_offsets, sp)
        compact = [ctx.compress(g, mask, prefix, nnz) for g in wl.grads[:2]]
        red = ctx.reduce_local(compact, nnz)
        w2 = wl.weights.clone()
        pac.pac_decompress_update(ctx.handle, red, mask, prefix, 1e-3, w2, nnz)
        torch.cuda.synchronize()
        assert int((w2 == 0).sum()) >= n - nnz
        print(f"[full] pruned C4 weights: {n - nnz} zeros of {n}", flush=True)
        for label, w in (("pruned", w2), ("all-equal", torch.full((n,), 0.02, device=dev))):
            m2, p2, k2 = ctx.build_mask(w, wl.scope_offsets, sp)
            torch.cuda.synchronize()
            st = ctx.device_status(clear=True)
            em, ep, k = oracle.build_mask(w.cpu().numpy(), wl.scope_offsets, sp)
            assert k2 == k == nnz
            assert np.array_equal(m2.cpu().numpy().view(np.uint64), em), f"{label}: mask words differ"
            assert np.array_equal(p2.cpu().numpy().view(np.uint32), ep), f"{label}: prefix differs"
            assert st == 0, f"{label}: device status {st:#x} (an error bit, or a slow path)"
            if label == "pruned":
                assert np.array_equal(em, mask.cpu().numpy().view(np.uint64)), "re-pruning the pruned model moved the mask"
            print(f"[full]   {label}: mask and prefix equal, status 0", flush=True)
            del w, m2, p2, em, ep
    finally:
        ctx.close()
        del wl
        torch.cuda.empty_cache()


def test_full_config5_decoder_1p3b_per_layer_schedule_all_eight_workers():
    """1,315,723,264 elements, 292 prune scopes (the large ones sampled), every sparsity of the schedule,
    all 8 workers: 24 gathers, three 8-way fp32 sums of up to 657,861,632 elements, three scatters."""
    run_full(5, steps=(0, 1, 2))


@pytest.mark.parametrize("config_id", [6, 7, 8])
def test_full_paper_models_pruning_ratio_half_eight_workers(config_id):
    """The paper's own evaluation models (VGG19, ResNet152, ViT-Base-16 with a 100-way classifier) at its
    default pruning ratio 0.5 and its 8 workers (Sec. IV-A, IV-C), every tensor its own prune scope."""
    run_full(config_id)

"""stage_blend_update_noalloc (the update/blend entry point that keeps its reduction partials in a device array
of the library instead of the caller's workspace) against stage_blend_update: same kernels, same arguments, so
every output -- momentum, the new version in the ring, both bf16 compute copies, the diagnostics -- must be the
same bits.  Two calls in a row, the second on a much smaller stage (fewer blocks than the first call left
partials for)."""
import numpy as np
import pytest

from synth_inputs import workloads as W

pytestmark = pytest.mark.gpu


def _stage(specs, params, mb, n):
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    return GpuStage([layer_tuple(l) for l in specs], params, dtype="bf16", mb=mb, n=n, stage_index=0, num_stages=2,
                    policy="convex", lam=0.4, lr=0.01, momentum=0.9, needs_dx=True)


def _to_backward(st, w, mb, n):
    """Two mini-batches forward, backward of the first: a gradient is pending, mini-batch 1 waits on version 0."""
    import torch
    for j in range(2):
        x = torch.from_numpy(W.stage_input(w, 0, j).reshape(n * mb, -1)).cuda().to(st.tdtype)
        for ub in range(n):
            st.forward(j, ub, x[ub * mb:(ub + 1) * mb])
    dy = torch.from_numpy(W.stage_upstream_grad(w, 0, 0).reshape(n * mb, -1)).cuda().to(st.tdtype)
    st.backward(0, dy)


def _outputs(st, version):
    import torch
    torch.cuda.synchronize()
    return {"m": st.momentum.clone(), "W_new": st.export(version).clone(), "wfwd": st.wfwd.clone(), "wb": st.wbwd.clone(),
            "diag": st.diag.clone()}


def test_noalloc_update_matches_update_twice_in_a_row():
    import torch
    from paper_2509_23241_amd import binding as B
    cases = []
    for name, specs, mb, n in (("big", (W.Dense(512, 768, "gelu"), W.Dense(768, 512, "gelu")), 32, 2),
                               ("small", (W.Dense(24, 40, "gelu"),), 4, 2)):
        w = W.Workload(name=f"noalloc_{name}", dtype="bf16", stages=(tuple(specs), ()), mb=mb, n=n, classes=2)
        params = W.init_params(w, 0)
        rng = np.random.default_rng(3)
        params = [p if p.ndim > 1 else W.round_f32(p + 0.1 * rng.standard_normal(p.shape)) for p in params]
        ref, new = _stage(specs, params, mb, n), _stage(specs, params, mb, n)
        _to_backward(ref, w, mb, n)
        _to_backward(new, w, mb, n)
        assert torch.equal(ref.grad, new.grad)                       # same kernels on the same inputs
        cases.append((name, ref, new))
    for name, ref, new in cases:                                     # the existing entry point
        assert ref.blend_update(0, 1) == 1
    for name, ref, new in cases:                                     # the new one: big, then small, back to back
        print("stage_blend_update_noalloc:", name, "P =", new.P, flush=True)
        assert new.blend_update_noalloc(0, 1) == 1
    for name, ref, new in cases:
        a, b = _outputs(ref, 1), _outputs(new, 1)
        for k in a:
            assert torch.equal(a[k], b[k]), (name, k)
        assert float(a["diag"][B.TP_DIAG_GRAD_SQ]) > 0 and float(a["diag"][B.TP_DIAG_WB_SQ]) > 0
        assert float(a["wb"].float().abs().sum()) > 0                # the look-ahead blend was built (delta 1)
        qa, qb = ref.query(), new.query()
        assert qa.latest_version == qb.latest_version == 1 and qa.wb_ready_mb == qb.wb_ready_mb == 1
        # and the stage goes on as usual: the next backward takes the blend the call built
        dy = torch.randn(new.n * new.mb, new.out_elems, device="cuda").to(new.tdtype)
        dxa, da = ref.backward(1, dy)
        dxb, db = new.backward(1, dy)
        assert da == db == 1 and torch.equal(dxa, dxb) and torch.equal(ref.grad, new.grad)
        assert ref.blend_update(1) == 2 and new.blend_update_noalloc(1) == 2      # without a look-ahead
        a, b = _outputs(ref, 2), _outputs(new, 2)
        for k in ("m", "W_new", "wfwd", "diag"):
            assert torch.equal(a[k], b[k]), (name, k, "second update")
        ref.close()
        new.close()

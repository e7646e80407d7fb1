"""V-TiMePReSt looks for newer weights even during a pass (Section "V-TiMePReSt", Challenge 1): when an
update lands at a stage between two micro-batches of one mini-batch, the later micro-batch runs on the
newer version.  The emulated schedule is mini-batch granular and never does that, so this test drives the
stage by hand: the versions reported per micro-batch, the outputs, the gradients and the update are
compared with the oracle following the same order.  Under the stashing policies the same order is refused
(a mini-batch has ONE forward version to stash)."""
import numpy as np
import pytest

from oracle.stage import Stage, StageError
from parity_utils import TOL, oracle_flat_to_arena, rel_err, to_np
from synth_inputs import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_update_between_micro_batches_under_v(dtype):
    import torch
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple

    specs = (W.Dense(48, 64, "gelu"), W.Dense(64, 32, "none"))
    mb, n = 8, 2
    w = W.Workload(name=f"vpass_{dtype}", dtype=dtype, stages=(specs, ()), mb=mb, n=n, classes=2)
    params = W.init_params(w, 0)
    ost = Stage(specs, params, policy="latest", lam=0.1, lr=0.05, momentum=0.9, n=n, storage=W.round_bf16 if dtype == "bf16" else None)
    st = GpuStage([layer_tuple(l) for l in specs], params, dtype=dtype, mb=mb, n=n, stage_index=0, num_stages=2,
                  policy="latest", lam=0.1, lr=0.05, momentum=0.9, needs_dx=True)
    tol = TOL[dtype]
    xs = [W.stage_input(w, 0, j) for j in range(2)]
    dys = [W.stage_upstream_grad(w, 0, j) for j in range(2)]
    xt = [torch.from_numpy(x).cuda().to(st.tdtype) for x in xs]
    y = [torch.empty(n * mb, 32, dtype=st.tdtype, device="cuda") for _ in range(2)]

    def fwd(j, ub):
        ref = ost.forward(j, ub, xs[j][ub * mb:(ub + 1) * mb])
        _, v = st.forward(j, ub, xt[j][ub * mb:(ub + 1) * mb], y[j][ub * mb:(ub + 1) * mb])
        assert rel_err(to_np(y[j][ub * mb:(ub + 1) * mb]), ref) <= tol
        return v

    def bwd(j):
        ref_dx = ost.backward(j, dys[j])
        dx, delta = st.backward(j, torch.from_numpy(dys[j]).cuda().to(st.tdtype))
        assert delta == 0
        assert rel_err(to_np(dx), ref_dx) <= tol
        assert rel_err(to_np(st.grad), oracle_flat_to_arena(st, ost.flat(ost.g))) <= tol
        ost.update(j)
        assert st.blend_update(j) == ost.latest
        assert rel_err(to_np(st.export(ost.latest)), oracle_flat_to_arena(st, ost.flat(ost.weights[ost.latest]))) <= tol

    assert fwd(0, 0) == 0 and fwd(0, 1) == 0
    assert fwd(1, 0) == 0                      # mini-batch 1 starts on version 0 ...
    bwd(0)                                     # ... the update of mini-batch 0 lands in the middle of its pass ...
    assert fwd(1, 1) == 1                      # ... and its second micro-batch already runs on version 1
    assert ost.inflight[1]["versions"] == [0, 1]
    bwd(1)                                     # one backward for both micro-batches, on the latest weights (version 1)
    assert ost.latest == 2 and st.query().latest_version == 2
    st.close()


def test_update_between_micro_batches_is_refused_when_stashing():
    from paper_2509_23241_amd import binding as B
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    import torch

    specs = (W.Dense(16, 16, "none"),)
    w = W.Workload(name="vpass_stash", dtype="f32", stages=(specs, ()), mb=4, n=2, classes=2)
    params = W.init_params(w, 0)
    ost = Stage(specs, params, policy="convex", lam=0.1, lr=0.05, momentum=0.9, n=2)
    st = GpuStage([layer_tuple(l) for l in specs], params, dtype="f32", mb=4, n=2, stage_index=0, num_stages=2,
                  policy="convex", lam=0.1, lr=0.05, momentum=0.9, needs_dx=True)
    x = torch.from_numpy(W.stage_input(w, 0, 0)).cuda().float()
    xn = W.stage_input(w, 0, 0)
    y = torch.empty(8, 16, device="cuda")
    for ub in range(2):
        st.forward(0, ub, x[ub * 4:(ub + 1) * 4], y[ub * 4:(ub + 1) * 4]); ost.forward(0, ub, xn[ub * 4:(ub + 1) * 4])
    st.forward(1, 0, x[:4], y[:4]); ost.forward(1, 0, xn[:4])
    dy = W.stage_upstream_grad(w, 0, 0)
    st.backward(0, torch.from_numpy(dy).cuda().float()); ost.backward(0, dy)
    st.blend_update(0); ost.update(0)
    with pytest.raises(B.StageLibError) as ei:
        st.forward(1, 1, x[4:], y[4:])
    assert ei.value.code == B.TP_ESTATE
    with pytest.raises(StageError):
        ost.forward(1, 1, xn[4:])
    st.close()

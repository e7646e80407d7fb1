"""GPU parity of a single stage on synthetic inputs and upstream gradients, over shapes chosen to
hit every tile edge of the GEMM kernels (rows, columns and contraction extents that are smaller
than a tile, one past a tile, not a multiple of 8, ...), in both precisions."""
import numpy as np
import pytest

from oracle.stage import Stage
from parity_utils import TOL, oracle_flat_to_arena, rel_err, to_np
from synth_inputs import normal, round_bf16, round_f32

pytestmark = pytest.mark.gpu

SHAPES = [
    # (mb, n, in, hidden, out)
    (1, 1, 8, 8, 8),
    (33, 2, 64, 72, 136),
    (130, 1, 200, 264, 72),
    (64, 3, 520, 128, 1000),
    (7, 2, 19, 23, 5),          # nothing is a multiple of 8: generic kernel
    (256, 2, 256, 512, 256),
    # outputs of 4096 x 4096 (the 256 x 256 tile: 256 workgroups) over contractions of one and three k tiles:
    # forward and input gradient ...
    (4096, 1, 64, 4096, 192),
    # ... and weight gradient (64 rows in the mini-batch)
    (64, 1, 4096, 4096, 8),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", SHAPES)
def test_stage_forward_backward_update(shape, dtype):
    import torch
    from paper_2509_23241_amd.runner import GpuStage

    mb, n, fin, hid, fout = shape
    cast = round_bf16 if dtype == "bf16" else round_f32
    layers = [(fin, hid, "gelu"), (hid, fout, "gelu")]
    name = f"shape{shape}{dtype}"
    params = []
    for li, (a, b, _) in enumerate(layers):
        params.append(round_f32(normal(f"{name}/W{li}", (b, a), std=float(np.sqrt(2.0 / a)))))
        params.append(round_f32(normal(f"{name}/b{li}", (b,), std=0.1)))
    x = cast(normal(f"{name}/x", (n * mb, fin)))
    dy = cast(normal(f"{name}/dy", (n * mb, fout), std=1.0 / np.sqrt(fout)))

    class Spec:
        def __init__(self, act):
            self.act = act
    ost = Stage([Spec("gelu"), Spec("gelu")], params, policy="convex", lam=0.1, lr=0.01, momentum=0.9, n=n)
    y_ref = np.concatenate([ost.forward(0, ub, x[ub * mb:(ub + 1) * mb]) for ub in range(n)])
    dx_ref = ost.backward(0, dy)
    g_ref = ost.flat(ost.g)
    ost.update(0)

    tol = TOL[dtype]
    st = GpuStage(layers, params, dtype=dtype, mb=mb, n=n, stage_index=1, num_stages=2, policy="convex", lam=0.1,
                  lr=0.01, momentum=0.9, ring_capacity=2, max_in_flight=1)
    xt = torch.from_numpy(x).cuda().to(st.tdtype)
    y = torch.empty(n * mb, fout, dtype=st.tdtype, device="cuda")
    for ub in range(n):
        st.forward(0, ub, xt[ub * mb:(ub + 1) * mb], y[ub * mb:(ub + 1) * mb])
    dx, delta = st.backward(0, torch.from_numpy(dy).cuda().to(st.tdtype))
    assert delta == 0
    errs = {"y": rel_err(to_np(y), y_ref), "dx": rel_err(to_np(dx), dx_ref),
            "g": rel_err(to_np(st.grad), oracle_flat_to_arena(st, g_ref))}
    assert st.blend_update(0) == 1
    errs["W_new"] = rel_err(to_np(st.export(1)), oracle_flat_to_arena(st, ost.flat(ost.weights[1])))
    errs["m"] = rel_err(to_np(st.momentum), oracle_flat_to_arena(st, ost.flat(ost.m)))
    print(shape, dtype, {k: f"{v:.2e}" for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= tol, (k, v)
    st.close()

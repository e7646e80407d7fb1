"""The statistical-efficiency harness on a small student: every policy trains (the loss falls), the
one-stage run has no staleness, and the stash sizes per stage are those the method prescribes
(one version under V-TiMePReSt, K - s versions under the stashing policies; Section "Memory Overhead")."""
import numpy as np
import pytest
import torch

from oracle.pipeline import Pipeline
from synth_inputs import workloads as W

pytestmark = pytest.mark.gpu


def _oracle_losses(w, policy, data, minibatches):
    params = [W.init_params(w, s) for s in range(w.K)]
    pipe = Pipeline(w.stages, params, policy=policy, lam=w.lam, lr=w.lr, momentum=w.momentum, n=w.n, mb=w.mb)
    pipe.run(minibatches, lambda j: data.host(j)[0], lambda j: data.host(j)[1])
    return np.array([pipe.losses[j] for j in range(minibatches)])


@pytest.mark.parametrize("policy", ["latest", "eq1", "convex", "stashed"])
def test_loss_sequence_equals_the_oracles_fp32(policy):
    # the statistical-efficiency experiment on the teacher's data, mini-batch by mini-batch against the fp64 oracle
    # pipeline run on the same inputs and labels: 30 mini-batches through 4 stages, staleness up to 3
    from paper_2509_23241_amd import convergence as C

    data = C.TeacherData(32, 64, 8, 16 * 2, torch.device("cuda:0"), torch.float32)
    w = C.student(64, 32, 8, 4, 2, 16, 2, 0.05, 0.3, "f32")
    got, _ = C.run_policy(w, policy, data, 30)
    ref = _oracle_losses(w, policy, data, 30)
    err = np.abs(got - ref) / np.abs(ref)
    print(policy, "loss 0, 29:", ref[0], ref[29], "largest relative difference", err.max())
    assert err.max() <= 1e-4, (policy, err)
    assert ref[-5:].mean() < ref[:5].mean()                       # and it trains


def test_loss_sequence_equals_the_oracles_bf16_wide_mlp_reduced():
    # the 4-stage 8-layer GELU MLP of the headline configuration at width / 8 and micro-batch / 8 (bf16 activations,
    # fp32 master weights, 8 micro-batches), trained on the teacher's labels: loss per mini-batch against the oracle
    from paper_2509_23241_amd import convergence as C

    w = W.mlp_wide(width=512, mb=32, n=8, classes=1000)
    data = C.TeacherData(512, 256, 1000, w.mb * w.n, torch.device("cuda:0"), torch.bfloat16)
    for policy in ("latest", "convex"):
        got, stash = C.run_policy(w, policy, data, 12)
        ref = _oracle_losses(w, policy, data, 12)
        err = np.abs(got - ref) / np.abs(ref)
        print(policy, "loss 0, 11:", ref[0], ref[11], "largest relative difference", err.max())
        assert err.max() <= 2e-2, (policy, err)
        assert [c for c, _ in stash] == ([1, 1, 1, 1] if policy == "latest" else [4, 3, 2, 1])


def test_policies_train_and_stash_sizes():
    from paper_2509_23241_amd import convergence as C

    dev = torch.device("cuda:0")
    data = C.TeacherData(32, 64, 8, 16 * 2, dev, torch.float32)
    K = 4
    final = {}
    for policy, stages in (("latest", 1), ("convex", 1), ("latest", K), ("eq1", K), ("convex", K), ("stashed", K)):
        w = C.student(64, 32, 8, stages, 8 // stages, 16, 2, 0.05, 0.1, "f32")
        loss, stash = C.run_policy(w, policy, data, 240)
        assert np.all(np.isfinite(loss)), policy
        assert loss[-40:].mean() < 0.93 * loss[:40].mean(), (policy, loss[:20].mean(), loss[-20:].mean())
        slots = [c for c, _ in stash]
        if policy == "latest":
            assert slots == [1] * stages
        else:
            assert slots == [stages - s for s in range(stages)]
        final[(policy, stages)] = loss
    # one stage = no staleness: the intermediate weight is the latest weight and the policies coincide
    assert np.array_equal(final[("latest", 1)], final[("convex", 1)])
    assert C.first_below(final[("latest", 1)], 1e9) == 20

"""The statistical-efficiency harness on a small student: every policy trains (the loss falls), the
one-stage run has no staleness, and the stash sizes per stage are those the method prescribes
(one version under V-TiMePReSt, K - s versions under the stashing policies; Section "Memory Overhead")."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


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

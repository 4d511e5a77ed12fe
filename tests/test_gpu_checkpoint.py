"""Checkpoint / resume: the method's whole per-worker state is (r, v) (Alg. 1 and Alg. 2 initialise nothing
else), so saving those two tensors after k steps, loading them into fresh buffers (fresh scratch, fresh message
buffers) and running k more steps must give bit-identical state and messages to 2k uninterrupted steps."""
import io

import numpy as np
import pytest

from paper_1802_06058_amd import workloads as W
from streams import sample_stream

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    import torch
    from paper_1802_06058_amd import vgc
    assert torch.cuda.is_available()
    vgc.load()
    return torch.device("cuda:0")


class Worker:
    def __init__(self, plan, dev, state=None):
        import torch
        self.plan, n = plan, plan.n
        if state is None:
            self.r = torch.zeros(n, dtype=torch.float32, device=dev)
            self.v = torch.zeros(n, dtype=torch.float32, device=dev)
        else:
            self.r, self.v = state["r"].to(dev), state["v"].to(dev)
        self.scratch = plan.new_scratch()
        self.scratch.fill_(0x5A)
        self.words = torch.empty(n, dtype=torch.int32, device=dev)
        self.hdrs, self.status = plan.new_headers(), plan.new_status()

    def step(self, g, s, hybrid):
        import torch
        from paper_1802_06058_amd import vgc
        if hybrid:
            vgc.accumulate_select_hybrid(g, s, self.r, self.v, self.plan, 2.0, 0.999, 0.004, self.scratch)
        else:
            vgc.accumulate_select(g, s, self.r, self.v, self.plan, 1.0, 0.999, self.scratch)
        vgc.pack(self.plan, self.scratch, self.words, self.hdrs, self.status)
        torch.cuda.synchronize()
        total, overflow = vgc.read_status(self.status)
        assert overflow == 0
        return self.words[:total].cpu().numpy().copy(), vgc.read_headers(self.hdrs)


@pytest.mark.parametrize("hybrid", [False, True])
def test_resume_from_saved_state_is_bit_identical(dev, hybrid):
    import torch
    from paper_1802_06058_amd import vgc
    sizes = [2048 * 7 + 13, 1, 5000, 2048 * 3, 77]
    groups = W.groups_from_sizes(sizes)
    plan = vgc.Plan(groups, dev)
    n, k = plan.n, 4
    inputs = []
    for step in range(2 * k):
        g, s = sample_stream(91, (int(hybrid), step), n, 16, "student", sigma=0.02)
        inputs.append((torch.from_numpy(g + np.float32(0.002)).to(dev), torch.from_numpy(s).to(dev)))
    straight = Worker(plan, dev)
    msgs = [straight.step(g, s, hybrid) for g, s in inputs]

    first = Worker(plan, dev)
    for g, s in inputs[:k]:
        first.step(g, s, hybrid)
    blob = io.BytesIO()
    torch.save({"r": first.r.cpu(), "v": first.v.cpu()}, blob)
    del first
    blob.seek(0)
    resumed = Worker(plan, dev, torch.load(blob, weights_only=True))
    for i, (g, s) in enumerate(inputs[k:]):
        words, hdrs = resumed.step(g, s, hybrid)
        assert hdrs == msgs[k + i][1]
        assert np.array_equal(words, msgs[k + i][0])
    assert torch.equal(resumed.r.view(torch.int32), straight.r.view(torch.int32))
    assert torch.equal(resumed.v.view(torch.int32), straight.v.view(torch.int32))
    assert sum(m[0].size for m in msgs[k:]) > 0

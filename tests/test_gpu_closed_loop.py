"""Closed loop on measured times: the controller is fed HIP-event timings of every worker's own
forward/backward launch instead of the synthetic plant.  Heterogeneity is emulated by repeating
a slow worker's launch r_k times (a worker r times slower per sample).  Timings are not
reproducible, so nothing here is compared bit for bit: the test checks the paper's goal state,
equal iteration times (Section "Proportional-Control Based Dynamic Policy"), and that the
dead-band stops the readjustments (subsection "Control stability")."""
import numpy as np
import pytest

from paper_2305_12213_amd import binding, synth

pytestmark = pytest.mark.gpu


def test_controller_equalises_measured_iteration_times():
    import torch
    spec = synth.mlp_spec([2048, 2048, 2048, 10], "bf16")
    K, G = 4, 4096
    slow = [1, 2, 4, 8]                                  # worker k is slow[k] times slower per sample
    model = binding.Model(spec)
    Pp = model.padded_params()
    params = torch.from_numpy(synth.flatten_params(synth.init_params(spec, "he", 3), 256)).cuda()
    nbytes = model.workspace_bytes(G, 1)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    model.bind(params, ws, nbytes, G, 1)
    grads = torch.empty(1, Pp, device="cuda")
    x, y = synth.make_batch(spec, "normal", G, 3, 0)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()

    def measure(b):
        """Wall time of each worker's iteration: its launch on its own rows, slow[k] times."""
        t, off = [], 0
        for k in range(K):
            if b[k] == 0:
                t.append(None); continue
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(slow[k]):
                binding.forward_backward(model, xd[off:off + b[k]], yd[off:off + b[k]], [b[k]], grads)
            e1.record(); e1.synchronize()
            t.append(e0.elapsed_time(e1)); off += b[k]
        busy = [v for v in t if v is not None]
        return [v if v is not None else sum(busy) / len(busy) for v in t]

    b = [G // K] * K
    gains = dict(kp=1.0, deadband=0.05, ewma_alpha=0.5, b_min=8, b_max=G)
    ctl = binding.Controller(b, G, gains, min_observations=2, adaptive_b_max=False)
    for _ in range(3):
        measure(b)                                        # warm-up (first launches, clocks)
    t0 = measure(b)
    history = []
    for it in range(40):
        t = measure(b)
        b, resized = ctl.observe(t)
        history.append((list(b), resized))
        assert sum(b) == G and min(b) >= 8
    t1 = measure(b)
    spread0 = (max(t0) - min(t0)) / (sum(t0) / K)
    spread1 = (max(t1) - min(t1)) / (sum(t1) / K)
    print("start b", [G // K] * K, "times", ["%.3f" % v for v in t0], "spread %.2f" % spread0)
    print("final b", b, "times", ["%.3f" % v for v in t1], "spread %.2f" % spread1,
          "readjustments", ctl.read()["readjustments"])
    assert spread0 > 1.0                                  # 8x heterogeneity at the equal split
    assert spread1 < 0.25                                 # iteration times equalised
    assert b[0] > b[1] > b[2] > b[3]                      # faster workers hold more samples
    assert not any(r for _, r in history[-10:])           # and the dead-band keeps it there

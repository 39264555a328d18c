"""The allocation-free entry point (dynb_forward_backward_static) against dynb_forward_backward.

Both run the same kernels; the only difference is where the scratch lives (a static device array
inside the library instead of the caller's workspace), so with the reference model bound for the
same batch and worker count the two gradient matrices must agree bit for bit.  Two calls in a row
per model, the second with a smaller input and fewer workers: the array then still holds the first
call's contents in another layout.
"""
import numpy as np
import pytest

from paper_2305_12213_amd import binding, synth

pytestmark = pytest.mark.gpu


def _reference(spec, params_dev, xd, yd, b):
    import torch
    model = binding.Model(spec)
    nbytes = model.workspace_bytes(max(1, sum(b)), len(b))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    model.bind(params_dev, ws, nbytes, max(1, sum(b)), len(b))
    grads = torch.full((len(b), model.padded_params()), float("nan"), device="cuda")
    binding.forward_backward(model, xd, yd, b, grads)
    torch.cuda.synchronize()
    return grads


CASES = [
    ("mlp bf16", lambda: synth.mlp_spec([96, 128, 10], "bf16"), [37, 5, 0, 22], [9, 3]),
    ("mlp f32", lambda: synth.mlp_spec([70, 33, 10], "f32"), [16, 1, 30], [4]),
    ("residual block bf16", lambda: synth.resnet_block_spec(8, (8, 8, 3), 5), [5, 3, 1], [2, 1]),
]


@pytest.mark.parametrize("name,make_spec,b_first,b_second", CASES, ids=[c[0] for c in CASES])
def test_static_scratch_matches_bound_workspace(dynb, name, make_spec, b_first, b_second):
    import torch
    spec = make_spec()
    params = synth.init_params(spec, "he", 3)
    pd = torch.from_numpy(synth.flatten_params(params, 256)).cuda()
    unbound = binding.Model(spec)                       # never bound: the call needs no workspace
    Pp = unbound.padded_params()
    for step, b in enumerate((b_first, b_second)):
        assert unbound.workspace_bytes(max(1, sum(b)), len(b)) <= binding.static_scratch_bytes()
        x, y = synth.make_batch(spec, "normal", sum(b), 3, step)
        xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
        got = torch.full((len(b), Pp), float("nan"), device="cuda")
        binding.forward_backward_static(unbound, pd, xd, yd, b, got)
        torch.cuda.synchronize()
        ref = _reference(spec, pd, xd, yd, b)
        assert torch.isfinite(got).all(), (name, b)
        assert torch.equal(got, ref), (name, b, float((got - ref).abs().max()))


def test_static_scratch_rejects_what_does_not_fit(dynb):
    import torch
    spec = synth.mlp_spec([4096, 4096, 10], "bf16")     # the weight copies alone exceed the area
    model = binding.Model(spec)
    assert model.workspace_bytes(8, 2) > binding.static_scratch_bytes()
    pd = torch.zeros(model.padded_params(), device="cuda")
    xd = torch.zeros(8, 4096, device="cuda"); yd = torch.zeros(8, dtype=torch.int32, device="cuda")
    grads = torch.zeros(2, model.padded_params(), device="cuda")
    with pytest.raises(binding.DynbError) as e:
        binding.forward_backward_static(model, pd, xd, yd, [5, 3], grads)
    assert e.value.code == -2 and "static" in str(e.value)

"""Shared plumbing of the GPU parity tests: device buffers (torch), the calls of one
training step through the C interface, and the error metric."""
import numpy as np

from paper_2305_12213_amd import binding, synth


def relerr(got, ref):
    """max|got - ref| / max|ref| (max-abs-normalised error of one tensor)."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    scale = np.max(np.abs(ref)) if ref.size else 0.0
    err = np.max(np.abs(got - ref)) if ref.size else 0.0
    return err / scale if scale > 0 else err


def worst_relerr(flat_got, spec, ref_params):
    """Largest per-tensor relerr between a flat device vector and [(W, b)] reference."""
    got = synth.unflatten_params(spec, np.asarray(flat_got))
    worst = 0.0
    for (gW, gb), (rW, rb) in zip(got, ref_params):
        worst = max(worst, relerr(gW, rW))
        if np.max(np.abs(rb)) > 0:
            worst = max(worst, relerr(gb, rb))
        else:
            assert np.max(np.abs(gb)) < 1e-30
    return worst


def worker_grads_as_lists(spec, g_host, P):
    """Rows of the device gradient matrix [K][P_pad] as per-worker [(dW, db)] lists."""
    return [synth.unflatten_params(spec, g_host[k, :P]) for k in range(g_host.shape[0])]


def worst_pair_relerr(got_list, ref_list):
    worst = 0.0
    for (gW, gb), (rW, rb) in zip(got_list, ref_list):
        worst = max(worst, relerr(gW, rW))
        if np.max(np.abs(rb)) > 0:
            worst = max(worst, relerr(gb, rb))
        else:
            assert np.max(np.abs(gb)) < 1e-30
    return worst


class DeviceRun:
    def __init__(self, spec, params_list, max_batch, max_workers):
        import torch
        self.torch = torch
        self.spec = spec
        self.model = binding.Model(spec)
        self.P = self.model.num_params()
        self.Pp = self.model.padded_params()
        self.params = torch.from_numpy(synth.flatten_params(params_list, 256)).cuda()
        assert self.params.numel() == self.Pp
        nbytes = self.model.workspace_bytes(max_batch, max_workers)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.model.bind(self.params, self.ws, nbytes, max_batch, max_workers)
        self.grads = torch.full((max_workers, self.Pp), float("nan"), device="cuda")
        self.out = torch.full((self.Pp,), float("nan"), device="cuda")
        self.velocity = None

    def set_params(self, params_list):
        self.params.copy_(self.torch.from_numpy(synth.flatten_params(params_list, 256)))
        self.model.sync_weights()

    def forward_backward(self, x, y, b):
        t = self.torch
        xd = t.from_numpy(np.ascontiguousarray(x, np.float32)).cuda() if isinstance(x, np.ndarray) else x
        yd = t.from_numpy(np.ascontiguousarray(y, np.int32)).cuda() if isinstance(y, np.ndarray) else y
        binding.forward_backward(self.model, xd, yd, b, self.grads)
        t.cuda.synchronize()
        return self.grads[:len(b)]

    def forward_backward_aggregate(self, x, y, b):
        """Gradients and their weighted aggregate (self.out) from one call."""
        t = self.torch
        xd = t.from_numpy(np.ascontiguousarray(x, np.float32)).cuda() if isinstance(x, np.ndarray) else x
        yd = t.from_numpy(np.ascontiguousarray(y, np.int32)).cuda() if isinstance(y, np.ndarray) else y
        binding.forward_backward_aggregate(self.model, xd, yd, b, self.grads, self.out)
        t.cuda.synchronize()
        return self.grads[:len(b)]

    def aggregate(self, b):
        binding.weighted_aggregate(self.grads, b, self.Pp, self.out)
        return self.out

    def set_velocity(self, vel_list):
        v = self.torch.from_numpy(synth.flatten_params(vel_list, 256)).cuda()
        if self.velocity is None:
            self.velocity = v
        else:
            self.velocity.copy_(v)

    def update(self, lr, mu=0.0):
        if mu:
            if self.velocity is None:
                self.velocity = self.torch.zeros(self.Pp, device="cuda")
            binding.model_sgd_update(self.model, self.out, lr, mu, self.velocity)
        else:
            binding.model_sgd_update(self.model, self.out, lr)

    def losses(self, K):
        return binding.read_worker_loss(self.model, K)

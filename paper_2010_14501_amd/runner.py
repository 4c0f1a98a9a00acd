"""Device-memory plumbing around a Plan: PyTorch owns the buffers and the stream, nothing else.

No arithmetic happens here; `StepRunner.step()` is one call into libmonet.so.
"""
import numpy as np
import torch

from . import monet


class StepRunner:
    def __init__(self, graph_text, schedule_text, exts, params, device="cuda:0", poison=False):
        """exts / params: {ref or pid: numpy array} in storage convention (N,H,W,C / K,R,S,C)."""
        if not torch.cuda.is_available():
            raise RuntimeError("StepRunner needs a GPU: the training step only exists as HIP kernels")
        self.plan = monet.Plan(graph_text, schedule_text)
        self.device = torch.device(device)
        self.inputs = [torch.from_numpy(np.ascontiguousarray(exts[-i])).to(self.device) for i in range(self.plan.num_inputs)]
        self.weights = [torch.from_numpy(np.ascontiguousarray(params[p])).to(self.device) for p in range(self.plan.num_params)]
        self.grads = [torch.zeros_like(w) for w in self.weights]
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.arena = torch.empty(self.plan.arena_bytes + 256, dtype=torch.uint8, device=self.device)
        base = self.arena.data_ptr()
        self.base = (base + 255) // 256 * 256
        self.plan.bind_arena(self.base, self.plan.arena_bytes)
        if poison:
            self.plan.set_poison(True)
        self._in_ptrs = [t.data_ptr() for t in self.inputs]
        self._w_ptrs = [t.data_ptr() for t in self.weights]
        self._g_ptrs = [t.data_ptr() for t in self.grads]

    def step(self, stream=None):
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        return self.plan.step(s.cuda_stream, self._in_ptrs, self._w_ptrs, self._g_ptrs, self.loss.data_ptr())

    def read(self, offset, shape, dtype=torch.float32):
        """Copy `shape` elements at byte `offset` of the bound memory to the host."""
        n = int(np.prod(shape))
        off = self.base - self.arena.data_ptr() + offset
        raw = self.arena[off:off + n * torch.empty((), dtype=dtype).element_size()]
        return raw.view(dtype).reshape(shape).cpu().numpy()

    def grads_numpy(self):
        torch.cuda.synchronize(self.device)
        return {p: g.cpu().numpy() for p, g in enumerate(self.grads)}

    def loss_value(self):
        torch.cuda.synchronize(self.device)
        return float(self.loss.item())

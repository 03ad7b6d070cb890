"""Device memory of one tensor list (allocated through PyTorch) bound to the HIP
optimizer.  Plumbing only: allocation, pointer lists, host copies."""
from __future__ import annotations

import numpy as np

from . import binding as B


def bf16_bits(t) -> np.ndarray:
    """torch.bfloat16 tensor (any device) -> numpy uint16 bit patterns on the host."""
    import torch
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def grad_to_host(t) -> np.ndarray:
    """Gradient tensor -> host array with the same bits (float32, or uint16 for bf16)."""
    import torch
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    return t.detach().cpu().numpy()


class DeviceState:
    """params / exp_avg / grads (one flat tensor each per spec) and v on one GPU,
    with an AdamMini optimizer bound to them.  m and v start at zero."""

    def __init__(self, specs, grad_dtype: str, device: int = 0, arena: bool = False):
        """arena=True: params, exp_avg and grads are each ONE allocation holding every tensor back to back
        (each tensor starting on a 4 KiB boundary), the way frameworks that keep flat parameter and state
        buffers lay them out; otherwise one allocation per tensor."""
        import torch
        self.specs = list(specs)
        self.grad_dtype = grad_dtype
        self.dev = torch.device("cuda:%d" % device)
        self.opt = B.AdamMini(self.specs, grad_dtype, device)
        gdt = torch.bfloat16 if grad_dtype == "bf16" else torch.float32
        if arena:
            def carve(dtype, zero):
                per = 4096 // torch.empty(0, dtype=dtype).element_size()
                starts, total = [], 0
                for s in self.specs:
                    starts.append(total)
                    total += (s.numel + per - 1) // per * per
                buf = (torch.zeros if zero else torch.empty)(total, dtype=dtype, device=self.dev)
                return buf, [buf[a:a + s.numel] for a, s in zip(starts, self.specs)]
            self._arenas = []
            for name, dtype, zero in (("p", torch.float32, False), ("m", torch.float32, True), ("g", gdt, True)):
                buf, views = carve(dtype, zero)
                self._arenas.append(buf)
                setattr(self, name, views)
        else:
            self.p = [torch.empty(s.numel, dtype=torch.float32, device=self.dev) for s in self.specs]
            self.m = [torch.zeros(s.numel, dtype=torch.float32, device=self.dev) for s in self.specs]
            self.g = [torch.zeros(s.numel, dtype=gdt, device=self.dev) for s in self.specs]
        self.v = torch.zeros(self.opt.num_blocks, dtype=torch.float32, device=self.dev)
        self.opt.bind(self.p, self.g, self.m, self.v)

    def close(self) -> None:
        self.opt.close()

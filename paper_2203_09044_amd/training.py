"""Algorithm 1 of the paper around a PyTorch model, all users on one GPU.

Each user computes the gradient of the shared model on its own mini-batch (torch autograd: the
caller's business); the gradients of all users are laid out as one [U][n] batch, one tensor of
the model per segment; the codec's calls do the rest of the iteration -- error correction, fp
conversion, compression on the user side, decompression and averaging on the parameter-server
side -- and the model takes the SGD step with the averaged reconstruction.  Plumbing only: no
arithmetic of the codec happens here.
"""
from __future__ import annotations

from typing import Callable, Iterable, Optional, Sequence, Tuple

import torch

from .binding import Fmt
from .pipeline import Co3Pipeline


class Co3SGD:
    def __init__(self, model: torch.nn.Module, users: int, fmt: Fmt, lr: float, gamma: float = 1.0,
                 chunk_syms: int = 256, bias: str = "absmax", codes: str = "user", code_group_min: int = 16384):
        self.model = model
        self.params = [p for p in model.parameters() if p.requires_grad]
        if not self.params:
            raise ValueError("the model has no trainable parameter")
        dev = self.params[0].device
        if dev.type != "cuda":
            raise ValueError("the codec runs on the GPU: move the model there first")
        self.sizes = [p.numel() for p in self.params]
        self.seg_off = [0]
        for s in self.sizes:
            self.seg_off.append(self.seg_off[-1] + s)
        self.n = self.seg_off[-1]
        self.U, self.lr = users, lr
        code_seg_off = None
        if codes == "layer":
            # tensors too small to pay for a table share the code of the large tensor before them
            groups, pending = [], 0
            for s in self.sizes:
                if s >= code_group_min:
                    groups.append(s + pending)
                    pending = 0
                elif groups:
                    groups[-1] += s
                else:
                    pending += s
            if pending:
                groups.append(pending)
            code_seg_off = [0]
            for gsz in groups:
                code_seg_off.append(code_seg_off[-1] + gsz)
        self.pipe = Co3Pipeline(users, self.n, fmt, chunk_syms=chunk_syms, seg_off=self.seg_off, gamma=gamma,
                                device=dev, bias=bias, codes=codes, code_seg_off=code_seg_off)
        self.g = self.pipe.new_gradient_buffer()

    def local_gradients(self, batches: Sequence[Tuple[torch.Tensor, torch.Tensor]],
                        loss_fn: Callable[[torch.Tensor, torch.Tensor], torch.Tensor]) -> float:
        """Fills row u of the gradient batch with user u's gradient; returns the mean loss."""
        if len(batches) != self.U:
            raise ValueError(f"expected {self.U} user batches")
        total = 0.0
        for u, (x, y) in enumerate(batches):
            self.model.zero_grad(set_to_none=True)
            loss = loss_fn(self.model(x), y)
            loss.backward()
            total += float(loss.detach())
            row = self.g[u]
            for p, a, b in zip(self.params, self.seg_off[:-1], self.seg_off[1:]):
                row[a:b].copy_(p.grad.reshape(-1))
        return total / self.U

    def apply_average(self, avg: Optional[torch.Tensor] = None):
        """Parameter-server update with the averaged reconstruction (Algorithm 1, last step)."""
        avg = self.pipe.avg if avg is None else avg
        with torch.no_grad():
            for p, a, b in zip(self.params, self.seg_off[:-1], self.seg_off[1:]):
                p.add_(avg[a:b].view_as(p), alpha=-self.lr)

    def step(self, batches, loss_fn) -> float:
        loss = self.local_gradients(batches, loss_fn)
        self.pipe.step(self.g)
        self.apply_average()
        return loss

    def bits_per_element(self) -> float:
        return float(self.pipe.total_bits.sum().item()) / (self.U * self.n)

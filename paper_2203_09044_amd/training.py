"""Algorithm 1 of the paper around a PyTorch model, all users on one GPU.

Each user computes the gradient of the shared model on its own mini-batch (torch autograd: the
caller's business); the gradients of all users are laid out as one [U][n] batch, one tensor of
the model per segment; the codec's calls do the rest of the iteration -- error correction, fp
conversion, compression on the user side, decompression and averaging on the parameter-server
side -- and the model takes the SGD step with the averaged reconstruction.  Plumbing only: no
arithmetic of the codec happens here.

``tables="model"`` is the scheme as Sec. III states it: the bias rule's multiplier on a fixed grid,
one code per layer shared by the users and designed from the GenNorm law fitted to the layer's
corrected gradients (no symbol statistics), refreshed every ``refresh`` iterations; between
refreshes the user side runs in one pass (conversion and compression without a symbol array).
``tables="lagged"``: per-user Huffman codes from the previous iteration's symbol counts, which the
one-pass user side gathers on the way.
"""
from __future__ import annotations

from typing import Callable, Iterable, Optional, Sequence, Tuple

import torch

from . import binding as B
from .binding import Fmt
from .pipeline import Co3Pipeline


class Co3SGD:
    def __init__(self, model: torch.nn.Module, users: int, fmt: Fmt, lr: float, gamma: float = 1.0,
                 chunk_syms: int = 256, bias: str = "absmax", codes: str = "user", code_group_min: int = 16384,
                 tables: str = "empirical", refresh: int = 10):
        if tables not in ("empirical", "model", "lagged"):
            raise ValueError("tables must be 'empirical', 'model' or 'lagged'")
        if tables == "model" and (bias != "moments" or codes != "layer"):
            raise ValueError("model tables go with bias='moments' and codes='layer'")
        if tables == "lagged" and (bias != "absmax" or codes != "user"):
            raise ValueError("lagged tables go with bias='absmax' and codes='user'")
        self.tables, self.refresh, self.t = tables, max(1, refresh), 0
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
                                device=dev, bias=bias, codes=codes, code_seg_off=code_seg_off,
                                statistics=tables != "model", single_pass=tables != "empirical",
                                lagged_codes=tables == "lagged")
        self.g = self.pipe.new_gradient_buffer()
        if tables == "model":
            # the tensor that designs each group's table: the largest one of the group
            cso = self.pipe.code_seg_off.cpu().tolist()
            self.design_tensor = []
            for a, b in zip(cso[:-1], cso[1:]):
                members = [k for k in range(len(self.sizes)) if a <= self.seg_off[k] < b and self.sizes[k] > 0]
                self.design_tensor.append(max(members, key=lambda k: self.sizes[k]) if members else 0)

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

    def refresh_tables(self):
        """One table per code group from the law fitted to the group's largest tensor (mean over the users of
        the fitted shape and of the fitted scale times the multiplier, i.e. the law of what is rounded onto
        the grid); host computation of the model weights, code build on the device."""
        pipe = self.pipe
        fit = pipe.fit.cpu().numpy()                   # [U][nseg][2]: (shape, scale) of x = g + gamma * m
        c = pipe.scale.cpu().numpy()                   # [U][nseg]
        A = int(pipe.anchor[0, 0].item())              # the fixed grid of the bias rule
        rows = []
        for k in self.design_tensor:
            beta = float(fit[:, k, 0].mean())
            alpha = float((fit[:, k, 1] * c[:, k]).mean())
            rows.append(B.model_weights(A, pipe.fmt, min(max(beta, 0.2), 4.0), max(alpha, 1e-30)))
        pipe.build(torch.stack(rows).to(pipe.device))

    def step(self, batches, loss_fn) -> float:
        loss = self.local_gradients(batches, loss_fn)
        if self.tables == "model":
            self.pipe.fit_bias(self.g)
            if self.t % self.refresh == 0:
                self.refresh_tables()
            self.pipe.convert_encode(self.g)
            self.pipe.aggregate()
        else:
            self.pipe.step(self.g)
        self.t += 1
        self.apply_average()
        return loss

    def bits_per_element(self) -> float:
        return float(self.pipe.total_bits.sum().item()) / (self.U * self.n)

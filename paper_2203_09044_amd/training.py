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

from co3_inputs import group_small_tensors, seg_offsets

from . import binding as B
from .binding import Fmt
from .pipeline import Co3Pipeline


class Co3SGD:
    def __init__(self, model: torch.nn.Module, users: int, fmt: Fmt, lr: float, gamma: float = 1.0,
                 chunk_syms: int = 256, bias: str = "absmax", codes: str = "user", code_group_min: int = 16384,
                 tables: str = "empirical", refresh: int = 10, cap_words: Optional[int] = None):
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
            code_seg_off = [int(x) for x in seg_offsets(group_small_tensors(self.sizes, code_group_min))]
        self.pipe = Co3Pipeline(users, self.n, fmt, chunk_syms=chunk_syms, seg_off=self.seg_off, gamma=gamma,
                                device=dev, bias=bias, codes=codes, code_seg_off=code_seg_off,
                                statistics=tables != "model", single_pass=tables != "empirical",
                                lagged_codes=tables == "lagged", cap_words=cap_words)
        self.g = self.pipe.new_gradient_buffer()
        # Views of every user's row of the gradient batch, shaped like the parameters: during a user's backward
        # pass they are the parameters' .grad, so autograd accumulates straight into the batch.
        self.grad_views = [[self.g[u, a:b].view_as(p) for p, a, b in zip(self.params, self.seg_off[:-1], self.seg_off[1:])]
                           for u in range(users)]
        # The one-pass user side overwrites the memory while it compresses; a stream that then does not fit its
        # buffer (possible with codes that are not the user's own counts) must be made again from the memory
        # as it was: those modes keep a copy of it per iteration.
        self.err_before = torch.empty_like(self.pipe.err) if self.pipe.single_pass else None
        self.codes_before = torch.empty_like(self.pipe.codes) if self.pipe.single_pass else None
        self.capacity_growths = 0

    def local_gradients(self, batches: Sequence[Tuple[torch.Tensor, torch.Tensor]],
                        loss_fn: Callable[[torch.Tensor, torch.Tensor], torch.Tensor]) -> float:
        """Fills row u of the gradient batch with user u's gradient; returns the mean loss."""
        if len(batches) != self.U:
            raise ValueError(f"expected {self.U} user batches")
        total = 0.0
        for u, (x, y) in enumerate(batches):
            self.g[u].zero_()
            for p, v in zip(self.params, self.grad_views[u]):
                p.grad = v
            loss = loss_fn(self.model(x), y)
            loss.backward()
            total += float(loss.detach())
            for p, v in zip(self.params, self.grad_views[u]):
                if p.grad is None or p.grad.data_ptr() != v.data_ptr():      # autograd replaced the tensor: copy it in
                    v.copy_(p.grad if p.grad is not None else torch.zeros_like(v))
        for p in self.params:
            p.grad = None
        return total / self.U

    def apply_average(self, avg: Optional[torch.Tensor] = None):
        """Parameter-server update with the averaged reconstruction (Algorithm 1, last step)."""
        avg = self.pipe.avg if avg is None else avg
        with torch.no_grad():
            for p, a, b in zip(self.params, self.seg_off[:-1], self.seg_off[1:]):
                p.add_(avg[a:b].view_as(p), alpha=-self.lr)

    def refresh_tables(self):
        """One table per code group from the law fitted to the group's largest tensor, pooled over the users
        (co3_design_layer_tables: host computation of the model weights), code build on the device."""
        pipe = self.pipe
        A = int(pipe.anchor[0, 0].item())              # the fixed grid of the bias rule
        weights = B.design_layer_tables(pipe.fit, pipe.scale, self.seg_off, pipe.code_seg_off.cpu().tolist(), A, pipe.fmt)
        pipe.build(weights.to(pipe.device))

    def _codec(self):
        if self.tables == "model":
            self.pipe.fit_bias(self.g)
            if self.t % self.refresh == 0:
                self.refresh_tables()
            self.pipe.convert_encode(self.g)
            self.pipe.aggregate()
        else:
            self.pipe.step(self.g)

    def step(self, batches, loss_fn) -> float:
        """One iteration of Algorithm 1.  The device status is read before the average reaches the model (one
        synchronisation per iteration).  A stream that did not fit its buffer (possible with codes that are
        not built from the user's own counts of the iteration) is made again in a larger one: from the symbols
        where the path keeps them, else from the saved memory and codes.  Any other condition raises Co3Error."""
        loss = self.local_gradients(batches, loss_fn)
        pipe = self.pipe
        if self.err_before is not None:
            self.err_before.copy_(pipe.err)
            self.codes_before.copy_(pipe.codes)
            had_codes = pipe.have_codes
        self._codec()
        for attempt in range(4):
            st = pipe.poll()
            if st == B.OK:
                break
            # total_bits holds what every stream needs, also after an overrun (the server's decoder then met a
            # truncated stream and may have reported that on top: the status word keeps the lowest code)
            need = (int(pipe.total_bits.max().item()) + 63) // 64
            if need <= pipe.cap_words or attempt == 3:
                raise B.Co3Error(st, "Co3SGD.step")
            pipe.grow_capacity(need)
            pipe.status.zero_()
            self.capacity_growths += 1
            if self.err_before is not None:
                pipe.err.copy_(self.err_before)
                pipe.codes.copy_(self.codes_before)
                pipe.have_codes = had_codes
                self._codec()
            else:                       # the symbols and the codes of this iteration are still there
                pipe.encode()
                pipe.aggregate()
        self.t += 1
        self.apply_average()
        return loss

    def bits_per_element(self) -> float:
        return float(self.pipe.total_bits.sum().item()) / (self.U * self.n)

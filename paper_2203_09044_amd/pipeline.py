"""Device buffers of one workload and the call sequence of one CO3 iteration.

Plumbing only: allocation through torch, then the six library calls in the order of
Algorithm 1 (user side: convert_ef [+ fused histogram] -> build_code -> encode; server
side: ps_aggregate, or decode for the round-trip check).  With ``bias="moments"`` the grid is
fixed (anchor ``grid_anchor``) and the paper's bias rule supplies a multiplier per (user,
tensor): moments -> bias_scale -> convert_ef_scaled ... ps_aggregate_scaled.  With
``codes="layer"`` there is one code per tensor shared by all users (built from the pooled
per-tensor counts of the iteration, or once from model weights handed to ``build``).
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B
from .binding import Fmt


def _round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


class Co3Pipeline:
    def __init__(self, U: int, n: int, fmt: Fmt, chunk_syms: int = 256, seg_off=None, gamma: float = 1.0,
                 cap_words: Optional[int] = None, device="cuda:0", fused_histogram: bool = True,
                 bias: str = "absmax", grid_anchor: Optional[int] = None, codes: str = "user", code_seg_off=None,
                 statistics: bool = True, single_pass: bool = False, lagged_codes: bool = False,
                 one_call: bool = False, keep_symbols: bool = True):
        if bias not in ("absmax", "moments"):
            raise ValueError("bias must be 'absmax' or 'moments'")
        if codes not in ("user", "layer"):
            raise ValueError("codes must be 'user' or 'layer'")
        self.code_mode = codes
        self.U, self.n, self.fmt, self.chunk_syms, self.gamma = U, n, fmt, chunk_syms, gamma
        self.fused_histogram = fused_histogram
        self.statistics = statistics      # False: fixed tables (designed from a model), no symbol counts are gathered
        # fixed tables only: conversion and compression in one pass, no symbol array (co3_convert_encode[_layers])
        self.single_pass = single_pass
        if single_pass and codes == "user" and bias != "absmax":
            raise ValueError("single_pass with the bias rule needs codes='layer'")
        # per-user empirical codes that follow the gradients one iteration behind: the one-pass user side also
        # counts the symbols (+1 each), and the codes of the next iteration are built from those counts
        self.lagged_codes = lagged_codes
        if lagged_codes and not single_pass:
            raise ValueError("lagged_codes needs single_pass")
        # the user's steps of an iteration through co3_user_encode (anchor from max|g|, one empirical code per user)
        self.one_call = one_call
        if one_call and (bias != "absmax" or codes != "user" or single_pass):
            raise ValueError("one_call is the path with the anchor from max|g| and per-user empirical codes")
        self.keep_symbols = keep_symbols  # one_call only: whether the symbol array is asked for
        self.have_codes = False
        self.bias = bias
        dev = torch.device(device)
        self.device = dev
        self.stride = _round_up(max(n, 1), 16)
        self.nchunks = (n + chunk_syms - 1) // chunk_syms
        # a user's own empirical code never exceeds the fixed-length size; a shared, model or lagged code can
        if cap_words is None:
            cap_words = B.cap_words_empirical(n, fmt) * (2 if codes == "layer" or single_pass else 1)
        self.cap_words = _round_up(cap_words, 2)
        self.seg_off = None if seg_off is None else torch.as_tensor(seg_off, dtype=torch.int64).to(dev)
        self.nseg = 1 if seg_off is None else self.seg_off.numel() - 1
        z = dict(device=dev)
        self.err = torch.zeros((U, self.stride), dtype=torch.float32, **z)
        self.sym = torch.zeros((U, self.stride), dtype=torch.uint8, **z)
        self.anchor = torch.zeros((U, self.nseg), dtype=torch.int32, **z)
        self.counts = torch.zeros((U, fmt.K), dtype=torch.int32, **z)
        self.codes = torch.zeros((U, B.CODE_BYTES), dtype=torch.uint8, **z)
        self.words = torch.zeros((U, max(self.cap_words, 2)), dtype=torch.int64, **z)
        self.chunk_bitoff = torch.zeros((U, self.nchunks + 1), dtype=torch.int64, **z)
        self.total_bits = torch.zeros((U,), dtype=torch.int64, **z)
        self.enc_ws = torch.zeros((max(B.encode_workspace_bytes(n, U), 8) // 8,), dtype=torch.int64, **z)
        self.agg_ws = torch.zeros((max(B.ps_aggregate_workspace_bytes(n, U, chunk_syms), 16),), dtype=torch.uint8, **z)
        self.fused_ws = (torch.empty((B.convert_encode_workspace_bytes(n, U, chunk_syms),), dtype=torch.uint8, **z)
                         if single_pass else None)
        self.user_ws = (torch.empty((max(B.user_encode_workspace_bytes(n, U, self.stride, self.nseg, keep_symbols), 256),), dtype=torch.uint8, **z)
                        if one_call else None)
        self.avg = torch.zeros((self.stride,), dtype=torch.float32, **z)
        self.sym_dec = torch.zeros((U, self.stride), dtype=torch.uint8, **z)
        self.status = torch.zeros((1,), dtype=torch.int32, **z)
        if codes == "layer":
            # boundaries of the shared codes: given, else those of the anchors, else one code for everything
            cso = code_seg_off if code_seg_off is not None else (seg_off if seg_off is not None else [0, n])
            self.code_seg_off = torch.as_tensor(cso, dtype=torch.int64).to(dev)
            self.ncodes = self.code_seg_off.numel() - 1
            self.layer_counts = torch.zeros((self.ncodes, fmt.K), dtype=torch.int32, **z)
            self.codes = torch.zeros((self.ncodes, B.CODE_BYTES), dtype=torch.uint8, **z)
        if bias == "moments":
            self.anchor.fill_((1 << (fmt.E - 1)) if grid_anchor is None else grid_anchor)
            self.sums = torch.zeros((U, self.nseg, 2), dtype=torch.float64, **z)
            self.fit = torch.zeros((U, self.nseg, 2), dtype=torch.float64, **z)
            self.scale = torch.ones((U, self.nseg), dtype=torch.float32, **z)

    def new_gradient_buffer(self) -> torch.Tensor:
        return torch.zeros((self.U, self.stride), dtype=torch.float32, device=self.device)

    # ---- user side
    def fit_bias(self, g: torch.Tensor):
        B.moments(g, self.err, self.n, self.gamma, self.sums, seg_off=self.seg_off)
        B.bias_scale(self.sums, self.n, self.U, self.scale, fit=self.fit, seg_off=self.seg_off)

    def convert(self, g: torch.Tensor, anchor_mode=B.ANCHOR_FROM_ABSMAX_G):
        counts = self.counts if self.statistics and self.fused_histogram and self.code_mode == "user" else None
        if self.bias == "moments":
            B.convert_ef_scaled(g, self.err, self.sym, self.n, self.anchor, self.scale, self.gamma, self.fmt,
                                seg_off=self.seg_off, counts=counts)
        else:
            B.convert_ef(g, self.err, self.sym, self.n, self.anchor, anchor_mode, self.gamma, self.fmt,
                         seg_off=self.seg_off, counts=counts)
        if self.statistics and not self.fused_histogram and self.code_mode == "user":
            B.histogram(self.sym, self.n, self.fmt, self.counts)

    def convert_encode(self, g: torch.Tensor, anchor_mode=B.ANCHOR_FROM_ABSMAX_G):
        """Conversion and compression in one pass with the codes already in ``self.codes`` (single_pass)."""
        if self.code_mode == "layer":
            scaled = self.bias == "moments"
            B.convert_encode_layers(g, self.err, self.n, self.anchor, B.ANCHOR_GIVEN if scaled else anchor_mode, self.gamma,
                                    self.fmt, self.codes, self.code_seg_off, self.words, self.chunk_syms,
                                    self.chunk_bitoff, self.total_bits, self.fused_ws, self.status, seg_off=self.seg_off,
                                    scale=self.scale if scaled else None,
                                    counts=self.layer_counts if self.lagged_codes else None)
        else:
            B.convert_encode(g, self.err, self.n, self.anchor, anchor_mode, self.gamma, self.fmt, self.codes, self.words,
                             self.chunk_syms, self.chunk_bitoff, self.total_bits, self.fused_ws, self.status,
                             seg_off=self.seg_off, counts=self.counts if self.lagged_codes else None)

    def user_encode(self, g: torch.Tensor):
        """Conversion, statistics, code and compression of all users in one library call (one_call)."""
        B.user_encode(g, self.err, self.n, self.anchor, self.gamma, self.fmt, self.counts, self.codes, self.words,
                      self.chunk_syms, self.chunk_bitoff, self.total_bits, self.user_ws, self.status,
                      sym=self.sym if self.keep_symbols else None, seg_off=self.seg_off)

    def build(self, weights: Optional[torch.Tensor] = None):
        """Per-user codes from the users' counts (or given weights [U][K]); per-tensor codes from the pooled
        per-tensor counts of this iteration (or given weights [nseg][K], e.g. model weights)."""
        if self.code_mode == "layer":
            if weights is None:
                B.histogram_layers(self.sym, self.n, self.fmt, self.code_seg_off, self.layer_counts, pool_users=True)
                weights = self.layer_counts
            B.build_code(weights, self.ncodes, self.fmt, self.codes, self.status)
        else:
            B.build_code(self.counts if weights is None else weights, self.U, self.fmt, self.codes, self.status)

    def encode(self):
        if self.code_mode == "layer":
            B.encode_layers(self.sym, self.n, self.fmt, self.codes, self.code_seg_off, self.words, self.chunk_syms,
                            self.chunk_bitoff, self.total_bits, self.enc_ws, self.status)
        else:
            B.encode(self.sym, self.n, self.fmt, self.codes, self.words, self.chunk_syms, self.chunk_bitoff,
                     self.total_bits, self.enc_ws, self.status)

    # ---- server side
    def decode(self):
        if self.code_mode == "layer":
            B.decode_layers(self.words, self.chunk_bitoff, self.chunk_syms, self.codes, self.code_seg_off, self.fmt,
                            self.n, self.sym_dec, self.status)
        else:
            B.decode(self.words, self.chunk_bitoff, self.chunk_syms, self.codes, self.fmt, self.n, self.sym_dec,
                     self.status)

    def aggregate(self):
        if self.code_mode == "layer":
            B.ps_aggregate_layers(self.words, self.chunk_bitoff, self.chunk_syms, self.codes, self.code_seg_off,
                                  self.fmt, self.n, self.U, self.anchor, self.avg, self.agg_ws, self.status,
                                  seg_off=self.seg_off, scale=self.scale if self.bias == "moments" else None)
        elif self.bias == "moments":
            B.ps_aggregate_scaled(self.words, self.chunk_bitoff, self.chunk_syms, self.codes, self.fmt, self.n,
                                  self.U, self.anchor, self.scale, self.avg, self.agg_ws, self.status,
                                  seg_off=self.seg_off)
        else:
            B.ps_aggregate(self.words, self.chunk_bitoff, self.chunk_syms, self.codes, self.fmt, self.n, self.U,
                           self.anchor, self.avg, self.agg_ws, self.status, seg_off=self.seg_off)

    def step(self, g: torch.Tensor, weights: Optional[torch.Tensor] = None, rebuild: bool = True):
        """One whole iteration: users encode, the server decodes and averages.  ``rebuild=False`` keeps the
        codes of the previous call (fixed tables designed from a model)."""
        if self.lagged_codes:
            if not self.have_codes:          # first iteration: nothing is known yet, every symbol weighs the same
                rows = self.ncodes if self.code_mode == "layer" else self.U
                self.build(torch.ones((rows, self.fmt.K), dtype=torch.int32, device=self.device)
                           if weights is None else weights)
                self.have_codes = True
            if self.bias == "moments":
                self.fit_bias(g)
            self.convert_encode(g)
            self.aggregate()                 # the server decodes with the codes this iteration was coded with
            # ... and the counts of this iteration code the next one
            self.build(self.layer_counts if self.code_mode == "layer" else None)
            return
        if self.single_pass and not rebuild:
            if self.bias == "moments":
                self.fit_bias(g)
            self.convert_encode(g)
            self.aggregate()
            return
        if self.one_call and rebuild and weights is None:
            self.user_encode(g)
            self.aggregate()
            return
        if self.bias == "moments":
            self.fit_bias(g)
        self.convert(g)
        if rebuild:
            self.build(weights)
        self.encode()
        self.aggregate()

    def grow_capacity(self, need_words: int):
        """A larger stream buffer per user (at least ``need_words`` 64-bit words plus an eighth); the streams
        it held are not kept."""
        cap = _round_up(max(need_words + need_words // 8, self.cap_words + 2), 2)
        self.cap_words = cap
        self.words = torch.zeros((self.U, cap), dtype=torch.int64, device=self.device)

    def poll(self) -> int:
        return B.poll_status(self.status)

"""Sequencing of the library calls for a multi-level encoder (conv3x3x3 -> ReLU -> 2x2x2
max-pool per level) forward and backward.  Only call order and buffer ownership live here;
every arithmetic step is a call into libhch.so."""
from __future__ import annotations

import torch

from . import binding as B


def _aligned_bytes(nbytes, device):
    t = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=device)
    off = (-t.data_ptr()) % 256
    return t[off: off + int(nbytes)]


class Encoder:
    """channels = [c0, c1, ..., cL]: level l runs conv c_l -> c_{l+1}, ReLU, pool to level l+1.
    `levels` must hold L+1 levels.  All buffers are allocated once here."""

    def __init__(self, levels, channels, algo=B.HCH_ALGO_COLUMNS, device="cuda", fuse_pointwise=True,
                 two_streams=False, keep_columns=True):
        self.levels, self.channels, self.algo = levels, list(channels), algo
        # columns algorithm: every level keeps the column matrix of its forward pass (1 GB in all
        # for the 256^3 x 8 workload) and the weight gradient reads it instead of gathering again
        self.keep_columns = keep_columns and algo == B.HCH_ALGO_COLUMNS
        self.fuse_pointwise = fuse_pointwise       # ReLU+pool (and their backward) as one call each
        # backward: the weight gradient of a level runs on a second stream (default priority)
        # beside the data gradient; both only read dY of that level
        self.two_streams = two_streams
        self.L = len(channels) - 1
        assert levels.n_levels >= self.L + 1
        self.n = [levels.n(l) for l in range(self.L + 1)]
        f32 = dict(dtype=torch.float32, device=device)
        ch = self.channels
        self.X = [torch.empty((self.n[l], ch[l]), **f32) for l in range(self.L + 1)]    # level inputs
        self.Y = [torch.empty((self.n[l], ch[l + 1]), **f32) for l in range(self.L)]    # conv outputs
        # the rectified rows are kept only when ReLU and pooling run as separate calls: the
        # fused calls take the sign for the backward pass from Y
        self.A = [None if fuse_pointwise else torch.empty((self.n[l], ch[l + 1]), **f32)
                  for l in range(self.L)]
        self.sw = [torch.empty((self.n[l + 1], ch[l + 1]), dtype=torch.int32, device=device)
                   for l in range(self.L)]
        self.W = [torch.empty((27, ch[l], ch[l + 1]), **f32) for l in range(self.L)]
        self.dW = [torch.empty((27, ch[l], ch[l + 1]), **f32) for l in range(self.L)]
        self.dX = [torch.empty((self.n[l], ch[l]), **f32) for l in range(self.L + 1)]   # dX[L] = upstream
        self.dA = [None if fuse_pointwise else torch.empty((self.n[l], ch[l + 1]), **f32)
                   for l in range(self.L)]
        self.dY = [torch.empty((self.n[l], ch[l + 1]), **f32) for l in range(self.L)]
        need = 256
        for l in range(self.L):
            for kind in (B.HCH_WS_FWD, B.HCH_WS_BWD_DATA, B.HCH_WS_BWD_WEIGHT):
                need = max(need, B.hch_conv_workspace_bytes(levels, l, ch[l], ch[l + 1], B.HCH_F32, kind, algo))
        self.ws = _aligned_bytes(need, device)
        self.ws_col = None
        if self.keep_columns:
            self.ws_col = [_aligned_bytes(max(B.hch_conv_workspace_bytes(levels, l, ch[l], ch[l + 1], B.HCH_F32, k, algo)
                                              for k in (B.HCH_WS_FWD, B.HCH_WS_BWD_WEIGHT)), device)
                           for l in range(self.L)]
        if two_streams:
            need_w = max(B.hch_conv_workspace_bytes(levels, l, ch[l], ch[l + 1], B.HCH_F32, B.HCH_WS_BWD_WEIGHT, algo)
                         for l in range(self.L))
            self.ws_side = _aligned_bytes(max(256, need_w), device)
            self.side = torch.cuda.Stream(device=device)
            self.ready = [torch.cuda.Event() for _ in range(self.L)]
            self.begin, self.coarse_ready = torch.cuda.Event(), torch.cuda.Event()

    def flops_per_step(self):
        """paper-method count: forward, data-gradient and weight-gradient products, each
        2 * 27 * c_in * c_out * N_l."""
        return sum(3 * 2 * 27 * self.channels[l] * self.channels[l + 1] * self.n[l] for l in range(self.L))

    def build_indices(self):
        if not self.two_streams:
            B.hch_build_neighbours(self.levels, -1)
            return
        # the finest level's lists on the main stream, the coarser levels' beside it; the main
        # stream picks them up before the first pooling (forward)
        main = torch.cuda.current_stream()
        self.begin.record(main)
        self.side.wait_event(self.begin)          # the side stream's previous work is in order anyway
        B.hch_build_neighbours_range(self.levels, 0, 1)
        B.hch_build_neighbours_range(self.levels, 1, self.levels.n_levels - 1, stream=self.side.cuda_stream)
        self.coarse_ready.record(self.side)

    def forward(self):
        ch = self.channels
        for l in range(self.L):
            B.hch_conv_fwd(self.levels, l, B.HCH_F32, self.X[l], self.W[l], self.Y[l], ch[l], ch[l + 1],
                           self.ws_col[l] if self.keep_columns else self.ws, self.algo)
            if l == 0 and self.two_streams:
                torch.cuda.current_stream().wait_event(self.coarse_ready)
            if self.fuse_pointwise:
                B.hch_relu_pool_fwd(self.levels, l, self.Y[l], None, self.X[l + 1], self.sw[l], ch[l + 1])
            else:
                B.hch_relu_fwd(self.Y[l], self.A[l], self.A[l].numel())
                B.hch_pool_fwd(self.levels, l, self.A[l], self.X[l + 1], self.sw[l], ch[l + 1])

    def backward(self):
        ch = self.channels
        main = torch.cuda.current_stream()
        for l in reversed(range(self.L)):
            if self.fuse_pointwise:
                B.hch_pool_relu_bwd_pooled(self.levels, l, self.dX[l + 1], self.sw[l], self.X[l + 1], self.dY[l], ch[l + 1])
            else:
                B.hch_pool_bwd(self.levels, l, self.dX[l + 1], self.sw[l], self.dA[l], ch[l + 1])
                B.hch_relu_bwd(self.A[l], self.dA[l], self.dY[l], self.dY[l].numel())
            walgo = B.HCH_ALGO_COLUMNS_RESIDENT if self.keep_columns else self.algo
            if self.two_streams:
                self.ready[l].record(main)
                self.side.wait_event(self.ready[l])
                B.hch_conv_bwd_weight(self.levels, l, B.HCH_F32, self.X[l], self.dY[l], self.dW[l], ch[l], ch[l + 1],
                                      self.ws_col[l] if self.keep_columns else self.ws_side, walgo,
                                      stream=self.side.cuda_stream)
            else:
                B.hch_conv_bwd_weight(self.levels, l, B.HCH_F32, self.X[l], self.dY[l], self.dW[l], ch[l], ch[l + 1],
                                      self.ws_col[l] if self.keep_columns else self.ws, walgo)
            B.hch_conv_bwd_data(self.levels, l, B.HCH_F32, self.dY[l], self.W[l], self.dX[l], ch[l], ch[l + 1], self.ws,
                                self.algo)
        if self.two_streams:
            main.wait_stream(self.side)     # the next pass overwrites what the side stream reads

    def step(self):
        """One pass of the whole hot path: index lists by hash lookup, forward, backward."""
        self.build_indices()
        self.forward()
        self.backward()

"""Sequencing helper: an L-layer GCN training step as a fixed series of C-ABI calls on
preallocated device buffers.  No arithmetic happens here."""
from __future__ import annotations

import torch

from . import binding as B


def padded_rows(n: int, f: int, dtype, device):
    """n x f tensor whose row pitch is an odd number of 128-byte lines.  With a power-of-two
    pitch the same column slice of every row falls on a few L2 channels only; an odd pitch
    spreads it over all of them (measured: 3.9 -> 3.1 ms for the 256-column aggregation)."""
    esize = torch.empty(0, dtype=dtype).element_size()
    if f * esize <= 128:  # rows of at most one line are left packed (16-byte granules)
        per16 = 16 // esize
        ld = (f + per16 - 1) // per16 * per16
        return torch.empty(n, ld, device=device, dtype=dtype)[:, :f]
    lines = (f * esize + 127) // 128
    if lines % 2 == 0:
        lines += 1
    ld = lines * 128 // esize
    return torch.empty(n, ld, device=device, dtype=dtype)[:, :f]


class GCNStep:
    """Forward + loss + backward of an L-layer GCN (ReLU between layers, none after the last).

    Buffers: Z_l and H_{l+1} per layer are kept for the backward pass; dH buffers are shared
    by width.  dW_l are fp32 like W_l.  The input gradient is not computed (dX is not needed
    for training)."""

    def __init__(self, g: B.Graph, x, weights, labels, n_chunks: int = 1, pipe: B.Pipeline = None,
                 reorder: bool = True, bandwidth: int = None):
        self.g = g
        self.n = x.shape[0]
        self.x = x
        self.w = list(weights)
        self.labels = labels
        self.n_chunks = n_chunks
        # bandwidth of the graph as numbered: the layers then run as one cross-layer pipeline of
        # n_chunks batches instead of layer by layer
        self.bandwidth = bandwidth
        self.pipe = pipe if pipe is not None else B.Pipeline()
        dev = x.device
        L = len(self.w)
        # a layer that narrows is updated first (Eq. 3 is associative): its aggregation then
        # runs at the output width
        self.order = [B.UPDATE_FIRST if (reorder and w.shape[1] < w.shape[0]) else B.AGG_FIRST
                      for w in self.w]
        def rows(f):
            return padded_rows(self.n, f, x.dtype, dev)

        x_p = rows(x.shape[1])
        x_p.copy_(x)
        self.x = x_p
        self.z = [rows(w.shape[1] if o == B.UPDATE_FIRST else w.shape[0])
                  for w, o in zip(self.w, self.order)]
        self.h = [x_p] + [rows(w.shape[1]) for w in self.w]
        # dW shares W's leading dimension (one ld_w in the layer descriptor)
        self.dw = [torch.empty_strided(w.shape, w.stride(), dtype=w.dtype, device=dev) for w in self.w]
        self.dlogits = rows(self.w[L - 1].shape[1])
        self.dh = [None] + [rows(self.w[l].shape[0]) for l in range(1, L)]
        self.loss = torch.zeros(1, dtype=torch.float64, device=dev)

    def forward(self, pipe=None):
        pipe = self.pipe if pipe is None else pipe
        L = len(self.w)
        if self.bandwidth is not None:
            B.forward_pipelined(self.g, self.h[0], self.w, self.z, self.h[1:], pipe, self.bandwidth,
                                self.n_chunks, orders=self.order)
            B.softmax_xent(self.h[L], self.labels, self.dlogits, self.loss, stream=pipe.primary)
            return
        for l in range(L):
            B.layer_fwd(self.g, self.h[l], self.w[l], self.z[l], self.h[l + 1], pipe,
                        relu=(l < L - 1), n_chunks=self.n_chunks, order=self.order[l])
        B.softmax_xent(self.h[L], self.labels, self.dlogits, self.loss, stream=pipe.primary)

    def backward(self, pipe=None):
        pipe = self.pipe if pipe is None else pipe
        L = len(self.w)
        if self.bandwidth is not None:
            B.backward_pipelined(self.g, self.h[0], self.z, self.h[1:], self.w,
                                 self.dh[1:] + [self.dlogits], self.dw, None, pipe, self.bandwidth,
                                 self.n_chunks, orders=self.order)
            return
        grad = self.dlogits
        for l in range(L - 1, -1, -1):
            B.layer_bwd(self.g, self.z[l], self.h[l + 1], self.w[l], grad, self.dw[l], self.dh[l],
                        pipe, relu=(l < L - 1), n_chunks=self.n_chunks, order=self.order[l],
                        H=self.h[l])
            grad = self.dh[l]

    def step(self):
        self.forward()
        self.backward()

    def capture(self):
        """Records one step (single-stream schedule) into a HIP graph; replay() then launches
        the whole step with one call, which matters when the graph is small and the step is
        bound by launch overhead.  One eager step runs first so that every scratch buffer has
        its final size (growing one allocates, which a capture cannot contain)."""
        assert self.n_chunks == 1, "the captured step uses one stream"
        self.step()
        torch.cuda.synchronize()
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph):
            cur = torch.cuda.current_stream()
            self._graph_pipe = B.Pipeline(primary=cur, secondary=cur)
            self.forward(self._graph_pipe)
            self.backward(self._graph_pipe)
        return self

    def replay(self):
        self._graph.replay()

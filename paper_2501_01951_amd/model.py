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
    if f * esize <= 128:
        # a row of at most one line gets a power-of-two pitch (16 .. 128 bytes), so that it never
        # straddles two lines: with 47 bf16 columns packed at 96 bytes a gathered row costs 1.5
        # line fetches on average (config 5's 47-column aggregation: 2.2 ms packed)
        pitch = 16
        while pitch < f * esize:
            pitch *= 2
        return torch.empty(n, pitch // esize, device=device, dtype=dtype)[:, :f]
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
        bound by launch overhead.  No warm-up step is needed: the library's work buffers exist
        once a pipeline has been created, and the aggregation scratch of the stream that the
        capture runs on is reserved here, before the capture starts."""
        assert self.n_chunks == 1, "the captured step uses one stream"
        B.graph_reserve_streams(self.g, 1)
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


class SAGEStep:
    """Forward + loss + backward of an L-layer GraphSAGE with the mean aggregator (the graph is
    normalised with NORM_MEAN, no self-loops).  Layer l keeps X_l = [H_l | mean of the neighbors'
    H_l] in ONE n x 2 d_l buffer: the aggregation reads its left half and writes its right half,
    the update of layer l - 1 writes H_l straight into the left half, and W_l (2 d_l x d_{l+1})
    multiplies the whole buffer.  Backward: dX_l = dP_l W_l^T into a buffer of the same shape,
    then the transposed aggregation ADDS A_hat^T of its right half onto its left half, which is
    the gradient with respect to H_l.  Widths must be multiples of 4 (fp32) / 8 (bf16)."""

    def __init__(self, g: B.Graph, x, weights, labels):
        self.g, self.n, self.labels = g, x.shape[0], labels
        self.w = list(weights)
        dev, dt = x.device, x.dtype
        L = len(self.w)
        self.dims = [x.shape[1]] + [w.shape[1] for w in self.w]
        vec = 16 // torch.empty(0, dtype=dt).element_size()
        for l, w in enumerate(self.w):
            assert self.dims[l] % vec == 0 and w.shape[0] == 2 * self.dims[l]
        self.xc = [padded_rows(self.n, 2 * self.dims[l], dt, dev) for l in range(L)]
        self.xc[0][:, :self.dims[0]].copy_(x)
        self.logits = padded_rows(self.n, self.dims[L], dt, dev)
        self.dlogits = padded_rows(self.n, self.dims[L], dt, dev)
        self.dxc = [None] + [padded_rows(self.n, 2 * self.dims[l], dt, dev) for l in range(1, L)]
        self.dw = [torch.empty_strided(w.shape, w.stride(), dtype=w.dtype, device=dev) for w in self.w]
        self.loss = torch.zeros(1, dtype=torch.float64, device=dev)

    def h(self, l):
        """H_l: the left half of X_l, or the logits."""
        return self.logits if l == len(self.w) else self.xc[l][:, :self.dims[l]]

    def forward(self):
        L = len(self.w)
        for l in range(L):
            d = self.dims[l]
            B.aggregate(self.g, self.xc[l][:, :d], self.xc[l][:, d:2 * d])
            B.update(B.OP_FWD_RELU if l < L - 1 else B.OP_FWD, self.xc[l], self.w[l], self.h(l + 1),
                     self.n, 2 * d, self.dims[l + 1])
        B.softmax_xent(self.logits, self.labels, self.dlogits, self.loss)

    def backward(self):
        L = len(self.w)
        grad = self.dlogits
        for l in range(L - 1, -1, -1):
            d = self.dims[l]
            ref = self.h(l + 1) if l < L - 1 else None
            B.update(B.OP_WGRAD, self.xc[l], grad, self.dw[l], self.n, 2 * d, self.dims[l + 1],
                     relu_ref=ref)
            if l == 0:
                break
            B.update(B.OP_DGRAD, grad, self.w[l], self.dxc[l], self.n, 2 * d, self.dims[l + 1],
                     relu_ref=ref)
            B.aggregate(self.g, self.dxc[l][:, d:2 * d], self.dxc[l][:, :d], transpose=True,
                        accumulate=True)
            grad = self.dxc[l][:, :d]

    def step(self):
        self.forward()
        self.backward()


class GINStep:
    """Forward + loss + backward of an L-layer GIN (the graph is normalised with NORM_SUM and
    has self-loops, whose value carries 1 + eps).  Layer l: Z_l = A_hat H_l, T_l = relu(Z_l W1_l),
    H_{l+1} = relu(T_l W2_l) (no ReLU after the last layer)."""

    def __init__(self, g: B.Graph, x, w1s, w2s, labels):
        self.g, self.n, self.labels = g, x.shape[0], labels
        self.w1, self.w2 = list(w1s), list(w2s)
        dev, dt = x.device, x.dtype
        L = len(self.w1)
        rows = lambda f: padded_rows(self.n, f, dt, dev)
        x_p = rows(x.shape[1])
        x_p.copy_(x)
        self.h = [x_p] + [rows(w.shape[1]) for w in self.w2]
        self.z = [rows(w.shape[0]) for w in self.w1]
        self.t = [rows(w.shape[1]) for w in self.w1]
        self.dt = [rows(w.shape[1]) for w in self.w1]
        self.dh = [None] + [rows(self.w1[l].shape[0]) for l in range(1, L)]
        self.dlogits = rows(self.w2[L - 1].shape[1])
        like = lambda w: torch.empty_strided(w.shape, w.stride(), dtype=w.dtype, device=dev)
        self.dw1 = [like(w) for w in self.w1]
        self.dw2 = [like(w) for w in self.w2]
        self.loss = torch.zeros(1, dtype=torch.float64, device=dev)

    def forward(self):
        L = len(self.w1)
        for l in range(L):
            k, hd, m = self.w1[l].shape[0], self.w1[l].shape[1], self.w2[l].shape[1]
            B.aggregate(self.g, self.h[l], self.z[l])
            B.update(B.OP_FWD_RELU, self.z[l], self.w1[l], self.t[l], self.n, k, hd)
            B.update(B.OP_FWD_RELU if l < L - 1 else B.OP_FWD, self.t[l], self.w2[l], self.h[l + 1],
                     self.n, hd, m)
        B.softmax_xent(self.h[L], self.labels, self.dlogits, self.loss)

    def backward(self):
        L = len(self.w1)
        grad = self.dlogits
        for l in range(L - 1, -1, -1):
            k, hd, m = self.w1[l].shape[0], self.w1[l].shape[1], self.w2[l].shape[1]
            ref = self.h[l + 1] if l < L - 1 else None
            B.update(B.OP_WGRAD, self.t[l], grad, self.dw2[l], self.n, hd, m, relu_ref=ref)
            B.update(B.OP_DGRAD, grad, self.w2[l], self.dt[l], self.n, hd, m, relu_ref=ref)
            B.update(B.OP_WGRAD, self.z[l], self.dt[l], self.dw1[l], self.n, k, hd, relu_ref=self.t[l])
            if l == 0:
                break
            # dZ_l over Z_l (the weight gradient above was its last reader), then A_hat^T
            B.update(B.OP_DGRAD, self.dt[l], self.w1[l], self.z[l], self.n, k, hd, relu_ref=self.t[l])
            B.aggregate(self.g, self.z[l], self.dh[l], transpose=True)
            grad = self.dh[l]

    def step(self):
        self.forward()
        self.backward()


class GCNDropoutStep:
    """GCNStep in the order of Algorithm 2 with the output mask of Eq. 4 on every aggregation
    (forward use of the S-SpMM): Z_l = (A_hat H_l) (.) M_l with M_l the dropout bitmap of seed
    `seed + l`, regenerated where the backward pass needs it instead of being kept.  Backward:
    dZ_l (.) M_l before the transposed aggregation."""

    def __init__(self, g: B.Graph, x, weights, labels, seed: int, keep: float):
        self.g, self.n, self.labels = g, x.shape[0], labels
        self.w = list(weights)
        self.seed, self.keep = seed, keep
        dev, dt = x.device, x.dtype
        L = len(self.w)
        rows = lambda f: padded_rows(self.n, f, dt, dev)
        x_p = rows(x.shape[1])
        x_p.copy_(x)
        self.h = [x_p] + [rows(w.shape[1]) for w in self.w]
        self.z = [rows(w.shape[0]) for w in self.w]
        self.dw = [torch.empty_strided(w.shape, w.stride(), dtype=w.dtype, device=dev) for w in self.w]
        self.dlogits = rows(self.w[L - 1].shape[1])
        self.dh = [None] + [rows(self.w[l].shape[0]) for l in range(1, L)]
        self.loss = torch.zeros(1, dtype=torch.float64, device=dev)

    def mask(self, l):
        return B.dropout_bitmap(self.seed + l, self.n, self.w[l].shape[0], self.keep)

    def forward(self):
        L = len(self.w)
        for l in range(L):
            k, m = self.w[l].shape
            B.aggregate_masked(self.g, self.h[l], self.z[l], self.mask(l))
            B.update(B.OP_FWD_RELU if l < L - 1 else B.OP_FWD, self.z[l], self.w[l], self.h[l + 1],
                     self.n, k, m)
        B.softmax_xent(self.h[L], self.labels, self.dlogits, self.loss)

    def backward(self):
        L = len(self.w)
        grad = self.dlogits
        for l in range(L - 1, -1, -1):
            k, m = self.w[l].shape
            ref = self.h[l + 1] if l < L - 1 else None
            B.update(B.OP_WGRAD, self.z[l], grad, self.dw[l], self.n, k, m, relu_ref=ref)
            if l == 0:
                break
            B.update(B.OP_DGRAD, grad, self.w[l], self.z[l], self.n, k, m, relu_ref=ref)
            B.apply_bitmap(self.z[l], self.mask(l))
            B.aggregate(self.g, self.z[l], self.dh[l], transpose=True)
            grad = self.dh[l]

    def step(self):
        self.forward()
        self.backward()

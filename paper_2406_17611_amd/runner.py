"""Harness that holds all partitions of a graph in one GPU's memory and drives the C ABI "in turn":
Algorithm 1's forward and backward for every layer and partition, with the inter-machine exchange
replaced by on-device buffers (the compressed rows an owner writes are read in place by its consumers).

Only sequencing and buffer bookkeeping live here; all arithmetic is in libvarco's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as vb


class PartitionedNetwork:
    def __init__(self, host_parts, widths, conv: str, mask_key: int, device="cuda", need_backward=True, dtype="f32",
                 n_streams=1, transform_first=()):
        """dtype: storage of activations, messages and their gradients ("f32" or "bf16"); weights and weight
        gradients are always fp32. n_streams > 1: the partitions of a layer are dealt to that many HIP
        streams, so that the matrix-core-bound kernels of one partition overlap the memory-bound kernels of
        another; streams are joined wherever a step needs all partitions (layer boundaries, owner-side sums).
        transform_first: layers whose calls apply the weights before the aggregation (varco_set_layer_order)."""
        assert dtype in ("f32", "bf16")
        assert 1 <= n_streams <= 4
        self.n_streams = self.max_streams = n_streams
        self.dtype = dtype
        self.act_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.device = torch.device(device)
        self.host_parts = host_parts
        self.P = len(host_parts)
        self.widths = list(widths)
        self.L = len(widths) - 1
        self.conv = conv
        act = [vb.ACT_RELU] * (self.L - 1) + [vb.ACT_IDENTITY]
        self.ctx = vb.Context(self.widths, act, vb.CONV_SAGE if conv == "sage" else vb.CONV_GCN, self.P, mask_key,
                              vb.BF16 if dtype == "bf16" else vb.F32)
        self.dev_parts = [self.ctx.register_partition(q, hp, self.device) for q, hp in enumerate(host_parts)]
        self.transform_first = frozenset(transform_first)
        for l in self.transform_first:
            self.ctx.set_layer_order(l, vb.ORDER_TRANSFORM_FIRST)

        self.n_local = [hp.n_local for hp in host_parts]
        self.n_halo = [hp.n_halo for hp in host_parts]
        self.row_off = np.concatenate(([0], np.cumsum(self.n_local))).astype(np.int64)
        self.halo_off = np.concatenate(([0], np.cumsum(self.n_halo))).astype(np.int64)
        self.n_total = int(self.row_off[-1])
        self.b_total = int(sum(hp.n_boundary for hp in host_parts))
        self.nnz_total = int(sum(hp.nnz for hp in host_parts))

        self.boundary_gid = [torch.from_numpy(hp.local_gid[hp.boundary_rows]).to(self.device) for hp in host_parts]

        # the backward exchange seen from the owners (built by varco_partition_build, uploaded at registration):
        # for each boundary row, the rows returned for it in the concatenation of all consumers' dz_halo buffers
        self.ret_ptr = [dp["ret_ptr"] for dp in self.dev_parts]
        self.ret_src = [dp["ret_src"] for dp in self.dev_parts]
        assert all(hp.halo_row_offset == off for hp, off in zip(host_parts, self.halo_off))

        f32 = dict(dtype=torch.float32, device=self.device)
        act = dict(dtype=self.act_dtype, device=self.device)
        self.x = [torch.empty((self.n_total, w), **act) for w in self.widths]
        self.m = [torch.empty((self.n_total, self.widths[l]), **act) for l in range(self.L)]
        self.h1 = [torch.empty((self.widths[l], self.widths[l + 1]), **f32) for l in range(self.L)]
        self.h0 = [torch.empty_like(h) if conv == "sage" else None for h in self.h1]
        self.z = [None] * self.L           # allocated per step (k changes with the ratio)
        self.need_backward = need_backward
        if need_backward:
            self.dh1 = [torch.zeros_like(h) for h in self.h1]
            self.dh0 = [torch.zeros_like(h) if conv == "sage" else None for h in self.h1]
            # one more set of weight-gradient accumulators per extra stream (overlapping calls must not
            # read-modify-write the same buffer); folded into dh1 / dh0 at the end of backward()
            self._dh1_extra = [[torch.zeros_like(h) for h in self.h1] for _ in range(n_streams - 1)]
            self._dh0_extra = [[torch.zeros_like(h) if conv == "sage" else None for h in self.h1]
                               for _ in range(n_streams - 1)]
            self.dx = [None] + [torch.empty((self.n_total, self.widths[l]), **act) for l in range(1, self.L + 1)]
            self.dz_halo = [None] * self.L
        self._zcap = [0] * self.L
        self._dzcap = [0] * self.L
        self._streams = None
        self._prepared = set()
        self._prepare([None])

    # ------------------------------------------------------------------ streams
    def _prepare(self, streams):
        """The library allocates per-stream workspaces in varco_prepare only; every stream is prepared once."""
        for st in streams:
            handle = vb._stream(st)
            if handle not in self._prepared:
                self.ctx.prepare(st)
                self._prepared.add(handle)

    def use_streams(self, n: int):
        """Issue the following steps on the first n of the network's streams (1 <= n <= n_streams)."""
        assert 1 <= n <= self.max_streams
        self.n_streams = n

    def _stream_set(self, stream):
        """The streams a step is issued on: the caller's (or torch's current) stream first, then the extra ones."""
        if self.n_streams == 1:
            return [stream]
        if self._streams is None:
            self._streams = [torch.cuda.Stream(device=self.device) for _ in range(self.max_streams - 1)]
        return [stream if stream is not None else torch.cuda.current_stream(self.device)] + self._streams[:self.n_streams - 1]

    @staticmethod
    def _join(streams):
        """Every stream waits for everything issued so far on all of them. Written as fork - join - fork from the
        first stream, so that under graph capture every event is recorded on a stream that is already part of the
        capture."""
        if len(streams) == 1:
            return
        main, others = streams[0], streams[1:]

        def fork():
            e = torch.cuda.Event()
            e.record(main)
            for st in others:
                st.wait_event(e)

        fork()
        for st in others:
            e = torch.cuda.Event()
            e.record(st)
            main.wait_event(e)
        fork()

    # ------------------------------------------------------------------ data placement
    def rows(self, q):
        return slice(int(self.row_off[q]), int(self.row_off[q + 1]))

    def set_inputs(self, x0_global: np.ndarray):
        """Scatter a global [n, F_0] feature matrix into the partition-ordered arena."""
        order = np.concatenate([hp.local_gid for hp in self.host_parts]).astype(np.int64)
        self.x[0].copy_(torch.from_numpy(np.ascontiguousarray(x0_global[order])).to(self.device))

    def set_weights(self, h1_list, h0_list=None):
        for l in range(self.L):
            self.h1[l].copy_(torch.from_numpy(h1_list[l]).to(self.device))
            if self.conv == "sage":
                self.h0[l].copy_(torch.from_numpy(h0_list[l]).to(self.device))

    def set_upstream(self, dx_global: np.ndarray):
        order = np.concatenate([hp.local_gid for hp in self.host_parts]).astype(np.int64)
        self.dx[self.L].copy_(torch.from_numpy(np.ascontiguousarray(dx_global[order])).to(self.device))

    def to_global(self, arena: torch.Tensor) -> np.ndarray:
        order = np.concatenate([hp.local_gid for hp in self.host_parts]).astype(np.int64)
        out = np.empty(tuple(arena.shape), dtype=np.float32)
        out[order] = arena.float().cpu().numpy()
        return out

    # ------------------------------------------------------------------ one step
    def _ensure_buffers(self):
        for l in range(self.L):
            k = self.ctx.keep(l)
            need = self.b_total * k
            if self.z[l] is None or self._zcap[l] < need:
                self.z[l] = torch.empty(max(need, 1), dtype=self.act_dtype, device=self.device)
                self._zcap[l] = need
            if self.need_backward and l > 0:
                need = int(self.halo_off[-1]) * k
                if self.dz_halo[l] is None or self._dzcap[l] < need:
                    self.dz_halo[l] = torch.empty(max(need, 1), dtype=self.act_dtype, device=self.device)
                    self._dzcap[l] = need

    def forward(self, step: int, ratio=None, stream=None):
        """Forward of all layers and partitions for training step `step`. `ratio` = (num, den) for every layer
        or a list of per-layer pairs: Algorithm 1 updates the rate at the step boundary."""
        ctx = self.ctx
        if step is None:
            ctx.advance_step(stream)        # the step lives on the device (graph replay): next step
        else:
            ctx.set_step(step, stream)
        if ratio is not None:
            if isinstance(ratio[0], (tuple, list)):
                for l, (num, den) in enumerate(ratio):
                    ctx.set_ratio(l, num, den)
            else:
                ctx.set_ratio(-1, ratio[0], ratio[1])
        self._ensure_buffers()
        streams = self._stream_set(stream)
        self._prepare(streams)
        ns = len(streams)
        self._join(streams)
        # layer 0's exchange: owners compress the boundary rows of the input features
        k0 = ctx.keep(0)
        for p, hp in enumerate(self.host_parts):
            if hp.n_boundary:
                zp = self.z[0][hp.z_row_offset * k0:]
                ctx.compress(0, self.boundary_gid[p], self.dev_parts[p]["boundary_rows"], hp.n_boundary,
                             self.x[0][self.rows(p)], self.widths[0], zp, streams[p % ns])
        for l in range(self.L):
            last = l == self.L - 1
            self._join(streams)         # every owner's compressed rows of this layer's input are complete
            for q in range(self.P):
                r = self.rows(q)
                ctx.layer_fwd(l, q, self.x[l][r], self.z[l], self.h1[l], self.h0[l], self.x[l + 1][r],
                              None if last else self.z[l + 1], self.m[l][r], streams[q % ns])
        self._join(streams)

    def backward(self, stream=None):
        ctx = self.ctx
        streams = self._stream_set(stream)
        self._prepare(streams)
        ns = len(streams)
        self._join(streams)
        for l in range(self.L - 1, -1, -1):
            need = l > 0
            k = ctx.keep(l)
            for q in range(self.P):
                r = self.rows(q)
                si = q % ns
                dzh = None
                if need and self.n_halo[q]:
                    dzh = self.dz_halo[l][int(self.halo_off[q]) * k:]
                dh1 = self.dh1[l] if si == 0 else self._dh1_extra[si - 1][l]
                dh0 = self.dh0[l] if si == 0 else self._dh0_extra[si - 1][l]
                # what the forward call saved: the aggregated rows, or (transform-first) the compressed rows it read
                saved = self.z[l] if l in self.transform_first else self.m[l][r]
                ctx.layer_bwd(l, q, self.dx[l + 1][r], self.x[l + 1][r], self.x[l][r], saved, self.h1[l],
                              self.h0[l], dh1, dh0, self.dx[l][r] if need else None, dzh, streams[si])
            self._join(streams)         # all consumers' returned rows and all local gradients of the layer exist
            if need:
                # errors handed back: every owner adds what its consumers returned, at the kept positions
                for p in range(self.P):
                    if self.host_parts[p].n_boundary:
                        ctx.accumulate_returned(l, p, self.ret_ptr[p], self.ret_src[p], self.dz_halo[l],
                                                self.dx[l][self.rows(p)], streams[p % ns])
                self._join(streams)
        # the partitions' weight gradients are summed (Algorithm 1): fold the per-stream accumulators
        if ns > 1:
            with torch.cuda.stream(streams[0]):
                for extra1, extra0 in zip(self._dh1_extra[:ns - 1], self._dh0_extra[:ns - 1]):
                    for l in range(self.L):
                        vb.sum_gradients(self.dh1[l], extra1[l], streams[0])
                        extra1[l].zero_()
                        if self.dh0[l] is not None:
                            vb.sum_gradients(self.dh0[l], extra0[l], streams[0])
                            extra0[l].zero_()

    # ------------------------------------------------------------------ training (Algorithm 1's iteration)
    def set_labels(self, labels_global: np.ndarray, train_mask: np.ndarray):
        """Class labels of all nodes and which of them are training nodes (the rest is held out)."""
        order = np.concatenate([hp.local_gid for hp in self.host_parts]).astype(np.int64)
        lab = np.asarray(labels_global, dtype=np.int32)[order]
        tr = np.asarray(train_mask, dtype=bool)[order]
        self.labels_train = torch.from_numpy(np.where(tr, lab, -1).astype(np.int32)).to(self.device)
        self.labels_test = torch.from_numpy(np.where(tr, -1, lab).astype(np.int32)).to(self.device)
        self.n_train, self.n_test = int(tr.sum()), int((~tr).sum())
        self._row_loss = torch.empty(self.n_total, dtype=torch.float32, device=self.device)
        self._row_correct = torch.empty(self.n_total, dtype=torch.int32, device=self.device)
        self._totals = torch.zeros(2, dtype=torch.float32, device=self.device)

    def loss(self, train: bool = True, with_gradient: bool = True, stream=None):
        """Cross-entropy of the last layer's output on the training (or held-out) nodes, partition by partition;
        with_gradient writes the upstream gradient of the backward pass. Returns the device tensor
        [risk, number of correct rows] (read it after synchronising)."""
        labels = self.labels_train if train else self.labels_test
        scale = 1.0 / max(1, self.n_train if train else self.n_test)
        c = self.widths[-1]
        self._totals.zero_()
        for q in range(self.P):
            r = self.rows(q)
            self.ctx.softmax_xent(self.x[self.L][r], labels[r], c, scale, self.dx[self.L][r] if with_gradient else None,
                                  self._row_loss[r], self._row_correct[r], self._totals, stream)
        return self._totals

    def sgd(self, lr: float, stream=None):
        for l in range(self.L):
            vb.sgd_step(self.h1[l], self.dh1[l], lr, stream)
            if self.h0[l] is not None:
                vb.sgd_step(self.h0[l], self.dh0[l], lr, stream)

    def train_step(self, step: int, ratio, lr: float, stream=None):
        """Forward with the compressed exchange, loss, backward, summed weight gradients, gradient step."""
        self.zero_grads()
        self.forward(step, ratio, stream)
        totals = self.loss(True, True, stream)
        self.backward(stream)
        self.sgd(lr, stream)
        return totals

    # ------------------------------------------------------------------ HIP graph of one step
    def capture_step(self, ratio):
        """Captures "advance to the next step, forward, backward" at a fixed ratio into a HIP graph and returns it
        (torch.cuda.CUDAGraph): every replay() is one more step, without per-launch host work. The step counter
        and the key words of the kept positions live on the device from here on (varco_step_table_enable); the
        ratio, i.e. every k, is frozen into the graph. Set the step the first replay should follow with
        ctx.set_step(step). Host-side exchange counters do not see replays."""
        side = torch.cuda.Stream(device=self.device)
        side.wait_stream(torch.cuda.current_stream(self.device))
        with torch.cuda.stream(side):
            self.ctx.step_table_enable()
            self.step(None, ratio)          # warm-up on the capture stream: its workspace set and all buffers exist
        torch.cuda.current_stream(self.device).wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            self.step(None, ratio)
        return graph

    def zero_grads(self):
        for l in range(self.L):
            self.dh1[l].zero_()
            if self.dh0[l] is not None:
                self.dh0[l].zero_()

    def step(self, step: int, ratio=None, stream=None):
        self.forward(step, ratio, stream)
        self.backward(stream)


class KTapNetwork(PartitionedNetwork):
    """General K-tap layers, X_l = rho( sum_{k<K} S^k X_{l-1} H_{l,k} ) (eq. (1)-(2)), driven through the library's
    building-block calls: every hop k = 1..K-1 has a compressed exchange of its own (tap address (layer, hop)),
    the transform is a sum of K dense products, and the backward pass walks the hops in reverse, handing the
    errors of halo rows back to their owners at every hop. Same buffers and bookkeeping as PartitionedNetwork."""

    def __init__(self, host_parts, widths, n_taps: int, mask_key: int, device="cuda", dtype="f32"):
        super().__init__(host_parts, widths, "sage", mask_key, device, True, dtype, 1)
        assert n_taps >= 1
        self.K = n_taps
        f32 = dict(dtype=torch.float32, device=self.device)
        act = dict(dtype=self.act_dtype, device=self.device)
        self.h = [[torch.empty((self.widths[l], self.widths[l + 1]), **f32) for _ in range(n_taps)] for l in range(self.L)]
        self.dh = [[torch.zeros_like(w) for w in hs] for hs in self.h]
        # y[l][hop] = S^hop X_l rows (hop 0 is x[l] itself)
        self.y = [[self.x[l]] + [torch.empty((self.n_total, self.widths[l]), **act) for _ in range(1, n_taps)]
                  for l in range(self.L)]
        wmax = max(self.widths[:-1])
        self._g = [torch.empty(self.n_total * wmax, **act) for _ in range(2)]

    def set_tap_weights(self, weights):
        for l in range(self.L):
            for hop in range(self.K):
                self.h[l][hop].copy_(torch.from_numpy(weights[l][hop]).to(self.device))

    def zero_grads(self):
        for hs in self.dh:
            for w in hs:
                w.zero_()

    def forward(self, step: int, ratio=None, stream=None):
        ctx = self.ctx
        ctx.set_step(step, stream)
        if ratio is not None:
            ctx.set_ratio(-1, ratio[0], ratio[1])
        self._ensure_buffers()
        self._prepare([stream])
        for l in range(self.L):
            fi, k = self.widths[l], ctx.keep(l)
            for hop in range(1, self.K):
                tap, src = vb.tap(l, hop), self.y[l][hop - 1]
                for p, hp in enumerate(self.host_parts):
                    if hp.n_boundary:
                        ctx.compress(tap, self.boundary_gid[p], self.dev_parts[p]["boundary_rows"], hp.n_boundary,
                                     src[self.rows(p)], fi, self.z[l][hp.z_row_offset * k:], stream)
                for q in range(self.P):
                    r = self.rows(q)
                    ctx.aggregate_fwd(tap, q, src[r], self.z[l], self.y[l][hop][r], stream)
            for q in range(self.P):
                r = self.rows(q)
                for hop in range(self.K):
                    ctx.transform_fwd(l, self.y[l][hop][r], self.h[l][hop], self.x[l + 1][r], hop > 0, hop == self.K - 1,
                                      stream)

    def backward(self, stream=None):
        ctx = self.ctx
        for l in range(self.L - 1, -1, -1):
            fi, k = self.widths[l], ctx.keep(l)
            for q in range(self.P):
                r = self.rows(q)
                for hop in range(self.K):
                    ctx.transform_bwd_weight(l, self.y[l][hop][r], self.dx[l + 1][r], self.x[l + 1][r], self.dh[l][hop], stream)
            if l == 0:
                continue
            bufs = [b[:self.n_total * fi].view(self.n_total, fi) for b in self._g]
            cur = self.dx[l] if self.K == 1 else bufs[0]
            for q in range(self.P):
                r = self.rows(q)
                ctx.transform_bwd_input(l, self.dx[l + 1][r], self.x[l + 1][r], self.h[l][self.K - 1], cur[r], False, stream)
            for hop in range(self.K - 1, 0, -1):
                tap = vb.tap(l, hop)
                nxt = self.dx[l] if hop == 1 else (bufs[1] if cur is bufs[0] else bufs[0])
                for q in range(self.P):
                    r = self.rows(q)
                    dzh = self.dz_halo[l][int(self.halo_off[q]) * k:] if self.n_halo[q] else None
                    ctx.aggregate_bwd(tap, q, cur[r], nxt[r], dzh, stream)
                    ctx.transform_bwd_input(l, self.dx[l + 1][r], self.x[l + 1][r], self.h[l][hop - 1], nxt[r], True, stream)
                for p in range(self.P):
                    if self.host_parts[p].n_boundary:
                        ctx.accumulate_returned(tap, p, self.ret_ptr[p], self.ret_src[p], self.dz_halo[l],
                                                nxt[self.rows(p)], stream)
                cur = nxt

"""Device-side plumbing of one emulated rank: move seeded inputs to the GPU, lay out the buffers
of a rank step (what the ring neighbour would deliver, landing buffers, send buffers), call the
C ABI through the binding, bring results back.  Used by the benchmark, the smoke check and the GPU
parity tests.  No arithmetic of the method lives here: every step of the path runs in the library."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as cf
from . import inputs

DEV = "cuda:0"


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Host array (bf16 bits as uint16, or float32) -> device tensor."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return inputs.bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max|got - ref| / max|ref| (the benchmark's parity measure)."""
    den = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    num = float(np.max(np.abs(got - ref)))
    return num / den if den > 0 else num


def desc_of(w: inputs.Workload, rank: int, w_layout=cf.CF_W_KN, **kw) -> cf.LayerDesc:
    return cf.layer_desc(w.p, rank, w.m_chunk, w.n, w.k, w.dtype, w.out_dtype, w_layout, **kw)


def w_to_dev(W: np.ndarray, dtype: str, w_layout: int) -> torch.Tensor:
    """Weight shard on the device in the requested memory order."""
    if w_layout == cf.CF_W_NK:
        W = np.ascontiguousarray(W.T)
    return to_dev(W, dtype)


class RsRun:
    """One GEMM + reduce-scatter rank step on the device."""

    def __init__(self, w: inputs.Workload, data: dict, rank: int, w_layout=cf.CF_W_KN, with_sink=False, m=1, each=False):
        self.w, self.rank, self.m = w, rank, m
        self.desc = desc_of(w, rank, w_layout, m=m)
        self.A = to_dev(data["A"], w.dtype)
        self.W = w_to_dev(data["W"], w.dtype, w_layout)
        self.stage = [to_dev(r, "f32") for r in data["R"][1:]]
        mk = lambda: torch.empty((w.m_chunk, w.n), dtype=torch.float32, device=DEV)
        self.slot = [mk(), mk()]
        self.send = [mk(), mk()]
        self.O = mk()
        self.sink = [mk() for _ in range(w.p - 1)] if with_sink else None
        self.each = [mk() for _ in range(w.p - 1)] if each else None     # one landing buffer per hop
        self.send_each = [mk() for _ in range(w.p - 1)] if each else None   # and one B_out buffer per sending step
        self.bufs = cf.make_buffers(self.A, self.W, self.O, self.stage, self.slot, self.send, self.sink, self.each,
                                    self.send_each)
        self.cs = torch.cuda.Stream()
        self.xs = torch.cuda.Stream()

    def run_steps(self):
        """Calls commfuse_rs_step once per step with the staged partial sums as B_in; returns every step's output."""
        outs = []
        m, ms = self.m, self.w.m_chunk // self.m
        for j in range(self.w.p * m):                    # sub-step j: hop j // m, row block j % m
            i, s = divmod(j, m)
            out = torch.full((ms, self.w.n), float("nan"), dtype=torch.float32, device=DEV)
            recv = self.stage[i - 1][s * ms:(s + 1) * ms] if i > 0 else None
            cf.rs_step(self.desc, j, self.A, self.W, recv, out, None)
            outs.append(out)
        torch.cuda.synchronize()
        return [to_host_f64(o) for o in outs]

    def run_schedule(self, flags=0):
        torch.cuda.synchronize()     # what the test enqueued on other streams (fills, uploads) comes first
        cf.run_schedule(self.desc, cf.CF_KIND_RS, self.bufs, self.cs, self.xs, flags)
        self.cs.synchronize()


class AgRun:
    """One all-gather + GEMM rank step on the device."""

    def __init__(self, w: inputs.Workload, data: dict, rank: int, w_layout=cf.CF_W_KN, with_sink=False, m=1, each=False):
        self.w, self.rank, self.m = w, rank, m
        self.desc = desc_of(w, rank, w_layout, m=m)
        self.X = to_dev(data["X"], w.dtype)
        self.W = w_to_dev(data["W"], w.dtype, w_layout)
        self.stage = [to_dev(s, w.dtype) for s in data["S"][1:]]
        tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        odt = torch.bfloat16 if w.out_dtype == "bf16" else torch.float32
        mk = lambda: torch.empty((w.m_chunk, w.k), dtype=tdt, device=DEV)
        self.slot = [mk(), mk()]
        self.O = torch.full((w.p * w.m_chunk, w.n), float("nan"), dtype=odt, device=DEV)
        self.sink = [mk() for _ in range(w.p - 1)] if with_sink else None
        self.each = [mk() for _ in range(w.p - 1)] if each else None
        self.bufs = cf.make_buffers(self.X, self.W, self.O, self.stage, self.slot, (None, None), self.sink, self.each)
        self.cs = torch.cuda.Stream()
        self.xs = torch.cuda.Stream()

    def run_steps(self):
        m, ms = self.m, self.w.m_chunk // self.m
        for j in range(self.w.p * m):
            i, s = divmod(j, m)
            shard = (self.X if i == 0 else self.stage[i - 1])[s * ms:(s + 1) * ms]
            cf.ag_step(self.desc, j, shard, self.W, self.O, None)
        torch.cuda.synchronize()
        return to_host_f64(self.O)

    def run_schedule(self, flags=0):
        torch.cuda.synchronize()     # what the test enqueued on other streams (fills, uploads) comes first
        cf.run_schedule(self.desc, cf.CF_KIND_AG, self.bufs, self.cs, self.xs, flags)
        self.cs.synchronize()


class DpRun:
    """The gradient reduce-scatter rank step on the device."""

    def __init__(self, w: inputs.Workload, data: dict, rank: int, with_sink=False, m=1, each=False):
        self.w, self.rank, self.m = w, rank, m
        self.desc = cf.layer_desc(w.p, rank, w.m_chunk, 0, 0, "f32", "f32", m=m)
        self.bucket = to_dev(data["bucket"], "f32")
        self.stage = [to_dev(r, "f32") for r in data["R"][1:]]
        mk = lambda: torch.empty((w.m_chunk,), dtype=torch.float32, device=DEV)
        self.slot = [mk(), mk()]
        self.sink = [mk() for _ in range(w.p - 1)] if with_sink else None
        self.each = [mk() for _ in range(w.p - 1)] if each else None      # a landing buffer per hop (CF_PERSISTENT)
        self.bufs = cf.make_buffers(None, None, self.bucket, self.stage, self.slot, (None, None), self.sink, self.each)
        self.cs = torch.cuda.Stream()
        self.xs = torch.cuda.Stream()

    def run_steps(self):
        for i in range(self.w.p):
            recv = self.stage[i - 1] if i > 0 else None
            cf.dp_reduce_step(self.w.p, self.rank, i, self.bucket, self.w.m_chunk, recv, None)
        torch.cuda.synchronize()
        return to_host_f64(self.bucket)

    def run_schedule(self, flags=0):
        torch.cuda.synchronize()     # what the test enqueued on other streams (fills, uploads) comes first
        cf.run_schedule(self.desc, cf.CF_KIND_DP, self.bufs, self.cs, self.xs, flags)
        self.cs.synchronize()


class Workspace:
    """Registers a split-K workspace sized for a layer for the duration of a ``with`` block."""

    def __init__(self, desc: cf.LayerDesc, kind: int):
        self.nbytes = cf.workspace_bytes(desc, kind)
        self.buf = torch.empty(max(self.nbytes, 16), dtype=torch.uint8, device=DEV) if self.nbytes else None

    def __enter__(self):
        if self.buf is not None:
            cf.set_workspace(self.buf, self.nbytes)
            torch.cuda.synchronize()
        return self

    def __exit__(self, *exc):
        torch.cuda.synchronize()
        cf.set_workspace(None)
        return False


class RsPairRun(RsRun):
    """One GEMM + reduce-scatter rank step under the pairwise bidirectional schedule.
    ``data["R"][t]`` stands for what the partner of round ``t`` delivers.  With ``keep_all`` every
    round's arrival has a buffer of its own and the last step sums them (deferred aggregation)."""

    def __init__(self, w, data, rank, w_layout=cf.CF_W_KN, with_sink=False, keep_all=False):
        super().__init__(w, data, rank, w_layout, with_sink)
        if keep_all:
            self.each = [torch.full((w.m_chunk, w.n), float("nan"), dtype=torch.float32, device=DEV) for _ in range(w.p - 1)]
            self.send_each = [torch.full((w.m_chunk, w.n), float("nan"), dtype=torch.float32, device=DEV)
                              for _ in range(w.p - 1)]
            self.bufs = cf.make_buffers(self.A, self.W, self.O, self.stage, (None, None), self.send, self.sink, self.each,
                                        self.send_each)

    def run_steps_deferred(self):
        """Steps with recv = acc = NULL, then commfuse_rs_pair_last_step over the staged arrivals."""
        p = self.w.p
        outs = []
        for i in range(p):
            out = torch.full((self.w.m_chunk, self.w.n), float("nan"), dtype=torch.float32, device=DEV)
            if i < p - 1:
                cf.rs_pair_step(self.desc, i, self.A, self.W, None, None, out, None)
            else:
                cf.rs_pair_last_step(self.desc, self.A, self.W, self.stage, out, None)
            outs.append(out)
        torch.cuda.synchronize()
        return [to_host_f64(o) for o in outs]

    def run_steps(self):
        """Calls commfuse_rs_pair_step once per step; returns every step's output (the sent partials, then O)."""
        p = self.w.p
        outs = []
        acc = torch.full((self.w.m_chunk, self.w.n), float("nan"), dtype=torch.float32, device=DEV)
        for i in range(p):
            out = torch.full((self.w.m_chunk, self.w.n), float("nan"), dtype=torch.float32, device=DEV)
            recv = self.stage[i - 1] if i > 0 else None
            cf.rs_pair_step(self.desc, i, self.A, self.W, recv, acc if p > 2 else None, out, None)
            outs.append(out)
        torch.cuda.synchronize()
        return [to_host_f64(o) for o in outs]

    def run_schedule(self, flags=0):
        torch.cuda.synchronize()     # what the test enqueued on other streams (fills, uploads) comes first
        cf.run_schedule(self.desc, cf.CF_KIND_RS_PAIR, self.bufs, self.cs, self.xs, flags)
        self.cs.synchronize()


class DpPairRun(DpRun):
    """The gradient reduce rank step under the pairwise bidirectional schedule."""

    def run_steps(self):
        for i in range(self.w.p):
            recv = self.stage[i - 1] if i > 0 else None
            cf.dp_pair_step(self.w.p, self.rank, i, self.bucket, self.w.m_chunk, recv, None)
        torch.cuda.synchronize()
        return to_host_f64(self.bucket)

    def run_schedule(self, flags=0):
        torch.cuda.synchronize()     # what the test enqueued on other streams (fills, uploads) comes first
        cf.run_schedule(self.desc, cf.CF_KIND_DP_PAIR, self.bufs, self.cs, self.xs, flags)
        self.cs.synchronize()


class WgradRun:
    """The weight-gradient loop of one layer on the device.  ``moving[i]`` (host arrays) is the slice in
    hand at step ``i`` (own slice first, then the deliveries), ``local`` the rank's full operand.
    ``moving_is_left``: all-gather layer (dW += moving^T local[l]), else reduce-scatter layer."""

    def __init__(self, p, rank, m_chunk, k, n, moving, local, moving_is_left, with_sink=False, m=1, each=False,
                 gathered=False):
        self.p, self.rank, self.m, self.mc, self.k, self.n = p, rank, m, m_chunk, k, n
        self.left_moves = moving_is_left
        self.kind = cf.CF_KIND_WGRAD_X if moving_is_left else cf.CF_KIND_WGRAD_G
        self.desc = cf.layer_desc(p, rank, m_chunk, n, k, "bf16", "f32", m=m)
        self.own = to_dev(moving[0], "bf16")
        self.stage = [to_dev(s, "bf16") for s in moving[1:]]
        self.local = to_dev(local, "bf16")
        width = k if moving_is_left else n
        mk = lambda: torch.empty((m_chunk, width), dtype=torch.bfloat16, device=DEV)
        self.slot = [mk(), mk()]
        self.dW = torch.full((k, n), float("nan"), dtype=torch.float32, device=DEV)
        self.sink = [mk() for _ in range(p - 1)] if with_sink else None
        self.each = [mk() for _ in range(p - 1)] if each else None
        if gathered:
            # one [p*m_chunk x width] buffer: the own slice in row block `rank`, hop i lands in row block (rank - i) mod p
            self.gathered = torch.full((p * m_chunk, width), float("nan"), dtype=torch.bfloat16, device=DEV)
            blk = lambda c: self.gathered[c * m_chunk:(c + 1) * m_chunk]
            blk(rank).copy_(self.own)
            self.own = blk(rank)
            self.each = [blk((rank - i) % p) for i in range(1, p)]
        self.bufs = cf.make_buffers(self.own, self.local, self.dW, self.stage, self.slot, (None, None), self.sink, self.each)
        self.cs = torch.cuda.Stream()
        self.xs = torch.cuda.Stream()

    def run_steps(self):
        """One commfuse_wgrad_step per (sub-)step; returns dW after every one of them."""
        outs = []
        m, ms = self.m, self.mc // self.m
        for j in range(self.p * m):
            i, s = divmod(j, m)
            hand = (self.own if i == 0 else self.stage[i - 1])[s * ms:(s + 1) * ms]
            c = cf.subslice_index(cf.CF_KIND_AG, self.p, m, self.rank, j)
            loc = self.local[c * ms:(c + 1) * ms]
            left, right = (hand, loc) if self.left_moves else (loc, hand)
            cf.wgrad_step(self.desc, j, left, right, self.dW, None)
            torch.cuda.synchronize()
            outs.append(to_host_f64(self.dW))
        return outs

    def run_schedule(self, flags=0):
        torch.cuda.synchronize()     # what the test enqueued on other streams (fills, uploads) comes first
        cf.run_schedule(self.desc, self.kind, self.bufs, self.cs, self.xs, flags)
        self.cs.synchronize()

"""Parity of the pairwise bidirectional schedule (Appendix A(a)) on the HIP path with
the CPU oracle, through the C ABI.  Needs an MI355X: run with ``-m gpu``.

Tolerances as in test_gpu_parity.py; the received partials are summed in fp32 in round
order, which adds at most (p-1) * 2^-24 relative to the largest partial sum, well inside
the tight bf16 bound.  Small-integer inputs are compared bit for bit.
"""
import contextlib
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_24013_amd import binding as cf
from paper_2604_24013_amd import inputs
from tests import harness as H

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 1e-2
TIGHT_BF16 = 1e-4


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(cf.LIB_PATH), "libcommfuse.so must be built in-tree before the GPU run"
    cf.load()
    yield
    torch.cuda.synchronize()


def _oracle_pair(w, data, rank):
    return oracle.rs_pair_rank_steps(inputs.as_f64(data["A"], w.dtype), inputs.as_f64(data["W"], w.dtype),
                                     [None] + [r.astype(np.float64) for r in data["R"][1:]], w.p, rank)


PAIR_SHAPES = [
    # (p, m_chunk, n, k)
    (2, 200, 264, 168),     # one round: out = recv + own product, no accumulator
    (4, 72, 136, 1376),     # the appendix's four devices
    (6, 130, 72, 96),       # even but not a power of two: circle-method pairing
    (8, 264, 392, 200),     # several tiles in both directions plus tails
    (1, 40, 8, 8),          # p = 1: plain GEMM
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("shape", PAIR_SHAPES)
def test_rs_pair_reduced(shape, layout, dtype):
    p, mc, n, k = shape
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k, dtype=dtype)
    data = inputs.make_rs(w, salt=11)
    tol = TOL_F32 if dtype == "f32" else TIGHT_BF16
    for rank in sorted({0, p // 2, p - 1}):
        ref = _oracle_pair(w, data, rank)
        run = H.RsPairRun(w, data, rank, layout, with_sink=True)
        outs = run.run_steps()
        for i in range(p):
            e = H.rel_err(outs[i], ref[i])
            assert e <= tol, f"rank {rank} step {i}: rel err {e:.3e}"
            assert not np.isnan(outs[i]).any()
        # aggregation deferred to the last step: same additions in the same order, so the same bits
        outs_d = run.run_steps_deferred()
        for i in range(p):
            assert np.array_equal(outs_d[i], outs[i]), f"rank {rank} step {i} (deferred)"
        keep = H.RsPairRun(w, data, rank, layout, with_sink=True, keep_all=True)
        for r_ in (run, keep):
            for flags in (0, cf.CF_SERIAL, cf.CF_POISON, cf.CF_GRAPH):
                r_.O.fill_(float("nan"))
                for s in r_.sink:
                    s.fill_(float("nan"))
                r_.run_schedule(flags)
                assert np.array_equal(H.to_host_f64(r_.O), outs[-1]), f"rank {rank} flags {flags}"
                for i in range(p - 1):
                    assert np.array_equal(H.to_host_f64(r_.sink[i]), outs[i]), f"rank {rank} flags {flags} sink {i}"
        if dtype == "bf16":
            # all steps in one launch: the same GEMMs and the same additions in the same order
            pers = H.RsPairRun(w, data, rank, layout, keep_all=True)
            PS = cf.CF_PERSISTENT | cf.CF_SERIAL
            # (CF_FUSED_COPY: no copy is launched; the work items of step t - 1 land the arrival of round t tile by
            # tile, the last step's work items wait for their tile's count -- with a registered workspace; without
            # one the copies go in front as without the flag)
            FC = PS | cf.CF_FUSED_COPY
            for flags, with_ws in ((PS, False), (PS | cf.CF_GRAPH, False), (PS | cf.CF_POISON, False), (FC, False),
                                   (FC, True), (FC | cf.CF_GRAPH, True)):
                pers.O.fill_(float("nan"))
                for t in pers.send_each + pers.each:
                    t.fill_(float("nan"))
                ws = H.Workspace(pers.desc, cf.CF_KIND_RS_PAIR) if with_ws else contextlib.nullcontext()
                with ws:
                    pers.run_schedule(flags)
                    pers.run_schedule(flags)
                    cf.device_status()               # no wait timed out
                assert np.array_equal(H.to_host_f64(pers.O), outs[-1]), f"rank {rank} flags {flags} (persistent)"
                for i in range(p - 1):               # the partial every step sends to its partner
                    assert np.array_equal(H.to_host_f64(pers.send_each[i]), outs[i]), \
                        f"rank {rank} flags {flags} (persistent) B_out of step {i}"
                    assert torch.equal(pers.each[i], pers.stage[i]), f"rank {rank} flags {flags}: delivery of round {i + 1}"


def test_rs_pair_deferred_with_the_staged_kernel():
    """The register-staged bf16 kernel takes no list of arrivals: they are summed in `out` first."""
    p, mc, n, k = 4, 136, 264, 200
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=13)
    ref = _oracle_pair(w, data, 2)
    os.environ["COMMFUSE_KERNEL"] = "staged"
    try:
        run = H.RsPairRun(w, data, 2, keep_all=True)
        outs = run.run_steps_deferred()
        run.run_schedule(0)
    finally:
        os.environ.pop("COMMFUSE_KERNEL", None)
    for i in range(p):
        assert H.rel_err(outs[i], ref[i]) <= TIGHT_BF16
    assert np.array_equal(H.to_host_f64(run.O), outs[-1])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rs_pair_integer_inputs_are_bit_exact(dtype):
    p, mc, n, k = 4, 136, 264, 200
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k, dtype=dtype)
    rng = np.random.default_rng(78)
    A = inputs.small_int_like((p * mc, k), rng)
    W = inputs.small_int_like((k, n), rng)
    R = [None] + [inputs.small_int_like((mc, n), rng, -50, 50) for _ in range(p - 1)]
    data = {"A": inputs._as_dtype(A, dtype), "W": inputs._as_dtype(W, dtype), "R": R}
    for rank in range(p):
        ref = _oracle_pair(w, data, rank)
        run = H.RsPairRun(w, data, rank)
        outs = run.run_steps()
        for i in range(p):
            assert np.array_equal(outs[i], ref[i]), f"rank {rank} step {i}"
        run.run_schedule(0)
        assert np.array_equal(H.to_host_f64(run.O), ref[-1])


def test_rs_pair_steps_address_the_partner_slices():
    """Step i of rank r multiplies the slice of the partner of round i+1 (the appendix's table for p = 4)."""
    p, mc, n, k = 4, 8, 8, 8
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    # slice l of A is the constant l+1, W the identity: step output = l+1 everywhere
    A = np.concatenate([np.full((mc, k), float(l + 1), dtype=np.float32) for l in range(p)])
    data = {"A": inputs._as_dtype(A, "bf16"), "W": inputs._as_dtype(np.eye(k, dtype=np.float32), "bf16"),
            "R": [None] + [np.zeros((mc, n), dtype=np.float32) for _ in range(p - 1)]}
    table = {0: [1, 2, 3, 0], 1: [0, 3, 2, 1], 2: [3, 0, 1, 2], 3: [2, 1, 0, 3]}   # A<->B, A<->C, A<->D ... then own
    for rank in range(p):
        outs = H.RsPairRun(w, data, rank).run_steps()
        assert [int(o[0, 0]) - 1 for o in outs] == table[rank]
        assert [cf.chunk_index(cf.CF_KIND_RS_PAIR, p, rank, i) for i in range(p)] == table[rank]


@pytest.mark.parametrize("p,c", [(8, 1_000_003), (4, 4096), (2, 5), (1, 64), (6, 262144)])
def test_dp_pair_reduced(p, c):
    w = inputs.scaled(inputs.CONFIGS["c5_dp"], p=p, m_chunk=c)
    rank = p - 1
    # integer-valued gradients: every fp32 sum is exact, so the comparison is bit for bit
    rng = np.random.default_rng(5 * p + 1)
    data = {"bucket": inputs.small_int_like((p * c,), rng, -1000, 1000),
            "R": [None] + [inputs.small_int_like((c,), rng, -1000, 1000) for _ in range(p - 1)]}
    ref = oracle.dp_pair_rank(data["bucket"], data["R"], p, rank)
    got = H.DpPairRun(w, data, rank).run_steps()
    assert np.array_equal(got, ref)
    run = H.DpPairRun(w, data, rank, with_sink=True)
    run.run_schedule()
    assert np.array_equal(H.to_host_f64(run.bucket), ref)
    for i in range(p - 1):
        l = oracle.slice_index_pair(p, rank, i)
        assert np.array_equal(H.to_host_f64(run.sink[i]), data["bucket"][l * c:(l + 1) * c].astype(np.float64))
    # CF_PERSISTENT: all rounds' deliveries as one batched copy into a buffer per round, then the adds in round order
    # (with CF_FUSED_COPY no copy is launched: the one add pass reads the partners' buffers and lands what it reads)
    for flags in (cf.CF_PERSISTENT | cf.CF_SERIAL, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY):
        pers = H.DpPairRun(w, data, rank, each=True)
        for t in pers.each:
            t.fill_(float("nan"))
        torch.cuda.synchronize()                     # the fills run on another stream than the schedule
        pers.run_schedule(flags)
        assert np.array_equal(H.to_host_f64(pers.bucket), ref), f"flags {flags}"
        for i in range(p - 1):
            assert torch.equal(pers.each[i], pers.stage[i]), f"flags {flags}: delivery of round {i + 1}"
    # normally distributed gradients: p-1 fp32 additions in round order
    data = inputs.make_dp(w, salt=9)
    ref = oracle.dp_pair_rank(data["bucket"], data["R"], p, rank)
    got = H.DpPairRun(w, data, rank).run_steps()
    scale = max(1.0, float(np.abs(ref).max()))
    assert np.max(np.abs(got - ref)) <= (p - 1) * 2.0 ** -24 * scale * 2
    pers = H.DpPairRun(w, data, rank, each=True)
    pers.run_schedule(cf.CF_PERSISTENT | cf.CF_SERIAL)
    assert np.array_equal(H.to_host_f64(pers.bucket), got)       # the same adds in the same order


_full_refs = {}


def _full_ref(name, rank):
    """Seeded inputs and the oracle's outputs of every step of a full-size configuration (computed once)."""
    if (name, rank) not in _full_refs:
        w = inputs.CONFIGS[name]
        data = inputs.make_rs(w, salt=12)
        ref = oracle.rs_pair_rank_steps(inputs.as_f64(data["A"], w.dtype), inputs.as_f64(data["W"], w.dtype),
                                        [None] + [r.astype(np.float64) for r in data["R"][1:]], w.p, rank)
        _full_refs[(name, rank)] = (data, ref)
    return _full_refs[(name, rank)]


@pytest.mark.parametrize("keep_all", [False, True])
@pytest.mark.parametrize("flags", [0, cf.CF_GRAPH, cf.CF_PERSISTENT | cf.CF_SERIAL,
                                   cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY])
@pytest.mark.parametrize("name", ["c2_rs_7b", "c4_rs_70b_down"])
def test_full_size_rs_pair(name, flags, keep_all):
    """Full benchmark sizes; every element of every step's output (the partials sent to the partners, then the
    reduced own slice) against the oracle."""
    w = inputs.CONFIGS[name]
    rank = 5
    persistent = bool(flags & cf.CF_PERSISTENT)      # deferred aggregation only; every B_out in a buffer of its own
    if persistent and not keep_all:
        pytest.skip("the persistent launch keeps every arrival (recv_each)")
    data, ref = _full_ref(name, rank)
    run = H.RsPairRun(w, data, rank, with_sink=True, keep_all=keep_all)
    for t in run.sink + [run.O]:
        t.fill_(float("nan"))
    with H.Workspace(run.desc, cf.CF_KIND_RS_PAIR):       # as the benchmark runs it
        run.run_schedule(flags)
        if flags & cf.CF_FUSED_COPY:
            run.run_schedule(flags)                       # (the tiles' counters are ready for a second launch)
        cf.device_status()
    for i in range(w.p):
        got = H.to_host_f64(run.sink[i] if i < w.p - 1 else run.O)
        assert not np.isnan(got).any(), f"step {i}"
        e = H.rel_err(got, ref[i])
        assert e <= TOL_BF16 and e <= TIGHT_BF16, f"step {i}: {e:.3e}"
        if persistent and i < w.p - 1:
            assert torch.equal(run.sink[i], run.send_each[i])
            assert torch.equal(run.each[i], run.stage[i]), f"delivery of round {i + 1}"


def test_pair_rejects_what_it_cannot_do():
    d = cf.layer_desc(3, 0, 64, 64, 64)
    t = torch.zeros(64 * 64 * 3, dtype=torch.float32, device=H.DEV)
    with pytest.raises(cf.CommFuseError) as ei:
        cf.rs_pair_step(d, 0, t, t, None, t, t, None)            # odd p
    assert ei.value.status == cf.CF_ERR_INVALID_ARG
    d = cf.layer_desc(4, 0, 64, 64, 64)
    with pytest.raises(cf.CommFuseError):
        cf.rs_pair_step(d, 1, t, t, t[:4096], t[4096:8192], t[4096:8192], None)   # out aliases acc before the last step
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=4, m_chunk=64, n=64, k=64)
    run = H.RsPairRun(w, inputs.make_rs(w), 0)
    for flags in (cf.CF_FUSED_COPY, cf.CF_DEVICE_WAIT):          # (CF_FUSED_COPY goes with CF_PERSISTENT only)
        with pytest.raises(cf.CommFuseError) as ei:
            run.run_schedule(flags)
        assert ei.value.status == cf.CF_ERR_UNSUPPORTED


def test_rs_pair_carried_wait_is_bounded_and_recovers():
    """The last step's wait for its tile's arrivals is a bounded spin.  With a limit of one poll, forced from the host,
    a work item may give up (then the status call says so and the result is void); every kernel exits either way, and
    the next launch -- its counters filled with zero in front -- is correct again."""
    p, mc, n, k = 4, 256, 256, 128                   # one output tile per step: the four work items run side by side
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=17)
    ref = _oracle_pair(w, data, 1)
    run = H.RsPairRun(w, data, 1, keep_all=True)
    FC = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY
    os.environ["COMMFUSE_SPIN_LIMIT"] = "1"
    try:
        with H.Workspace(run.desc, cf.CF_KIND_RS_PAIR):
            run.run_schedule(FC)
            try:
                cf.device_status(run.cs)
                timed_out = False
            except cf.CommFuseError as e:
                assert "gave up waiting" in str(e)
                timed_out = True
            if not timed_out:
                assert H.rel_err(H.to_host_f64(run.O), ref[-1]) <= TIGHT_BF16
            os.environ.pop("COMMFUSE_SPIN_LIMIT", None)
            run.O.fill_(float("nan"))
            for t in run.each:
                t.fill_(float("nan"))
            run.run_schedule(FC)
            cf.device_status(run.cs)
            assert H.rel_err(H.to_host_f64(run.O), ref[-1]) <= TIGHT_BF16
            for i in range(p - 1):
                assert torch.equal(run.each[i], run.stage[i])
    finally:
        os.environ.pop("COMMFUSE_SPIN_LIMIT", None)


@pytest.mark.parametrize("tile", ["128x128", "256x128", "256x256"])
def test_rs_pair_carried_on_every_tile_shape(tile):
    """The landing of the arrivals behind the work items and the per-tile wait, on each tile shape of the one-launch
    kernel (the work item's part of an arrival is its own output tile), several tiles per step and ragged edges."""
    p, mc, n, k = 8, 520, 776, 328
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=19)
    rank = 6
    ref = _oracle_pair(w, data, rank)
    FC = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY
    os.environ["COMMFUSE_TILE"] = tile
    try:
        for layout in (cf.CF_W_KN, cf.CF_W_NK):
            run = H.RsPairRun(w, data, rank, layout, keep_all=True)
            with H.Workspace(run.desc, cf.CF_KIND_RS_PAIR):
                for rep in range(2):
                    run.O.fill_(float("nan"))
                    for t in run.send_each + run.each:
                        t.fill_(float("nan"))
                    run.run_schedule(FC)
                    cf.device_status(run.cs)
                    for i in range(p):
                        got = H.to_host_f64(run.send_each[i] if i < p - 1 else run.O)
                        e = H.rel_err(got, ref[i])
                        assert e <= TIGHT_BF16, f"layout {layout} step {i}: {e:.3e}"
                    for i in range(p - 1):
                        assert torch.equal(run.each[i], run.stage[i]), f"layout {layout}: delivery of round {i + 1}"
    finally:
        os.environ.pop("COMMFUSE_TILE", None)


@pytest.mark.parametrize("k", [64, 192, 1096, 2304])
def test_rs_pair_carried_under_the_16x16x32_main_loop(k):
    """Whole 256x256 tiles: the kernel deals the landing of an arrival over the k-tiles of its main loop (one
    16-byte load and one store per lane and k-tile) and copies what the k range leaves over behind the epilogue:
    one k-tile (nothing dealt), three, seventeen with a ragged tail, thirty-six (everything dealt)."""
    p, mc, n = 4, 512, 768
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=23 + k)
    rank = 1
    ref = _oracle_pair(w, data, rank)
    FC = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY
    os.environ["COMMFUSE_TILE"] = "256x256"
    try:
        for layout in (cf.CF_W_KN, cf.CF_W_NK):
            run = H.RsPairRun(w, data, rank, layout, keep_all=True)
            with H.Workspace(run.desc, cf.CF_KIND_RS_PAIR):
                for rep in range(2):
                    run.O.fill_(float("nan"))
                    for t in run.send_each + run.each:
                        t.fill_(float("nan"))
                    run.run_schedule(FC)
                    cf.device_status(run.cs)
                    for i in range(p):
                        got = H.to_host_f64(run.send_each[i] if i < p - 1 else run.O)
                        e = H.rel_err(got, ref[i])
                        assert e <= TIGHT_BF16, f"layout {layout} step {i}: {e:.3e}"
                    for i in range(p - 1):
                        assert torch.equal(run.each[i], run.stage[i]), f"layout {layout}: delivery of round {i + 1}"
    finally:
        os.environ.pop("COMMFUSE_TILE", None)

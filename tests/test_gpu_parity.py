"""Parity of the HIP path with the CPU oracle, element by element, on the same
seeded inputs, through the C ABI.  Needs an MI355X: run with ``-m gpu``.

Tolerances (max|gpu - ref| / max|ref| per checked tensor):
  * fp32 operands: 1e-5 (the benchmark's bound).
  * bf16 operands with fp32 accumulation: 1e-2 (the benchmark's bound); in
    addition a tight bound of 1e-4 is asserted -- the inputs are exact bf16
    values and the only error is fp32 accumulation over K <= 8192 terms,
    about sqrt(K) * 2^-24 of the largest partial sum.
  * bf16 output: adds half a bf16 ulp of the element, 2^-9 relative.
  * small-integer inputs: bit-exact (every product and partial sum is exact).
"""
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
TIGHT_BF16_OUT = 2.0 ** -8


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(cf.LIB_PATH), "libcommfuse.so must be built in-tree before the GPU run"
    cf.load()
    yield
    torch.cuda.synchronize()


def _tile_env(tile):
    if tile is None:
        os.environ.pop("COMMFUSE_TILE", None)
    else:
        os.environ["COMMFUSE_TILE"] = tile


def _oracle_rs(w, data, rank):
    return oracle.rs_rank_steps(inputs.as_f64(data["A"], w.dtype), inputs.as_f64(data["W"], w.dtype),
                                [None] + [r.astype(np.float64) for r in data["R"][1:]], w.p, rank)


def _oracle_ag(w, data, rank):
    S = [None] + [inputs.as_f64(s, w.dtype) for s in data["S"][1:]]
    O = oracle.ag_rank(inputs.as_f64(data["X"], w.dtype), S, inputs.as_f64(data["W"], w.dtype), w.p, rank)
    return O


def _tols(w):
    if w.dtype == "f32":
        return TOL_F32, TOL_F32
    if w.out_dtype == "bf16" and w.kind == "ag":
        return TOL_BF16, TIGHT_BF16_OUT
    return TOL_BF16, TIGHT_BF16


# ----------------------------------------------------------------------------
# configuration 1 in full: fp32, p = 2, both ranks, per-step calls and schedule
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("rank", [0, 1])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
def test_c1_fp32_full(rank, layout):
    w = inputs.CONFIGS["c1_rs_f32"]
    data = inputs.make_rs(w)
    ref = _oracle_rs(w, data, rank)
    run = H.RsRun(w, data, rank, layout, with_sink=True)
    outs = run.run_steps()
    for i in range(w.p):
        assert H.rel_err(outs[i], ref[i]) <= TOL_F32, f"step {i}"
    run.run_schedule()
    assert H.rel_err(H.to_host_f64(run.O), ref[-1]) <= TOL_F32
    for i in range(w.p - 1):
        assert H.rel_err(H.to_host_f64(run.sink[i]), ref[i]) <= TOL_F32


# ----------------------------------------------------------------------------
# reduced shapes spanning several tiles and ragged tails, every tile config
# ----------------------------------------------------------------------------

RS_SHAPES = [
    # (p, m_chunk, n, k)
    (3, 200, 264, 168),     # ragged in M, N and K (K = 2*64 + 40)
    (2, 256, 512, 64),      # exact tiles, a single k-tile
    (4, 72, 136, 1376),     # the 7B down-projection's K (21*64 + 32)
    (1, 40, 8, 8),          # p = 1: plain GEMM, minimum n and k
    (8, 520, 392, 200),     # several tiles in both directions plus tails
    (3, 200, 264, 1160),    # 19 k-tiles, the last ragged: long enough for B_in to be brought in under the main loop
    (2, 256, 512, 1152),    # 18 whole k-tiles, exact tiles
]


@pytest.mark.parametrize("tile", [None, "256x256", "256x128", "128x128"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("shape", RS_SHAPES)
def test_rs_bf16_reduced(shape, layout, tile):
    p, mc, n, k = shape
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=1)
    rank = (p - 1) // 2
    ref = _oracle_rs(w, data, rank)
    _tile_env(tile)
    try:
        run = H.RsRun(w, data, rank, layout)
        outs = run.run_steps()
    finally:
        _tile_env(None)
    for i in range(p):
        e = H.rel_err(outs[i], ref[i])
        assert e <= TOL_BF16 and e <= TIGHT_BF16, f"step {i}: rel err {e:.3e}"
        assert not np.isnan(outs[i]).any()


@pytest.mark.parametrize("splitk", [2, 3, 8])
@pytest.mark.parametrize("tile", ["256x256", "128x128"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
def test_split_k_reduced(layout, tile, splitk):
    """k range of every output tile split over several workgroups (workspace registered)."""
    p, mc, n, k = 3, 200, 264, 1000          # 16 k-tiles of 64 (the last one ragged)
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=8)
    ref = _oracle_rs(w, data, 1)
    wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=p, m_chunk=mc, n=n, k=k, out_dtype="bf16")
    da = inputs.make_ag(wa, salt=8)
    refa = _oracle_ag(wa, da, 1)
    ws = torch.empty(cf.workspace_bytes(H.desc_of(w, 1), cf.CF_KIND_RS), dtype=torch.uint8, device=H.DEV)
    cf.set_workspace(ws)
    torch.cuda.synchronize()
    _tile_env(tile)
    os.environ["COMMFUSE_SPLITK"] = str(splitk)
    try:
        outs = H.RsRun(w, data, 1, layout).run_steps()
        outs2 = H.RsRun(w, data, 1, layout).run_steps()      # counters must be back at zero
        got_ag = H.AgRun(wa, da, 1, layout).run_steps()
    finally:
        _tile_env(None)
        os.environ.pop("COMMFUSE_SPLITK", None)
        torch.cuda.synchronize()
        cf.set_workspace(None)
    for i in range(p):
        e = H.rel_err(outs[i], ref[i])
        assert e <= TIGHT_BF16, f"step {i}: rel err {e:.3e}"
        assert np.array_equal(outs[i], outs2[i]), "split-K result must not depend on arrival order"
    assert H.rel_err(got_ag, refa) <= TIGHT_BF16_OUT


def test_two_layers_in_flight_split_k_with_a_workspace_per_stream():
    """A workspace registered for a stream serves the work enqueued on that stream: two rank steps that run side by
    side on two streams, both with their k ranges split, each park their partial tiles in a workspace of their own."""
    p, mc, n, k = 4, 264, 520, 2112          # 33 k-tiles
    runs, refs, wss = [], [], []
    for salt in (31, 32):
        w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
        data = inputs.make_rs(w, salt=salt)
        refs.append(_oracle_rs(w, data, 2))
        run = H.RsRun(w, data, 2, with_sink=True)
        ws = torch.full((cf.workspace_bytes(run.desc, cf.CF_KIND_RS),), 0xFF, dtype=torch.uint8, device=H.DEV)
        torch.cuda.synchronize()                            # the fill first: the registration zeroes the counters on run.cs
        cf.set_workspace(ws, stream=run.cs)                 # for the work enqueued on this run's compute stream
        runs.append(run)
        wss.append(ws)
    torch.cuda.synchronize()
    os.environ["COMMFUSE_TILE"] = "128x128"
    os.environ["COMMFUSE_SPLITK"] = "3"
    try:
        for rep in range(3):                                 # enqueue both, then wait: the two rank steps overlap in time
            for run in runs:
                cf.run_schedule(run.desc, cf.CF_KIND_RS, run.bufs, run.cs, run.xs, 0)
        torch.cuda.synchronize()
        for run in runs:
            cf.device_status(run.cs)
    finally:
        os.environ.pop("COMMFUSE_TILE", None)
        os.environ.pop("COMMFUSE_SPLITK", None)
        torch.cuda.synchronize()
        for run in runs:
            cf.set_workspace(None, stream=run.cs)
    for run, ref, ws in zip(runs, refs, wss):
        for i in range(p):
            got = H.to_host_f64(run.sink[i] if i < p - 1 else run.O)
            e = H.rel_err(got, ref[i])
            assert e <= TIGHT_BF16, f"step {i}: {e:.3e}"
        # the partial tiles were parked in this run's own workspace (it was all 0xFF bytes before)
        assert not bool((ws[64 * 1024:64 * 1024 + 4096] == 0xFF).all())


AG_SHAPES = [(3, 200, 264, 168), (2, 128, 128, 4096), (4, 72, 136, 1376), (1, 33, 16, 24), (8, 260, 520, 72)]


@pytest.mark.parametrize("tile", [None, "256x256", "256x128", "128x128"])
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("shape", AG_SHAPES)
def test_ag_bf16_reduced(shape, layout, out_dtype, tile):
    p, mc, n, k = shape
    w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=p, m_chunk=mc, n=n, k=k, out_dtype=out_dtype)
    data = inputs.make_ag(w, salt=2)
    rank = p // 2
    ref = _oracle_ag(w, data, rank)
    _tile_env(tile)
    try:
        got = H.AgRun(w, data, rank, layout).run_steps()
    finally:
        _tile_env(None)
    gate, tight = _tols(w)
    e = H.rel_err(got, ref)
    assert not np.isnan(got).any(), "a slice of O was never written"
    assert e <= gate and e <= tight, f"rel err {e:.3e}"


@pytest.mark.parametrize("tile", ["64x64", "128x128"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("shape", [(2, 100, 68, 36), (3, 64, 128, 16), (1, 130, 132, 260), (4, 129, 260, 100)])
def test_fp32_reduced(shape, layout, tile):
    p, mc, n, k = shape
    w = inputs.scaled(inputs.CONFIGS["c1_rs_f32"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=3)
    rank = p - 1
    ref = _oracle_rs(w, data, rank)
    os.environ["COMMFUSE_TILE_F32"] = tile
    try:
        outs = H.RsRun(w, data, rank, layout).run_steps()
        wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=p, m_chunk=mc, n=n, k=k, dtype="f32", sigma_a=1.0, sigma_w=1.0)
        da = inputs.make_ag(wa, salt=3)
        got_ag = H.AgRun(wa, da, rank, layout).run_steps()
    finally:
        os.environ.pop("COMMFUSE_TILE_F32", None)
    for i in range(p):
        assert H.rel_err(outs[i], ref[i]) <= TOL_F32, f"step {i}"
    assert H.rel_err(got_ag, _oracle_ag(wa, da, rank)) <= TOL_F32


# ----------------------------------------------------------------------------
# bit-exact cases: small-integer inputs, strides, and the step/slice addressing
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
def test_integer_inputs_are_bit_exact(dtype, layout):
    p, mc, n, k = 4, 136, 264, 200
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k, dtype=dtype)
    rng = np.random.default_rng(77)
    A = inputs.small_int_like((p * mc, k), rng)
    W = inputs.small_int_like((k, n), rng)
    R = [None] + [inputs.small_int_like((mc, n), rng, -50, 50) for _ in range(p - 1)]
    data = {"A": inputs._as_dtype(A, dtype), "W": inputs._as_dtype(W, dtype), "R": R}
    for rank in range(p):
        ref = _oracle_rs(w, data, rank)
        outs = H.RsRun(w, data, rank, layout).run_steps()
        for i in range(p):
            assert np.array_equal(outs[i], ref[i]), f"rank {rank} step {i}"


@pytest.mark.parametrize("stream", ["1", "0"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
def test_b_in_added_in_mid_sum_is_bit_exact_on_integers(layout, stream):
    """256x256 tile with a long k range: the received partial lands in LDS under the main loop and is added to
    the accumulators in mid-sum (another order of the same additions).  On small-integer data every order gives
    the same bits, per-step launches and the one-launch rank step alike; with the path switched off too."""
    p, mc, n, k = 4, 264, 520, 1224                     # 20 k-tiles (the last ragged), tiles ragged in M and N
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    rng = np.random.default_rng(78)
    A = inputs.small_int_like((p * mc, k), rng, -4, 4)
    W = inputs.small_int_like((k, n), rng, -4, 4)
    R = [None] + [inputs.small_int_like((mc, n), rng, -50, 50) for _ in range(p - 1)]
    data = {"A": inputs._as_dtype(A, "bf16"), "W": inputs._as_dtype(W, "bf16"), "R": R}
    os.environ["COMMFUSE_TILE"] = "256x256"
    os.environ["COMMFUSE_STREAM_RECV"] = stream
    try:
        for rank in (0, p - 1):
            ref = _oracle_rs(w, data, rank)
            run = H.RsRun(w, data, rank, layout, each=True)
            outs = run.run_steps()
            for i in range(p):
                assert np.array_equal(outs[i], ref[i]), f"rank {rank} step {i}"
            for fl in (cf.CF_PERSISTENT | cf.CF_SERIAL, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY):
                for t in run.each + run.send_each + [run.O]:
                    t.fill_(float("nan"))
                run.run_schedule(fl)
                for i in range(p):
                    got = H.to_host_f64(run.send_each[i] if i < p - 1 else run.O)
                    assert np.array_equal(got, ref[i]), f"rank {rank} step {i} (one launch, flags {fl})"
                for i in range(p - 1):               # delivered by the batched copy or by the kernel itself
                    assert torch.equal(run.each[i], run.stage[i]), f"rank {rank} hop {i + 1} (flags {fl})"
    finally:
        os.environ.pop("COMMFUSE_TILE", None)
        os.environ.pop("COMMFUSE_STREAM_RECV", None)


@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("shape", [(3, 200, 264, 168), (4, 72, 136, 1376), (2, 264, 520, 328)])
def test_register_staged_kernel(shape, layout):
    """The fallback kernel for operands of 2 GiB and more (global -> registers -> LDS), forced on small shapes."""
    p, mc, n, k = shape
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=17)
    ref = _oracle_rs(w, data, 1)
    wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=p, m_chunk=mc, n=n, k=k, out_dtype="bf16")
    da = inputs.make_ag(wa, salt=17)
    refa = _oracle_ag(wa, da, 1)
    os.environ["COMMFUSE_KERNEL"] = "staged"
    try:
        outs = H.RsRun(w, data, 1, layout).run_steps()
        O = H.AgRun(wa, da, 1, layout).run_steps()
    finally:
        os.environ.pop("COMMFUSE_KERNEL", None)
    for i in range(p):
        assert H.rel_err(outs[i], ref[i]) <= TIGHT_BF16, f"step {i}"
    assert H.rel_err(O, refa) <= TIGHT_BF16_OUT


def test_slice_of_two_gib_takes_the_fallback_kernel():
    """Maximum sizes: a slice whose byte extent reaches 2^31 cannot use 32-bit buffer offsets; the step still
    runs (register-staged kernel) and the rows at both ends and around the 2 GiB / 32-bit-index marks are right."""
    p, mc, n, k = 1, 131072, 8, 8192                      # the slice is 131072 x 8192 bf16 = 2 GiB exactly
    blk = 4096
    wb = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=1, m_chunk=blk, n=n, k=k)
    data = inputs.make_rs(wb, salt=18)                    # one seeded block of rows, repeated to fill the slice
    A = H.to_dev(data["A"], "bf16").repeat(mc // blk, 1)
    assert A.numel() * 2 == 1 << 31
    W = H.to_dev(data["W"], "bf16")
    out = torch.full((mc, n), float("nan"), dtype=torch.float32, device=H.DEV)
    cf.rs_step(cf.layer_desc(p, 0, mc, n, k), 0, A, W, None, out, None)
    torch.cuda.synchronize()
    got = H.to_host_f64(out)
    assert not np.isnan(got).any()
    ref_blk = oracle.gemm(inputs.as_f64(data["A"], "bf16"), inputs.as_f64(data["W"], "bf16"))
    for r0 in (0, 65536 - blk, 65536, mc - blk):          # first, either side of the middle, last block
        assert H.rel_err(got[r0:r0 + blk], ref_blk) <= TIGHT_BF16, f"rows from {r0}"
    assert np.array_equal(got[:blk], got[mc - blk:]), "the same rows give the same bits wherever they sit"


def test_row_strides_are_honoured():
    p, mc, n, k = 2, 96, 72, 136
    lda, ldw, ldo = k + 24, n + 8, n + 16
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    rng = np.random.default_rng(78)
    A = inputs.small_int_like((p * mc, lda), rng)
    W = inputs.small_int_like((k, ldw), rng)
    Rp = inputs.small_int_like((mc, ldo), rng, -9, 9)
    desc = cf.layer_desc(p, 0, mc, n, k, "bf16", "f32", cf.CF_W_KN, lda=lda, ldw=ldw, ldo=ldo)
    dA, dW, dR = H.to_dev(inputs.f32_to_bf16_bits(A), "bf16"), H.to_dev(inputs.f32_to_bf16_bits(W), "bf16"), H.to_dev(Rp, "f32")
    out = torch.full((mc, ldo), -777.0, dtype=torch.float32, device=H.DEV)
    cf.rs_step(desc, 1, dA, dW, dR, out, None)          # rank 0, step 1 -> slice (0-1-1) mod 2 = 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.gemm(A[:mc, :k], W[:, :n]) + Rp[:, :n]
    assert np.array_equal(got[:, :n], ref)
    assert np.all(got[:, n:] == -777.0), "padding columns of the output were written"


# ----------------------------------------------------------------------------
# gradient path
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("p,c", [(8, 1_000_003), (4, 4096), (2, 5), (1, 64), (3, 0), (8, 262144)])
def test_dp_reduced(p, c):
    w = inputs.scaled(inputs.CONFIGS["c5_dp"], p=p, m_chunk=c)
    data = inputs.make_dp(w, salt=4)
    rank = p - 1
    ref = oracle.dp_rank(data["bucket"], data["R"], p, rank)
    got = H.DpRun(w, data, rank).run_steps()
    # one fp32 addition per element: the result is the correctly rounded sum
    want32 = ref.astype(np.float32).astype(np.float64)
    assert np.array_equal(got, want32)
    if c == 0:
        return
    run = H.DpRun(w, data, rank, with_sink=True)
    run.run_schedule()
    assert np.array_equal(H.to_host_f64(run.bucket), want32)
    for i in range(p - 1):
        l = (rank - i - 1) % p
        assert np.array_equal(H.to_host_f64(run.sink[i]), want32[l * c:(l + 1) * c])
    # CF_PERSISTENT: every hop lands in a buffer of its own, all deliveries as one batched copy (slices whose
    # byte size is no multiple of 16: one copy per hop), then the same adds
    run = H.DpRun(w, data, rank, each=True)
    # (with CF_FUSED_COPY no copy is launched: the add kernels read the neighbours' buffers and land what they read)
    for flags in (cf.CF_PERSISTENT | cf.CF_SERIAL, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_GRAPH,
                  cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_GRAPH, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY,
                  cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY | cf.CF_GRAPH):
        run.bucket.copy_(H.to_dev(data["bucket"], "f32"))
        for t in run.each:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        run.run_schedule(flags)
        assert np.array_equal(H.to_host_f64(run.bucket), want32), f"flags {flags}"
        for i in range(p - 1):
            assert torch.equal(run.each[i], run.stage[i]), f"flags {flags}: delivery of hop {i + 1}"
    if p > 1:
        with pytest.raises(cf.CommFuseError) as ei:              # a landing buffer per hop is a CF_PERSISTENT matter here
            run.run_schedule(cf.CF_SERIAL)
        assert ei.value.status == cf.CF_ERR_INVALID_ARG


# ----------------------------------------------------------------------------
# the emulated rank step: flags, poison, graph replays, sinks
# ----------------------------------------------------------------------------

def test_schedule_modes_agree_rs():
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=8, m_chunk=264, n=520, k=328)
    data = inputs.make_rs(w, salt=5)
    rank = 3
    ref = _oracle_rs(w, data, rank)
    for flags in (0, cf.CF_SERIAL, cf.CF_POISON, cf.CF_POISON | cf.CF_SERIAL, cf.CF_GRAPH, cf.CF_FUSED_COPY,
                  cf.CF_FUSED_COPY | cf.CF_GRAPH, cf.CF_DEVICE_WAIT,
                  cf.CF_DEVICE_WAIT | cf.CF_POISON):
        run = H.RsRun(w, data, rank, with_sink=True)
        run.O.fill_(float("nan"))
        with H.Workspace(run.desc, cf.CF_KIND_RS):
            run.run_schedule(flags)
            cf.device_status(run.cs)
        e = H.rel_err(H.to_host_f64(run.O), ref[-1])
        assert e <= TIGHT_BF16, f"flags {flags}: {e:.3e}"
        for i in range(w.p - 1):
            assert H.rel_err(H.to_host_f64(run.sink[i]), ref[i]) <= TIGHT_BF16, f"flags {flags} sink {i}"
    # compute-only after a full run reuses whatever the slots hold: last two deliveries
    run = H.RsRun(w, data, rank)
    run.run_schedule(cf.CF_NO_COMPUTE)
    assert np.array_equal(H.to_host_f64(run.slot[(w.p - 1) & 1]), data["R"][w.p - 1].astype(np.float64))
    assert np.array_equal(H.to_host_f64(run.slot[(w.p - 2) & 1]), data["R"][w.p - 2].astype(np.float64))


def test_schedule_modes_agree_ag():
    w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=136, n=264, k=520)
    data = inputs.make_ag(w, salt=6)
    rank = 5
    ref = _oracle_ag(w, data, rank)
    for flags in (0, cf.CF_SERIAL, cf.CF_POISON, cf.CF_GRAPH, cf.CF_FUSED_COPY, cf.CF_FUSED_COPY | cf.CF_GRAPH,
                  cf.CF_DEVICE_WAIT, cf.CF_DEVICE_WAIT | cf.CF_POISON):
        run = H.AgRun(w, data, rank, with_sink=True)
        with H.Workspace(run.desc, cf.CF_KIND_AG):
            run.run_schedule(flags)
            cf.device_status(run.cs)
        got = H.to_host_f64(run.O)
        assert not np.isnan(got).any()
        assert H.rel_err(got, ref) <= TIGHT_BF16
        # the slice forwarded at step i is the one in hand: X^r, then the received ones
        assert np.array_equal(H.to_host_f64(run.sink[0]), inputs.as_f64(data["X"], "bf16"))
        for i in range(1, w.p - 1):
            assert np.array_equal(H.to_host_f64(run.sink[i]), inputs.as_f64(data["S"][i], "bf16"))


@pytest.mark.parametrize("m", [1, 2])
def test_landing_buffer_per_hop(m):
    """cf_buffers.recv_each for the ring kinds: every hop's delivery has a buffer of its own (slot[] unused)."""
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=8, m_chunk=264, n=520, k=328)
    data = inputs.make_rs(w, salt=15)
    rank = 6
    ref = _oracle_rs(w, data, rank)
    wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=136, n=264, k=520)
    da = inputs.make_ag(wa, salt=16)
    refa = _oracle_ag(wa, da, rank)
    for flags in (0, cf.CF_SERIAL, cf.CF_POISON, cf.CF_GRAPH, cf.CF_FUSED_COPY, cf.CF_FUSED_COPY | cf.CF_GRAPH,
                  cf.CF_DEVICE_WAIT, cf.CF_DEVICE_WAIT | cf.CF_POISON):
        for sink in (False, True):
            run = H.RsRun(w, data, rank, with_sink=sink, m=m, each=True)
            run.bufs.slot[0] = run.bufs.slot[1] = None           # must not be touched
            run.O.fill_(float("nan"))
            with H.Workspace(run.desc, cf.CF_KIND_RS):
                run.run_schedule(flags)
                run.run_schedule(flags)                          # back to back: the landing buffers are reused across calls
                cf.device_status(run.cs)
            assert H.rel_err(H.to_host_f64(run.O), ref[-1]) <= TIGHT_BF16, f"flags {flags}"
            for i in range(w.p - 1):
                assert np.array_equal(H.to_host_f64(run.each[i]), data["R"][i + 1].astype(np.float64))
                if sink:
                    assert H.rel_err(H.to_host_f64(run.sink[i]), ref[i]) <= TIGHT_BF16, f"flags {flags} sink {i}"
            ag = H.AgRun(wa, da, rank, with_sink=sink, m=m, each=True)
            ag.bufs.slot[0] = ag.bufs.slot[1] = None
            with H.Workspace(ag.desc, cf.CF_KIND_AG):
                ag.run_schedule(flags)
                cf.device_status(ag.cs)
            assert H.rel_err(H.to_host_f64(ag.O), refa) <= TIGHT_BF16, f"flags {flags}"


def test_device_wait_sees_fresh_data_every_time():
    """The step kernel is already running when its delivery is written (by another kernel, possibly through
    another XCD's L2).  Each round delivers DIFFERENT data into the same buffers, with a NaN fill before
    the copy: a kernel that read through a stale cache line would produce the previous round's sum or NaN."""
    w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=4, m_chunk=256, n=264, k=520)
    wr = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=4, m_chunk=256, n=520, k=264)
    rank = 2
    runs = []
    for salt in (31, 32, 33):
        da, dr = inputs.make_ag(w, salt=salt), inputs.make_rs(wr, salt=salt)
        runs.append((da, _oracle_ag(w, da, rank), dr, _oracle_rs(wr, dr, rank)))
    ag = H.AgRun(w, runs[0][0], rank, each=True)
    rs = H.RsRun(wr, runs[0][2], rank, each=True)
    with H.Workspace(rs.desc, cf.CF_KIND_RS):
        for rnd in range(6):
            da, refa, dr, refr = runs[rnd % 3]
            for t, src in zip(ag.stage, da["S"][1:]):
                t.copy_(H.to_dev(src, w.dtype))
            for t, src in zip(rs.stage, dr["R"][1:]):
                t.copy_(H.to_dev(src, "f32"))
            ag.X.copy_(H.to_dev(da["X"], w.dtype)); ag.W.copy_(H.to_dev(da["W"], w.dtype))
            rs.A.copy_(H.to_dev(dr["A"], wr.dtype)); rs.W.copy_(H.to_dev(dr["W"], wr.dtype))
            torch.cuda.synchronize()
            ag.run_schedule(cf.CF_DEVICE_WAIT | cf.CF_POISON)
            rs.run_schedule(cf.CF_DEVICE_WAIT | cf.CF_POISON)
            cf.device_status(rs.cs)
            assert H.rel_err(H.to_host_f64(ag.O), refa) <= TIGHT_BF16, f"round {rnd}"
            assert H.rel_err(H.to_host_f64(rs.O), refr[-1]) <= TIGHT_BF16, f"round {rnd}"


@pytest.mark.parametrize("tile", [None, "256x256", "256x128", "128x128"])
@pytest.mark.parametrize("m", [1, 2])
@pytest.mark.parametrize("k", [328, 1224, 1280])      # 6 k-tiles; 20 (ragged) and 20 whole: B_in comes in under the main loop
def test_persistent_rank_step(m, tile, k):
    """CF_PERSISTENT: all steps in one launch; work items (step, tile) round robin over one chip-filling grid."""
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=8, m_chunk=264, n=520, k=k)
    data = inputs.make_rs(w, salt=19)
    rank = 5
    ref = _oracle_rs(w, data, rank)
    wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=136, n=264, k=520, out_dtype="bf16")
    da = inputs.make_ag(wa, salt=20)
    refa = _oracle_ag(wa, da, rank)
    _tile_env(tile)
    try:
        # (with CF_FUSED_COPY the reduce-scatter launch carries its deliveries itself where it brings B_in in through
        # LDS -- the 256x256 tile with the longer k ranges -- and the all-gather launch where k is whole k-tiles;
        # they have them copied in front otherwise: same results)
        # (without CF_SERIAL: groups of steps per launch, the deliveries of a group on the copy stream under the launches
        # before it)
        for flags in (cf.CF_PERSISTENT | cf.CF_SERIAL, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_GRAPH,
                      cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_POISON, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY,
                      cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY | cf.CF_GRAPH,
                      cf.CF_PERSISTENT, cf.CF_PERSISTENT | cf.CF_GRAPH, cf.CF_PERSISTENT | cf.CF_POISON):
            for layout in (cf.CF_W_KN, cf.CF_W_NK):
                run = H.RsRun(w, data, rank, layout, m=m, each=True)
                run.O.fill_(float("nan"))
                with H.Workspace(run.desc, cf.CF_KIND_RS):
                    run.run_schedule(flags)
                    for t in run.each + run.send_each:     # a step that does not wait for its delivery reads NaN
                        t.fill_(float("nan"))
                    torch.cuda.synchronize()
                    run.run_schedule(flags)
                    cf.device_status(run.cs)
                e = H.rel_err(H.to_host_f64(run.O), ref[-1])
                assert e <= TIGHT_BF16, f"flags {flags} layout {layout}: {e:.3e}"
                for i in range(w.p - 1):                   # every step's B_out (Alg. 2 "B_out <- O"), hop by hop
                    e = H.rel_err(H.to_host_f64(run.send_each[i]), ref[i])
                    assert e <= TIGHT_BF16, f"flags {flags} layout {layout} B_out of step {i}: {e:.3e}"
                    # and every delivery arrived: the landing buffer holds what the neighbour sent, bit for bit
                    assert torch.equal(run.each[i], run.stage[i]), f"flags {flags} layout {layout} delivery of hop {i + 1}"
                ag = H.AgRun(wa, da, rank, layout, m=m, each=True)
                with H.Workspace(ag.desc, cf.CF_KIND_AG):
                    ag.run_schedule(flags)
                    cf.device_status(ag.cs)
                o = H.to_host_f64(ag.O)
                assert not np.isnan(o).any(), f"flags {flags}"
                assert H.rel_err(o, refa) <= TIGHT_BF16_OUT, f"flags {flags} layout {layout}"
    finally:
        _tile_env(None)
    # compute-only on whatever the landing buffers hold after a full run; copy-only delivers everything
    run = H.RsRun(w, data, rank, each=True)
    run.run_schedule(cf.CF_PERSISTENT | cf.CF_NO_COMPUTE)
    for i in range(w.p - 1):
        assert np.array_equal(H.to_host_f64(run.each[i]), data["R"][i + 1].astype(np.float64))
    run.run_schedule(cf.CF_PERSISTENT | cf.CF_NO_COPY)
    assert H.rel_err(H.to_host_f64(run.O), ref[-1]) <= TIGHT_BF16
    # the emulated sends: every step's B_out reaches its sink after the launch
    run = H.RsRun(w, data, rank, each=True, with_sink=True)
    run.run_schedule(cf.CF_PERSISTENT | cf.CF_SERIAL)
    for i in range(w.p - 1):
        assert H.rel_err(H.to_host_f64(run.sink[i]), ref[i]) <= TIGHT_BF16, f"sink {i}"
        assert torch.equal(run.sink[i], run.send_each[i])
    ag = H.AgRun(wa, da, rank, each=True, with_sink=True)
    ag.run_schedule(cf.CF_PERSISTENT | cf.CF_SERIAL)
    for i in range(wa.p - 1):                                # Alg. 1 sends the slice in hand on
        hand = da["X"] if i == 0 else da["S"][i]
        assert np.array_equal(H.to_host_f64(ag.sink[i]), inputs.as_f64(hand, wa.dtype)), f"all-gather sink {i}"


@pytest.mark.parametrize("tile", [None, "256x256", "256x128", "128x128"])
@pytest.mark.parametrize("k", [64, 128, 1280])         # one k-tile (only the last iteration), two, twenty
def test_all_gather_carries_its_deliveries(tile, k):
    """CF_PERSISTENT | CF_FUSED_COPY, all-gather: no copy is launched; the kernel reads the gathered slices from the
    neighbours' buffers and stores every k-tile on to the landing buffer of its hop.  O against Alg. 1's result,
    the landing buffers bit for bit against what was sent -- for every tile shape, both weight orders, granularity
    1 and 2, with and without the k rotation, eagerly and as a replayed graph."""
    flags = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY
    rank = 3
    _tile_env(tile)
    try:
        for out_dtype, n in (("bf16", 520), ("f32", 264)):     # ragged tiles in M and N
            w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=264, n=n, k=k, out_dtype=out_dtype)
            data = inputs.make_ag(w, salt=61 + k)
            ref = _oracle_ag(w, data, rank)
            for layout, m, rot, extra in ((cf.CF_W_KN, 1, "1", 0), (cf.CF_W_NK, 2, "1", cf.CF_GRAPH), (cf.CF_W_KN, 2, "0", 0)):
                os.environ["COMMFUSE_K_ROTATE"] = rot
                run = H.AgRun(w, data, rank, layout, m=m, each=True)
                for rep in range(2):                       # (a graph: captured, then replayed)
                    run.O.fill_(float("nan"))
                    for t in run.each:
                        t.fill_(float("nan"))
                    run.run_schedule(flags | extra)
                    cf.device_status(run.cs)
                    o = H.to_host_f64(run.O)
                    assert not np.isnan(o).any(), f"{out_dtype} layout {layout} m {m} rot {rot} rep {rep}"
                    e = H.rel_err(o, ref)
                    assert e <= (TIGHT_BF16_OUT if out_dtype == "bf16" else TIGHT_BF16), f"{out_dtype} layout {layout} m {m}: {e:.3e}"
                    for i in range(w.p - 1):
                        assert torch.equal(run.each[i], run.stage[i]), f"{out_dtype} layout {layout} m {m} rot {rot} rep {rep}: hop {i + 1}"
        # a ragged k: the kernel cannot carry (whole k-tiles only), the deliveries are copied in front: same results
        w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=136, n=264, k=k + 8)
        data = inputs.make_ag(w, salt=62)
        run = H.AgRun(w, data, rank, each=True)
        for t in run.each:
            t.fill_(float("nan"))
        run.run_schedule(flags)
        assert H.rel_err(H.to_host_f64(run.O), _oracle_ag(w, data, rank)) <= TIGHT_BF16
        for i in range(w.p - 1):
            assert torch.equal(run.each[i], run.stage[i])
    finally:
        _tile_env(None)
        os.environ.pop("COMMFUSE_K_ROTATE", None)


@pytest.mark.parametrize("bands", ["1", "2", "4"])
@pytest.mark.parametrize("tile", ["256x256", "256x128", "128x128"])
def test_persistent_step_groups_and_column_bands(tile, bands):
    """The one-launch rank step deals its work items to the eight XCDs as 8 / NB step groups x NB bands of tile columns
    (NB = 1: whole steps per XCD).  Every NB must give every step's output and every delivery, for reduce-scatter and
    all-gather, with the deliveries copied in front and carried by the kernel, with granularity 1 and 2."""
    rank = 2
    os.environ["COMMFUSE_XCD_BANDS"] = bands
    _tile_env(tile)
    try:
        for m in (1, 2):
            w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=8, m_chunk=264, n=1000, k=1280)   # 4 (8) tile columns, the last ragged
            data = inputs.make_rs(w, salt=71)
            ref = _oracle_rs(w, data, rank)
            wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=264, n=1000, k=640, out_dtype="bf16")
            da = inputs.make_ag(wa, salt=72)
            refa = _oracle_ag(wa, da, rank)
            for flags in (PERSISTENT_SERIAL, PERSISTENT_SERIAL | cf.CF_FUSED_COPY):
                run = H.RsRun(w, data, rank, m=m, each=True)
                for t in run.each + run.send_each + [run.O]:
                    t.fill_(float("nan"))
                run.run_schedule(flags)
                for i in range(w.p):
                    got = H.to_host_f64(run.send_each[i] if i < w.p - 1 else run.O)
                    e = H.rel_err(got, ref[i])
                    assert e <= TIGHT_BF16, f"m {m} flags {flags} step {i}: {e:.3e}"
                ag = H.AgRun(wa, da, rank, m=m, each=True)
                for t in ag.each:
                    t.fill_(float("nan"))
                ag.run_schedule(flags)
                o = H.to_host_f64(ag.O)
                assert not np.isnan(o).any() and H.rel_err(o, refa) <= TIGHT_BF16_OUT, f"m {m} flags {flags}"
                for i in range(w.p - 1):
                    assert torch.equal(run.each[i], run.stage[i]) and torch.equal(ag.each[i], ag.stage[i]), f"m {m} flags {flags} hop {i + 1}"
    finally:
        os.environ.pop("COMMFUSE_XCD_BANDS", None)
        _tile_env(None)


@pytest.mark.parametrize("k", [64, 192, 456, 1032])        # one k-tile, three, a ragged eighth, seventeen with a ragged tail
@pytest.mark.parametrize("mfma16", ["1", "0"])
def test_persistent_mfma16_main_loop(k, mfma16):
    """The 256x256 tile of the one-launch rank step runs its main loop on 16x16x32 MFMAs where the steps are whole
    tiles and B_in is added in the epilogue (COMMFUSE_MFMA16 = 0 keeps the 32x32x16 loop).  The accumulator
    layout, the fragment reads and the order of the [k x n] weight tile in LDS all differ between the two, so both are
    compared with the oracle here: reduce-scatter (every step's B_out and O), all-gather with fp32 and bf16 output,
    both weight orders, granularity 1 and 2, the deliveries copied in front and carried by the kernel."""
    rank = 5
    os.environ["COMMFUSE_MFMA16"] = mfma16
    _tile_env("256x256")
    try:
        for m, m_chunk, n in ((1, 256, 512), (2, 512, 768)):
            w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=8, m_chunk=m_chunk, n=n, k=k)
            data = inputs.make_rs(w, salt=81 + k)
            ref = _oracle_rs(w, data, rank)
            # (CF_FUSED_COPY: these k ranges are too short for B_in to be streamed, so the epilogue reads it from the
            # neighbour's buffer and the work item lands it by a copy beside its GEMM)
            for layout, flags in ((cf.CF_W_KN, PERSISTENT_SERIAL), (cf.CF_W_NK, PERSISTENT_SERIAL),
                                  (cf.CF_W_KN, PERSISTENT_SERIAL | cf.CF_FUSED_COPY), (cf.CF_W_NK, PERSISTENT_SERIAL | cf.CF_FUSED_COPY)):
                run = H.RsRun(w, data, rank, layout, m=m, each=True)
                for t in run.each + run.send_each + [run.O]:
                    t.fill_(float("nan"))
                run.run_schedule(flags)
                cf.device_status(run.cs)
                for i in range(w.p):
                    got = H.to_host_f64(run.send_each[i] if i < w.p - 1 else run.O)
                    e = H.rel_err(got, ref[i])
                    assert e <= TIGHT_BF16, f"rs m {m} layout {layout} flags {flags} step {i}: {e:.3e}"
                for i in range(w.p - 1):
                    assert torch.equal(run.each[i], run.stage[i]), f"rs m {m} layout {layout} flags {flags}: hop {i + 1}"
            for out_dtype in ("bf16", "f32"):
                wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=m_chunk, n=n, k=k, out_dtype=out_dtype)
                da = inputs.make_ag(wa, salt=82 + k)
                refa = _oracle_ag(wa, da, rank)
                for layout, flags in ((cf.CF_W_KN, PERSISTENT_SERIAL), (cf.CF_W_NK, PERSISTENT_SERIAL | cf.CF_FUSED_COPY),
                                      (cf.CF_W_KN, PERSISTENT_SERIAL | cf.CF_FUSED_COPY)):
                    ag = H.AgRun(wa, da, rank, layout, m=m, each=True)
                    ag.O.fill_(float("nan"))
                    for t in ag.each:
                        t.fill_(float("nan"))
                    ag.run_schedule(flags)
                    cf.device_status(ag.cs)
                    o = H.to_host_f64(ag.O)
                    assert not np.isnan(o).any(), f"ag {out_dtype} m {m} layout {layout} flags {flags}"
                    e = H.rel_err(o, refa)
                    assert e <= (TIGHT_BF16_OUT if out_dtype == "bf16" else TIGHT_BF16), f"ag {out_dtype} m {m} layout {layout} flags {flags}: {e:.3e}"
                    for i in range(wa.p - 1):
                        assert torch.equal(ag.each[i], ag.stage[i]), f"ag {out_dtype} m {m} layout {layout} flags {flags}: hop {i + 1}"
    finally:
        os.environ.pop("COMMFUSE_MFMA16", None)
        _tile_env(None)


@pytest.mark.parametrize("kind", ["rs", "ag"])
def test_persistent_k_rotation(kind):
    """The persistent launch lets the workgroups of XCD x start their k loops x/8 of the way into the k range
    (wrapping around; the ragged last k-tile then falls in mid-loop).  With the rotation and without it the
    rank step must match the oracle; the two differ at most in last bits (another order of the same sum)."""
    rank = 6
    flags = cf.CF_PERSISTENT | cf.CF_SERIAL
    outs = {}
    try:
        for rot in ("1", "0"):
            os.environ["COMMFUSE_K_ROTATE"] = rot
            if kind == "rs":
                w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=8, m_chunk=264, n=520, k=1096)
                data = inputs.make_rs(w, salt=43)
                ref = _oracle_rs(w, data, rank)[-1]
                run = H.RsRun(w, data, rank, each=True)
                tol = TIGHT_BF16
            else:
                w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=8, m_chunk=136, n=264, k=1096)
                data = inputs.make_ag(w, salt=44)
                ref = _oracle_ag(w, data, rank)
                run = H.AgRun(w, data, rank, each=True)
                tol = TIGHT_BF16
            run.O.fill_(float("nan"))
            run.run_schedule(flags)
            outs[rot] = H.to_host_f64(run.O)
            e = H.rel_err(outs[rot], ref)
            assert e <= tol, f"rotate {rot}: {e:.3e}"
        assert H.rel_err(outs["1"], outs["0"]) <= 1e-5
    finally:
        os.environ.pop("COMMFUSE_K_ROTATE", None)


def _padded(t, rows, cols, ld, fill):
    """Device copy of a [rows x cols] tensor with row stride ld; the padding holds `fill`."""
    o = torch.full((rows, ld), fill, dtype=t.dtype, device=H.DEV)
    o[:, :cols] = t.reshape(rows, cols)
    return o


@pytest.mark.parametrize("m", [1, 2])
def test_run_schedule_padded_row_strides(m):
    """Slices and partial sums with padded rows (lda > k, ldw > n, ldo > n): every buffer of the schedule
    keeps the descriptor's strides, a delivery moves a row block with its padding; what sits in the padding
    (huge values here) reaches no result."""
    rank = 2
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=4, m_chunk=264, n=520, k=328)
    data = inputs.make_rs(w, salt=23)
    ref = _oracle_rs(w, data, rank)
    lda, ldw, ldo = w.k + 8, w.n + 24, w.n + 16
    base = H.RsRun(w, data, rank, m=m, each=True)
    pad32 = lambda t: _padded(t, w.m_chunk, w.n, ldo, 1e30)
    mk32 = lambda: torch.full((w.m_chunk, ldo), 1e30, dtype=torch.float32, device=H.DEV)
    A = _padded(base.A, w.p * w.m_chunk, w.k, lda, 1e30)
    W = _padded(base.W, w.k, w.n, ldw, 1e30)
    stage = [pad32(t) for t in base.stage]
    desc = cf.layer_desc(w.p, rank, w.m_chunk, w.n, w.k, w.dtype, w.out_dtype, cf.CF_W_KN, lda=lda, ldw=ldw, ldo=ldo, m=m)
    for flags, each in ((0, False), (cf.CF_SERIAL, False), (cf.CF_GRAPH, True), (cf.CF_FUSED_COPY, False),
                        (cf.CF_DEVICE_WAIT | cf.CF_POISON, True), (cf.CF_PERSISTENT | cf.CF_SERIAL, True)):
        O = mk32()
        keep = ([mk32(), mk32()], [mk32(), mk32()], [mk32() for _ in range(w.p - 1)], [mk32() for _ in range(w.p - 1)])
        bufs = cf.make_buffers(A, W, O, stage, keep[0], keep[1], None, keep[2] if each else None, keep[3] if each else None)
        with H.Workspace(desc, cf.CF_KIND_RS):
            cf.run_schedule(desc, cf.CF_KIND_RS, bufs, base.cs, base.xs, flags)
            base.cs.synchronize()
            cf.device_status(base.cs)
        got = H.to_host_f64(O)
        assert H.rel_err(got[:, :w.n], ref[-1]) <= TIGHT_BF16, f"flags {flags}"
        assert np.all(got[:, w.n:] == np.float64(np.float32(1e30))), f"flags {flags}: padding of O was written"
        if each:                                             # every B_out keeps the stride too
            for i in range(w.p - 1):
                got = H.to_host_f64(keep[3][i])
                assert H.rel_err(got[:, :w.n], ref[i]) <= TIGHT_BF16, f"flags {flags} B_out {i}"
                assert np.all(got[:, w.n:] == np.float64(np.float32(1e30))), f"flags {flags}: padding of B_out {i} was written"
    wa = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=4, m_chunk=136, n=264, k=520, out_dtype="bf16")
    da = inputs.make_ag(wa, salt=24)
    refa = _oracle_ag(wa, da, rank)
    lda, ldw, ldo = wa.k + 8, wa.n + 8, wa.n + 24
    ab = H.AgRun(wa, da, rank, m=m, each=True)
    pad16 = lambda t: _padded(t, wa.m_chunk, wa.k, lda, 1e30)
    mk16 = lambda: torch.full((wa.m_chunk, lda), 1e30, dtype=torch.bfloat16, device=H.DEV)
    W = _padded(ab.W, wa.k, wa.n, ldw, 1e30)
    desc = cf.layer_desc(wa.p, rank, wa.m_chunk, wa.n, wa.k, wa.dtype, wa.out_dtype, cf.CF_W_KN, lda=lda, ldw=ldw, ldo=ldo, m=m)
    for flags, each in ((0, False), (cf.CF_SERIAL | cf.CF_GRAPH, False), (cf.CF_FUSED_COPY, True),
                        (cf.CF_DEVICE_WAIT | cf.CF_POISON, True), (cf.CF_PERSISTENT | cf.CF_SERIAL, True)):
        O = torch.full((wa.p * wa.m_chunk, ldo), 3.0, dtype=torch.bfloat16, device=H.DEV)
        keep = (pad16(ab.X), [pad16(t) for t in ab.stage], [mk16(), mk16()], [mk16() for _ in range(wa.p - 1)])
        bufs = cf.make_buffers(keep[0], W, O, keep[1], keep[2], (None, None), None, keep[3] if each else None)
        with H.Workspace(desc, cf.CF_KIND_AG):
            cf.run_schedule(desc, cf.CF_KIND_AG, bufs, ab.cs, ab.xs, flags)
            ab.cs.synchronize()
            cf.device_status(ab.cs)
        got = H.to_host_f64(O)
        assert H.rel_err(got[:, :wa.n], refa) <= TIGHT_BF16_OUT, f"flags {flags}"
        assert np.all(got[:, wa.n:] == 3.0), f"flags {flags}: padding of O was written"


def test_persistent_needs_what_it_needs():
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=4, m_chunk=64, n=64, k=64)
    data = inputs.make_rs(w)
    PS = cf.CF_PERSISTENT | cf.CF_SERIAL
    for kw, flags, status in (({}, PS, cf.CF_ERR_INVALID_ARG),                                     # no recv_each
                              ({"each": True}, PS | cf.CF_DEVICE_WAIT, cf.CF_ERR_UNSUPPORTED)):
        run = H.RsRun(w, data, 0, **kw)
        with pytest.raises(cf.CommFuseError) as ei:
            run.run_schedule(flags)
        assert ei.value.status == status, (kw, flags)
    wd = inputs.scaled(inputs.CONFIGS["c5_dp"], p=4, m_chunk=4096)
    dp = H.DpRun(wd, inputs.make_dp(wd), 0, each=True)
    with pytest.raises(cf.CommFuseError) as ei:                  # two streams: the reduce-scatter and all-gather kinds only
        dp.run_schedule(cf.CF_PERSISTENT)
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED
    run = H.RsRun(w, data, 0, each=True)                                                           # no send_each
    run.bufs = cf.make_buffers(run.A, run.W, run.O, run.stage, run.slot, run.send, None, run.each)
    with pytest.raises(cf.CommFuseError) as ei:
        run.run_schedule(PS)
    assert ei.value.status == cf.CF_ERR_INVALID_ARG
    wf = inputs.scaled(inputs.CONFIGS["c1_rs_f32"], p=2)
    run = H.RsRun(wf, inputs.make_rs(wf), 0, each=True)
    with pytest.raises(cf.CommFuseError) as ei:
        run.run_schedule(cf.CF_PERSISTENT | cf.CF_SERIAL)                                          # fp32 operands
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED


def test_device_wait_cannot_be_captured():
    """A graph holds no edge from a flag write to the kernel that polls the flag: the combination is refused."""
    w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=2, m_chunk=64, n=64, k=64)
    run = H.AgRun(w, inputs.make_ag(w), 0)
    with H.Workspace(run.desc, cf.CF_KIND_AG):
        with pytest.raises(cf.CommFuseError) as ei:
            run.run_schedule(cf.CF_DEVICE_WAIT | cf.CF_GRAPH)
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED


def test_device_wait_times_out_instead_of_hanging():
    """No delivery is ever made (CF_NO_COPY), so no flag is raised: with a tiny spin limit, forced from
    the host, every kernel gives up its wait, finishes normally, and the status call reports it."""
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=3, m_chunk=128, n=256, k=128)
    data = inputs.make_rs(w, salt=11)
    run = H.RsRun(w, data, 0)
    os.environ["COMMFUSE_SPIN_LIMIT"] = "20"
    try:
        with H.Workspace(run.desc, cf.CF_KIND_RS):
            cf.device_status(run.cs)                       # clean before
            run.run_schedule(cf.CF_DEVICE_WAIT | cf.CF_NO_COPY)
            with pytest.raises(cf.CommFuseError) as e:
                cf.device_status(run.cs)
            assert "gave up waiting" in str(e.value)
            cf.device_status(run.cs)                       # the status word was cleared
            # and a normal run right after is correct again
            os.environ.pop("COMMFUSE_SPIN_LIMIT", None)
            run.run_schedule(cf.CF_DEVICE_WAIT)
            cf.device_status(run.cs)
            ref = _oracle_rs(w, data, 0)
            assert H.rel_err(H.to_host_f64(run.O), ref[-1]) <= TIGHT_BF16
    finally:
        os.environ.pop("COMMFUSE_SPIN_LIMIT", None)


def test_graph_replays_match_eager():
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=4, m_chunk=256, n=512, k=192)
    data = inputs.make_rs(w, salt=7)
    ref = _oracle_rs(w, data, 1)
    run = H.RsRun(w, data, 1, with_sink=True)
    run.run_schedule(0)
    eager = H.to_host_f64(run.O)
    for rep in range(4):
        run.O.fill_(float("nan"))
        for s in run.sink:
            s.fill_(float("nan"))
        scratch = torch.randn(1024, device=H.DEV).sum().item()      # eager work between replays
        run.run_schedule(cf.CF_GRAPH)
        assert np.array_equal(H.to_host_f64(run.O), eager), f"replay {rep}"
        for i in range(w.p - 1):
            assert H.rel_err(H.to_host_f64(run.sink[i]), ref[i]) <= TIGHT_BF16
    cf.destroy_cache()


# ----------------------------------------------------------------------------
# full benchmark sizes, launched as the benchmark launches them, every element of
# every step's output compared with the oracle (computed once per configuration)
# ----------------------------------------------------------------------------

PERSISTENT_SERIAL = cf.CF_PERSISTENT | cf.CF_SERIAL       # the mode the benchmark's best times come from

_full_refs = {}


def _full_ref(name, rank):
    """Oracle outputs of every step of a full-size configuration (a few seconds each, kept for the module)."""
    key = (name, rank)
    if key not in _full_refs:
        w = inputs.CONFIGS[name]
        if w.kind == "rs":
            data = inputs.make_rs(w)
            _full_refs[key] = (data, _oracle_rs(w, data, rank))
        else:
            data = inputs.make_ag(w)
            _full_refs[key] = (data, _oracle_ag(w, data, rank))
    return _full_refs[key]


@pytest.mark.parametrize("flags", [0, cf.CF_FUSED_COPY | cf.CF_GRAPH, cf.CF_GRAPH, cf.CF_DEVICE_WAIT, PERSISTENT_SERIAL,
                                   PERSISTENT_SERIAL | cf.CF_GRAPH, PERSISTENT_SERIAL | cf.CF_FUSED_COPY, cf.CF_PERSISTENT])
@pytest.mark.parametrize("name", ["c2_rs_7b", "c4_rs_70b_down"])
def test_full_size_rs(name, flags):
    w = inputs.CONFIGS[name]
    rank = 0
    data, ref = _full_ref(name, rank)
    persistent = bool(flags & cf.CF_PERSISTENT)      # every step's B_out stays in a buffer of its own there
    run = H.RsRun(w, data, rank, each=True) if persistent else H.RsRun(w, data, rank, with_sink=True)
    for t in (run.send_each + run.each if persistent else run.sink) + [run.O]:
        t.fill_(float("nan"))
    with H.Workspace(run.desc, cf.CF_KIND_RS):          # as the benchmark runs it
        run.run_schedule(flags)                         # with CF_FUSED_COPY the kernel carries its deliveries at both shapes
        cf.device_status(run.cs)
    if persistent:                                   # every delivery landed (copied in front, or carried by the kernel)
        for i in range(w.p - 1):
            assert torch.equal(run.each[i], run.stage[i]), f"delivery of hop {i + 1}"
    for i in range(w.p):
        got = H.to_host_f64((run.send_each if persistent else run.sink)[i] if i < w.p - 1 else run.O)
        assert not np.isnan(got).any(), f"step {i}"
        e = H.rel_err(got, ref[i])                   # all m_chunk x n elements
        assert e <= TOL_BF16 and e <= TIGHT_BF16, f"step {i}: {e:.3e}"


@pytest.mark.parametrize("flags", [0, cf.CF_FUSED_COPY | cf.CF_GRAPH, cf.CF_GRAPH, cf.CF_DEVICE_WAIT, PERSISTENT_SERIAL,
                                   PERSISTENT_SERIAL | cf.CF_GRAPH, PERSISTENT_SERIAL | cf.CF_FUSED_COPY, cf.CF_PERSISTENT])
@pytest.mark.parametrize("name", ["c3_ag_7b", "c4_ag_70b_up"])
def test_full_size_ag(name, flags):
    w = inputs.CONFIGS[name]
    rank = 0
    data, ref = _full_ref(name, rank)
    persistent = bool(flags & cf.CF_PERSISTENT)
    run = H.AgRun(w, data, rank, each=persistent)
    for t in run.each or []:
        t.fill_(float("nan"))
    with H.Workspace(run.desc, cf.CF_KIND_AG):          # as the benchmark runs it (the 7B shape splits k)
        run.run_schedule(flags)                         # with CF_FUSED_COPY the one launch carries its deliveries
        cf.device_status(run.cs)
    if persistent:                                   # every delivery landed (copied in front, or carried by the kernel)
        for i in range(w.p - 1):
            assert torch.equal(run.each[i], run.stage[i]), f"delivery of hop {i + 1}"
    got = H.to_host_f64(run.O)
    assert not np.isnan(got).any()
    gate, tight = _tols(w)
    for i in range(w.p):                             # slice by slice, so that a small slice cannot hide
        l = (rank - i) % w.p
        rows = slice(l * w.m_chunk, (l + 1) * w.m_chunk)
        e = H.rel_err(got[rows], ref[rows])
        assert e <= gate and e <= tight, f"step {i}: {e:.3e}"


@pytest.mark.parametrize("flags", [0, PERSISTENT_SERIAL, PERSISTENT_SERIAL | cf.CF_FUSED_COPY, cf.CF_PERSISTENT])
def test_full_size_pair_70b(flags):
    """AG-GEMM (up) writes H in bf16; GEMM-RS (down) consumes it.  No activation between.  Set up as the
    benchmark sets it up (a landing buffer per hop, a B_out buffer per step, one compute stream for both
    layers); every element of H, of every B_out and of O^r is compared."""
    up, dn = inputs.CONFIGS["c4_ag_70b_up"], inputs.CONFIGS["c4_rs_70b_down"]
    rank = 0
    dup, _ = _full_ref("c4_ag_70b_up", rank)
    ddn, _ = _full_ref("c4_rs_70b_down", rank)
    ag = H.AgRun(up, dup, rank, each=True)
    rs = H.RsRun(dn, ddn, rank, each=True)
    rs.A = ag.O                                            # hand H over on the device
    rs.bufs = cf.make_buffers(rs.A, rs.W, rs.O, rs.stage, rs.slot, rs.send, None, rs.each, rs.send_each)
    rs.cs, rs.xs = ag.cs, ag.xs
    with H.Workspace(rs.desc, cf.CF_KIND_RS):
        for _ in range(2):                                 # back to back, as in the timed loop
            for t in ag.each + rs.each + rs.send_each:     # a step that does not wait for its delivery reads NaN
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            cf.run_schedule(ag.desc, cf.CF_KIND_AG, ag.bufs, ag.cs, ag.xs, flags)
            cf.run_schedule(rs.desc, cf.CF_KIND_RS, rs.bufs, rs.cs, rs.xs, flags)
        rs.cs.synchronize()
        cf.device_status(rs.cs)
    if flags & cf.CF_PERSISTENT:
        for i in range(up.p - 1):
            assert torch.equal(ag.each[i], ag.stage[i]) and torch.equal(rs.each[i], rs.stage[i]), f"delivery of hop {i + 1}"
    # oracle: H = bf16(AG(X) W_up) (Alg. 1), then Alg. 2 on A = H
    H64 = oracle.round_to_bf16(_full_ref("c4_ag_70b_up", rank)[1])
    e = H.rel_err(H.to_host_f64(ag.O), H64)
    # (the reference is itself rounded to bf16 here, because the down-projection consumes it: where the fp32 sum lies
    # next to a rounding boundary the two roundings differ by one ulp of the element, which is at most 2^-7 of it)
    assert e <= 2 * TIGHT_BF16_OUT, f"H: {e:.3e}"
    ref = oracle.rs_rank_steps(H64, inputs.as_f64(ddn["W"], "bf16"),
                               [None] + [r.astype(np.float64) for r in ddn["R"][1:]], dn.p, rank)
    for i in range(dn.p):
        got = H.to_host_f64(rs.send_each[i] if i < dn.p - 1 else rs.O)
        e = H.rel_err(got, ref[i])
        # (the few elements of H whose bf16 rounding flips against the fp64 oracle move O by far less than this)
        assert e <= TOL_BF16 and e <= 1e-3, f"step {i}: {e:.3e}"


@pytest.mark.parametrize("flags", [0, PERSISTENT_SERIAL, PERSISTENT_SERIAL | cf.CF_FUSED_COPY])
def test_full_size_dp(flags):
    w = inputs.CONFIGS["c5_dp"]
    data = inputs.make_dp(w)
    rank = 0
    run = H.DpRun(w, data, rank, each=bool(flags & cf.CF_PERSISTENT))
    if run.each:
        for t in run.each:
            t.fill_(float("nan"))
        torch.cuda.synchronize()                     # the fills run on another stream than the schedule
    run.run_schedule(flags)
    if run.each:                                     # copied in front, or landed by the add kernels themselves
        for i in range(w.p - 1):
            assert torch.equal(run.each[i], run.stage[i]), f"delivery of hop {i + 1}"
    c = w.m_chunk
    touched = {(rank - i - 1) % w.p: i for i in range(1, w.p)}
    for l in range(w.p):
        got = run.bucket[l * c:(l + 1) * c].cpu().numpy()
        loc = data["bucket"][l * c:(l + 1) * c]
        if l in touched:
            idx = np.unique(np.concatenate([np.arange(0, 4096), np.arange(c - 4096, c), np.arange(0, c, 997)]))
            ref = oracle.add(data["R"][touched[l]][idx].astype(np.float64), loc[idx].astype(np.float64))
            assert np.array_equal(got[idx].astype(np.float64), ref.astype(np.float32).astype(np.float64)), f"slice {l}"
        else:
            assert np.array_equal(got, loc), f"slice {l} must be untouched"


# ----------------------------------------------------------------------------
# degenerate sizes
# ----------------------------------------------------------------------------

def test_empty_and_k_zero():
    d = cf.layer_desc(2, 0, 0, 64, 64)
    A = torch.zeros(16, dtype=torch.bfloat16, device=H.DEV)
    out = torch.zeros(16, dtype=torch.float32, device=H.DEV)
    cf.rs_step(d, 0, A, A, None, out, None)                       # no rows: nothing to do
    cf.ag_step(cf.layer_desc(2, 0, 8, 0, 64), 0, A, A, out, None)  # no columns
    # k = 0: the product is zero, the step reduces to out = recv
    mc, n = 40, 72
    recv = torch.randn(mc, n, device=H.DEV)
    out = torch.full((mc, n), float("nan"), device=H.DEV)
    cf.rs_step(cf.layer_desc(2, 0, mc, n, 0), 1, A, A, recv, out, None)
    torch.cuda.synchronize()
    assert torch.equal(out, recv)

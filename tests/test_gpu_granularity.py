"""Slicing granularity m > 1 (Sec. 3.2) on the HIP path against the CPU oracle, through the
C ABI.  Needs an MI355X: run with ``-m gpu``.  Tolerances as in test_gpu_parity.py.

Cutting a slice into m row blocks changes no value: besides the oracle comparison, the
results are compared bit for bit with the m = 1 run of the same kernels where the tile
choice is the same (forced with COMMFUSE_TILE).
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
TIGHT_BF16 = 1e-4
TIGHT_BF16_OUT = 2.0 ** -8


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(cf.LIB_PATH), "libcommfuse.so must be built in-tree before the GPU run"
    cf.load()
    yield
    torch.cuda.synchronize()


def _rs_ref(w, data, rank, m):
    return oracle.rs_rank_steps_m(inputs.as_f64(data["A"], w.dtype), inputs.as_f64(data["W"], w.dtype),
                                  [None] + [r.astype(np.float64) for r in data["R"][1:]], w.p, rank, m)


def _ag_ref(w, data, rank, m):
    S = [None] + [inputs.as_f64(s, w.dtype) for s in data["S"][1:]]
    return oracle.ag_rank_m(inputs.as_f64(data["X"], w.dtype), S, inputs.as_f64(data["W"], w.dtype), w.p, rank, m)


def _status_ok(run, flags):
    try:
        cf.device_status(run.cs)
    except cf.CommFuseError as e:
        raise AssertionError(f"flags {flags}: {e}") from e


RS_CASES = [
    # (p, m, m_chunk, n, k)
    (4, 2, 144, 264, 168),
    (3, 3, 201, 136, 1376),     # odd p, sub-slices of 67 rows (ragged against every tile)
    (8, 2, 528, 392, 200),
    (1, 4, 160, 72, 64),        # p = 1: m plain GEMMs
    (2, 8, 64, 520, 96),        # sub-slices of 8 rows
]

SCHED_FLAGS = (0, cf.CF_SERIAL, cf.CF_POISON, cf.CF_GRAPH, cf.CF_FUSED_COPY, cf.CF_FUSED_COPY | cf.CF_GRAPH,
               cf.CF_DEVICE_WAIT)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("case", RS_CASES)
def test_rs_granularity(case, layout, dtype):
    p, m, mc, n, k = case
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k, dtype=dtype)
    data = inputs.make_rs(w, salt=21)
    rank = p // 2
    ref = _rs_ref(w, data, rank, m)
    tol = TOL_F32 if dtype == "f32" else TIGHT_BF16
    ms = mc // m
    run = H.RsRun(w, data, rank, layout, with_sink=True, m=m)
    outs = run.run_steps()
    assert len(outs) == m * p
    for j in range(m * p):
        assert outs[j].shape == (ms, n)
        e = H.rel_err(outs[j], ref[j])
        assert e <= tol, f"sub-step {j}: {e:.3e}"
    final = np.concatenate(outs[(p - 1) * m:], axis=0)
    flag_set = SCHED_FLAGS if dtype == "bf16" else SCHED_FLAGS[:4]
    with H.Workspace(run.desc, cf.CF_KIND_RS):
        for flags in flag_set:
            run.O.fill_(float("nan"))
            for s in run.sink:
                s.fill_(float("nan"))
            run.run_schedule(flags)
            _status_ok(run, flags)
            assert H.rel_err(H.to_host_f64(run.O), np.concatenate(ref[(p - 1) * m:], axis=0)) <= tol, f"flags {flags}"
            for i in range(p - 1):
                want = np.concatenate(ref[i * m:(i + 1) * m], axis=0)
                assert H.rel_err(H.to_host_f64(run.sink[i]), want) <= tol, f"flags {flags} hop {i}"
    assert final.shape == (mc, n)


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", [cf.CF_W_KN, cf.CF_W_NK])
@pytest.mark.parametrize("case", [(4, 2, 144, 264, 168), (3, 3, 201, 136, 520), (8, 2, 272, 136, 328), (1, 4, 160, 72, 64)])
def test_ag_granularity(case, layout, out_dtype):
    p, m, mc, n, k = case
    w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], p=p, m_chunk=mc, n=n, k=k, out_dtype=out_dtype)
    data = inputs.make_ag(w, salt=22)
    rank = p - 1
    ref = _ag_ref(w, data, rank, m)
    tol = TIGHT_BF16 if out_dtype == "f32" else TIGHT_BF16_OUT
    run = H.AgRun(w, data, rank, layout, with_sink=True, m=m)
    got = run.run_steps()
    assert not np.isnan(got).any()
    assert H.rel_err(got, ref) <= tol
    with H.Workspace(run.desc, cf.CF_KIND_AG):
        for flags in SCHED_FLAGS:
            run.O.fill_(float("nan"))
            for s in run.sink:
                s.fill_(float("nan"))
            run.run_schedule(flags)
            _status_ok(run, flags)
            o = H.to_host_f64(run.O)
            assert not np.isnan(o).any(), f"flags {flags}"
            assert H.rel_err(o, ref) <= tol, f"flags {flags}"
            for i in range(p - 1):      # what is sent on at hop i is the slice in hand: own first, then hop i's delivery
                want = data["X"] if i == 0 else data["S"][i]
                assert np.array_equal(H.to_host_f64(run.sink[i]), inputs.as_f64(want, w.dtype)), f"flags {flags} hop {i}"


def test_granularity_changes_no_bit():
    """Same tile shape forced for m = 1 and m = 2: every output row is computed by the same
    instruction sequence, so the results agree bit for bit."""
    p, mc, n, k = 4, 512, 264, 328
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=23)
    os.environ["COMMFUSE_TILE"] = "128x128"
    os.environ["COMMFUSE_SPLITK"] = "1"
    try:
        base = H.RsRun(w, data, 1).run_steps()
        fine = H.RsRun(w, data, 1, m=2).run_steps()
    finally:
        os.environ.pop("COMMFUSE_TILE", None)
        os.environ.pop("COMMFUSE_SPLITK", None)
    for i in range(p):
        assert np.array_equal(np.concatenate(fine[2 * i:2 * i + 2], axis=0), base[i]), f"hop {i}"


@pytest.mark.parametrize("p,m,c", [(8, 2, 1_000_004), (4, 4, 4096), (3, 2, 10), (1, 2, 64)])
def test_dp_granularity(p, m, c):
    w = inputs.scaled(inputs.CONFIGS["c5_dp"], p=p, m_chunk=c)
    data = inputs.make_dp(w, salt=24)
    rank = 0
    ref = oracle.dp_rank_m(data["bucket"], data["R"], p, rank, m)
    want32 = ref.astype(np.float32).astype(np.float64)      # one fp32 addition per element
    run = H.DpRun(w, data, rank, with_sink=True, m=m)
    for flags in (0, cf.CF_SERIAL, cf.CF_GRAPH):
        run.bucket.copy_(H.to_dev(data["bucket"], "f32"))
        run.run_schedule(flags)
        assert np.array_equal(H.to_host_f64(run.bucket), want32), f"flags {flags}"
        for i in range(p - 1):
            l = (rank - i - 1) % p
            assert np.array_equal(H.to_host_f64(run.sink[i]), want32[l * c:(l + 1) * c]), f"flags {flags} hop {i}"
    for flags in (cf.CF_PERSISTENT | cf.CF_SERIAL, cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY):
        pers = H.DpRun(w, data, rank, m=m, each=True)             # the m sub-slices of a hop stacked in its landing buffer
        for t in pers.each:
            t.fill_(float("nan"))
        torch.cuda.synchronize()                     # the fills run on another stream than the schedule
        pers.run_schedule(flags)
        assert np.array_equal(H.to_host_f64(pers.bucket), want32), f"flags {flags}"
        for i in range(p - 1):                       # copied in front, or landed by the add kernels themselves
            assert torch.equal(pers.each[i], pers.stage[i]), f"flags {flags}: delivery of hop {i + 1}"


def test_granularity_bad_arguments():
    t = torch.zeros(4096, dtype=torch.float32, device=H.DEV)
    with pytest.raises(cf.CommFuseError) as ei:
        cf.rs_step(cf.layer_desc(2, 0, 30, 64, 64, m=4), 0, t, t, None, t, None)      # m does not divide m_chunk
    assert ei.value.status == cf.CF_ERR_INVALID_ARG
    d = cf.layer_desc(2, 0, 32, 64, 64, m=2)
    with pytest.raises(cf.CommFuseError):
        cf.rs_step(d, 4, t, t, t, t, None)                                            # sub-steps are 0 .. m*p-1
    with pytest.raises(cf.CommFuseError) as ei:
        cf.rs_step(d, 1, t, t, t[:1024], t[1024:2048], None)                          # first hop receives nothing
    assert ei.value.status == cf.CF_ERR_NULL_PTR
    with pytest.raises(cf.CommFuseError) as ei:
        cf.rs_pair_step(d, 0, t, t, None, None, t, None)                              # pairwise kinds need m = 1
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED
    assert [cf.subslice_index(cf.CF_KIND_RS, 4, 2, 1, j) for j in range(8)] == [0, 1, 6, 7, 4, 5, 2, 3]
    assert [cf.subslice_index(cf.CF_KIND_AG, 4, 2, 1, j) for j in range(8)] == [2, 3, 0, 1, 6, 7, 4, 5]

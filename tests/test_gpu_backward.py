"""Backward pass of the two TPSP layers on the HIP path against the CPU oracle, through the C ABI.
Needs an MI355X: run with ``-m gpu``.

  * data gradients: the forward entry points with the weight pointer unchanged and the other
    w_layout (W^r stored [k x n] read as its transpose);
  * weight gradients: commfuse_wgrad_step / the CF_KIND_WGRAD_* schedules.
Tolerances as in test_gpu_parity.py (bf16 operands, fp32 accumulation: 1e-2 stated, 1e-4 asserted;
the weight gradient adds one fp32 rounding per step); integer-valued inputs bit for bit.
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

TOL_BF16 = 1e-2
TIGHT_BF16 = 1e-4


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the GPU"
    assert os.path.exists(cf.LIB_PATH), "libcommfuse.so must be built in-tree before the GPU run"
    cf.load()
    yield
    torch.cuda.synchronize()


def _bf16(rng, shape, sigma=1.0, integer=False):
    a = inputs.small_int_like(shape, rng) if integer else (rng.standard_normal(shape).astype(np.float32) * sigma)
    bits = inputs.f32_to_bf16_bits(a)
    return bits, inputs.bf16_bits_to_f32(bits).astype(np.float64)


@pytest.mark.parametrize("integer", [False, True])
@pytest.mark.parametrize("shape", [(4, 72, 136, 200), (2, 256, 264, 64), (3, 40, 72, 328)])
def test_dgrad_of_the_all_gather_layer_is_an_rs_step_with_the_transposed_weight(shape, integer):
    """dX^r = RS_r(G^r (W^r)^T): Alg. 2 on A = G^r; W^r [k x n] is handed over as is and read as [n' x k']."""
    p, mc, n, k = shape                              # forward layer: X [mc x k], W [k x n], Y [p*mc x n]
    rng = np.random.default_rng(90 + p)
    Wb, W = _bf16(rng, (k, n), 0.05, integer)
    Gb, G = _bf16(rng, (p * mc, n), 1.0, integer)
    R = [None] + [(inputs.small_int_like((mc, k), rng, -50, 50) if integer else
                   rng.standard_normal((mc, k)).astype(np.float32)) for _ in range(p - 1)]
    rank = p - 1
    ref = oracle.rs_rank_steps(G, np.ascontiguousarray(W.T), [None] + [r.astype(np.float64) for r in R[1:]], p, rank)
    desc = cf.layer_desc(p, rank, mc, k, n, "bf16", "f32", cf.CF_W_NK)    # n' = k, k' = n
    Gd, Wd = H.to_dev(Gb, "bf16"), H.to_dev(Wb, "bf16")
    for i in range(p):
        out = torch.full((mc, k), float("nan"), dtype=torch.float32, device=H.DEV)
        recv = H.to_dev(R[i], "f32") if i > 0 else None
        cf.rs_step(desc, i, Gd, Wd, recv, out, None)
        torch.cuda.synchronize()
        got = H.to_host_f64(out)
        if integer:
            assert np.array_equal(got, ref[i]), f"step {i}"
        else:
            assert H.rel_err(got, ref[i]) <= TIGHT_BF16, f"step {i}"


@pytest.mark.parametrize("shape", [(4, 72, 136, 200), (3, 40, 72, 328)])
def test_dgrad_of_the_reduce_scatter_layer_is_an_ag_step_with_the_transposed_weight(shape):
    """dA^r = AG(G) (W^r)^T: Alg. 1 on the arriving slices of G."""
    p, mc, n, k = shape                              # forward layer: A [p*mc x k], W [k x n], Y [mc x n]
    rng = np.random.default_rng(95 + p)
    Wb, W = _bf16(rng, (k, n), 0.05)
    own_b, own = _bf16(rng, (mc, n))
    Sb, S = zip(*[_bf16(rng, (mc, n)) for _ in range(p - 1)])
    rank = 1
    ref = oracle.ag_rank(own, [None] + list(S), np.ascontiguousarray(W.T), p, rank)
    desc = cf.layer_desc(p, rank, mc, k, n, "bf16", "f32", cf.CF_W_NK)
    O = torch.full((p * mc, k), float("nan"), dtype=torch.float32, device=H.DEV)
    Wd = H.to_dev(Wb, "bf16")
    for i in range(p):
        cf.ag_step(desc, i, H.to_dev(own_b if i == 0 else Sb[i - 1], "bf16"), Wd, O, None)
    torch.cuda.synchronize()
    assert H.rel_err(H.to_host_f64(O), ref) <= TIGHT_BF16


WGRAD_SHAPES = [
    # (p, m_chunk, k, n)
    (4, 72, 136, 264),      # ragged everywhere; m_chunk = 64 + 8
    (2, 256, 512, 256),     # exact tiles
    (3, 200, 264, 1376),
    (1, 64, 8, 8),          # p = 1: one product, minimum k and n
    (8, 136, 520, 392),
]


@pytest.mark.parametrize("tile", [None, "256x256", "256x128", "128x128"])
@pytest.mark.parametrize("left_moves", [True, False])
@pytest.mark.parametrize("shape", WGRAD_SHAPES)
def test_wgrad_reduced(shape, left_moves, tile):
    p, mc, k, n = shape
    rng = np.random.default_rng(100 + p + (1 if left_moves else 0))
    width_mv, width_loc = (k, n) if left_moves else (n, k)
    mv = [_bf16(rng, (mc, width_mv), 0.5) for _ in range(p)]
    loc_b, loc = _bf16(rng, (p * mc, width_loc), 0.5)
    rank = p // 2
    ref = oracle.wgrad_rank_steps([x[1] for x in mv], loc, p, rank, left_moves)
    if tile is None:
        os.environ.pop("COMMFUSE_TILE", None)
    else:
        os.environ["COMMFUSE_TILE"] = tile
    try:
        run = H.WgradRun(p, rank, mc, k, n, [x[0] for x in mv], loc_b, left_moves, with_sink=True)
        outs = run.run_steps()
    finally:
        os.environ.pop("COMMFUSE_TILE", None)
    for i in range(p):
        e = H.rel_err(outs[i], ref[i])
        assert e <= TIGHT_BF16, f"step {i}: {e:.3e}"
        assert not np.isnan(outs[i]).any()
    if tile is not None:
        return
    with H.Workspace(run.desc, run.kind):
        for flags in (0, cf.CF_SERIAL, cf.CF_POISON, cf.CF_GRAPH, cf.CF_FUSED_COPY, cf.CF_DEVICE_WAIT):
            run.dW.fill_(float("nan"))
            run.run_schedule(flags)
            cf.device_status(run.cs)
            assert np.array_equal(H.to_host_f64(run.dW), outs[-1]), f"flags {flags}"
            for i in range(p - 1):
                assert np.array_equal(H.to_host_f64(run.sink[i]), mv[i][1]), f"flags {flags} hop {i}"


@pytest.mark.parametrize("m", [1, 2])
@pytest.mark.parametrize("left_moves", [True, False])
@pytest.mark.parametrize("shape", [(4, 72, 136, 200), (8, 128, 264, 136), (2, 264, 64, 328)])
def test_wgrad_persistent_is_one_gemm_over_the_gathered_operand(shape, left_moves, m):
    """CF_PERSISTENT for the weight gradient: the landing buffers form one gathered buffer, and the p chunk
    GEMMs become one GEMM over all its rows (other summation order: a tolerance, bit-exact on integers)."""
    p, mc, k, n = shape
    rng = np.random.default_rng(140 + p + (1 if left_moves else 0))
    width_mv, width_loc = (k, n) if left_moves else (n, k)
    PS = cf.CF_PERSISTENT | cf.CF_SERIAL
    for integer in (False, True):
        mv = [_bf16(rng, (mc, width_mv), 0.5, integer) for _ in range(p)]
        loc_b, loc = _bf16(rng, (p * mc, width_loc), 0.5, integer)
        for rank in (0, p - 1, p // 2):
            ref = oracle.wgrad_rank_steps([x[1] for x in mv], loc, p, rank, left_moves)[-1]
            run = H.WgradRun(p, rank, mc, k, n, [x[0] for x in mv], loc_b, left_moves, m=m, gathered=True)
            with H.Workspace(run.desc, run.kind):
                for flags in (PS, PS | cf.CF_GRAPH, PS | cf.CF_POISON, 0, cf.CF_DEVICE_WAIT):   # the layout serves every mode
                    run.dW.fill_(float("nan"))
                    run.run_schedule(flags)
                    run.run_schedule(flags)
                    cf.device_status(run.cs)
                    got = H.to_host_f64(run.dW)
                    if integer:
                        assert np.array_equal(got, ref), f"rank {rank} flags {flags}"
                    else:
                        assert H.rel_err(got, ref) <= TIGHT_BF16, f"rank {rank} flags {flags}"
            # every hop landed in its row block
            for i in range(1, p):
                c = (rank - i) % p
                assert np.array_equal(H.to_host_f64(run.gathered[c * mc:(c + 1) * mc]), mv[i][1])
    # separate landing buffers are not the gathered layout
    run = H.WgradRun(p, 0, mc, k, n, [x[0] for x in mv], loc_b, left_moves, each=True)
    with pytest.raises(cf.CommFuseError) as ei:
        run.run_schedule(PS)
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED


def test_wgrad_integer_inputs_are_bit_exact_and_granularity_changes_nothing_but_the_order():
    p, mc, k, n = 4, 128, 136, 264
    rng = np.random.default_rng(111)
    mv = [_bf16(rng, (mc, k), integer=True) for _ in range(p)]
    loc_b, loc = _bf16(rng, (p * mc, n), integer=True)
    for rank in range(p):
        ref = oracle.wgrad_rank_steps([x[1] for x in mv], loc, p, rank, True)
        outs = H.WgradRun(p, rank, mc, k, n, [x[0] for x in mv], loc_b, True).run_steps()
        for i in range(p):
            assert np.array_equal(outs[i], ref[i]), f"rank {rank} step {i}"
        fine = H.WgradRun(p, rank, mc, k, n, [x[0] for x in mv], loc_b, True, m=2)
        outs2 = fine.run_steps()
        assert len(outs2) == 2 * p and np.array_equal(outs2[-1], ref[-1])
        fine.dW.fill_(float("nan"))
        fine.run_schedule(0)
        assert np.array_equal(H.to_host_f64(fine.dW), ref[-1])


def test_wgrad_row_strides_and_bad_arguments():
    p, mc, k, n = 2, 72, 40, 72
    rng = np.random.default_rng(112)
    lda, ldw, ldo = 48, 80, 88
    Lb, L = _bf16(rng, (mc, lda))
    Rb, R = _bf16(rng, (mc, ldw))
    desc = cf.layer_desc(p, 0, mc, n, k, "bf16", "f32", lda=lda, ldw=ldw, ldo=ldo)
    dW = torch.full((k, ldo), -7.0, dtype=torch.float32, device=H.DEV)
    cf.wgrad_step(desc, 0, H.to_dev(Lb, "bf16"), H.to_dev(Rb, "bf16"), dW, None)
    torch.cuda.synchronize()
    got = H.to_host_f64(dW)
    ref = oracle.gemm(np.ascontiguousarray(L[:, :k].T), np.ascontiguousarray(R[:, :n]))
    assert H.rel_err(got[:, :n], ref) <= TIGHT_BF16
    assert np.all(got[:, n:] == -7.0), "padding columns are not written"
    t = torch.zeros(4096, dtype=torch.float32, device=H.DEV)
    with pytest.raises(cf.CommFuseError) as ei:
        cf.wgrad_step(cf.layer_desc(2, 0, 64, 64, 64, "f32", "f32"), 0, t, t, t, None)
    assert ei.value.status == cf.CF_ERR_UNSUPPORTED
    with pytest.raises(cf.CommFuseError) as ei:
        cf.wgrad_step(cf.layer_desc(2, 0, 64, 64, 64), 2, t, t, t, None)
    assert ei.value.status == cf.CF_ERR_INVALID_ARG
    with pytest.raises(cf.CommFuseError) as ei:
        cf.wgrad_step(cf.layer_desc(2, 0, 64, 64, 64), 0, None, t, t, None)
    assert ei.value.status == cf.CF_ERR_NULL_PTR


def test_wgrad_full_size_70b():
    """Weight gradient of the 70B up-projection: dW [8192 x 3584] from 8 slices of 1024 tokens."""
    p, mc, k, n = 8, 1024, 8192, 3584
    rng = np.random.default_rng(113)
    mv = [_bf16(rng, (mc, k), 0.5) for _ in range(p)]
    loc_b, loc = _bf16(rng, (p * mc, n), 0.5)
    rank = 3
    run = H.WgradRun(p, rank, mc, k, n, [x[0] for x in mv], loc_b, True)
    with H.Workspace(run.desc, run.kind):
        run.run_schedule(cf.CF_GRAPH)
    got = H.to_host_f64(run.dW)
    assert not np.isnan(got).any()
    rows = sorted({0, 1, 255, 256, 4095, 8191} | set(int(x) for x in rng.integers(0, k, size=6)))
    Xfull_T = np.concatenate([mv[i][1][:, rows] for i in range(p)], axis=0).T           # [rows x p*mc], ring order
    order = [(rank - i) % p for i in range(p)]
    G_ring = np.concatenate([loc[l * mc:(l + 1) * mc] for l in order], axis=0)
    ref = oracle.gemm(np.ascontiguousarray(Xfull_T), G_ring)
    assert H.rel_err(got[rows], ref) <= TOL_BF16
    assert H.rel_err(got[rows], ref) <= 2e-4          # eight fp32 partial sums of 1024 terms each

"""The entry point that allocates nothing (commfuse_rs_step_noalloc: split-K scratch in a static device array
inside the library) against the existing entry point (commfuse_rs_step with a registered workspace), through
the C ABI.  Same kernels, same split order, so the outputs must agree bit for bit -- and with the oracle within
the bf16 tolerance.  Two calls in a row, the second with a smaller input.  Needs an MI355X: ``-m gpu``."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_24013_amd import binding as cf
from paper_2604_24013_amd import inputs
from tests import harness as H

pytestmark = pytest.mark.gpu

TIGHT_BF16 = 1e-4


def _case(shape, salt, splitk):
    """Every step of one rank through both entry points; returns nothing, asserts."""
    p, mc, n, k = shape
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], p=p, m_chunk=mc, n=n, k=k)
    data = inputs.make_rs(w, salt=salt)
    rank = p // 2
    ref = oracle.rs_rank_steps(inputs.as_f64(data["A"], w.dtype), inputs.as_f64(data["W"], w.dtype),
                               [None] + [r.astype(np.float64) for r in data["R"][1:]], p, rank)
    run = H.RsRun(w, data, rank)
    if splitk:
        os.environ["COMMFUSE_SPLITK"] = str(splitk)
        os.environ["COMMFUSE_TILE"] = "128x128"
    try:
        with H.Workspace(run.desc, cf.CF_KIND_RS):
            want = run.run_steps()                                   # commfuse_rs_step, registered workspace
        got = []
        for i in range(p):                                           # no workspace registered now
            out = torch.full((mc, n), float("nan"), dtype=torch.float32, device=H.DEV)
            cf.rs_step_noalloc(run.desc, i, run.A, run.W, run.stage[i - 1] if i > 0 else None, out, None)
            got.append(out)
        torch.cuda.synchronize()
    finally:
        os.environ.pop("COMMFUSE_SPLITK", None)
        os.environ.pop("COMMFUSE_TILE", None)
    for i in range(p):
        g = H.to_host_f64(got[i])
        assert not np.isnan(g).any(), f"step {i}"
        assert np.array_equal(g, want[i]), f"step {i}: differs from commfuse_rs_step"
        e = H.rel_err(g, ref[i])
        assert e <= TIGHT_BF16, f"step {i}: {e:.3e} against the oracle"


def test_no_alloc_entry_point_matches_rs_step_twice_in_a_row():
    assert torch.cuda.is_available(), "this test needs the GPU"
    cf.load()
    # k-splits forced (3 splits of 34 k-tiles, several tiles and ragged tails), then the launcher's own choice
    # on a larger step, then a SMALLER input: the scratch still holds the partial tiles of the calls before
    _case((4, 520, 392, 2176), salt=51, splitk=3)
    _case((2, 512, 1536, 4096), salt=52, splitk=0)
    _case((3, 200, 264, 1096), salt=53, splitk=2)
    _case((2, 72, 136, 200), salt=54, splitk=0)


def test_no_alloc_entry_point_rejects_steps_beyond_its_scratch():
    cf.load()
    t = torch.zeros(4096, dtype=torch.bfloat16, device=H.DEV)
    o = torch.zeros(4096, dtype=torch.float32, device=H.DEV)
    with pytest.raises(cf.CommFuseError) as ei:
        cf.rs_step_noalloc(cf.layer_desc(8, 0, 1024, 8192, 3584), 0, t, t, None, o, None)   # 2^23 elements per step
    assert ei.value.status == cf.CF_ERR_INVALID_ARG and "static scratch" in str(ei.value)
    cf.rs_step_noalloc(cf.layer_desc(2, 0, 0, 64, 64), 0, t, t, None, o, None)               # empty step: nothing to do
    torch.cuda.synchronize()

"""The C ABI library: it loads, exports every function the header declares, and its
host-side argument checks turn bad calls into error codes.  No GPU is touched:
every call below fails validation before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2604_24013_amd import binding as cf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(cf.LIB_PATH):
        from paper_2604_24013_amd import build
        build.build()
    return cf.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "commfuse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(commfuse_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert len(names) >= 9
    for nm in names:
        assert hasattr(lib, nm), f"{nm} declared in commfuse.h but not exported"
    assert sorted(cf.EXPORTS) == names, "binding and header disagree on the entry points"


def test_struct_layout_matches_header():
    # cf_layer_desc: 2 x int32, 6 x int64, 4 x int32 = 72 bytes; cf_buffers: 11 pointers
    assert ctypes.sizeof(cf.LayerDesc) == 72
    assert cf.LayerDesc.m_chunk.offset == 8 and cf.LayerDesc.in_dtype.offset == 56
    assert ctypes.sizeof(cf.Buffers) == 11 * ctypes.sizeof(ctypes.c_void_p)


def test_attention_struct_layout_matches_header():
    # cf_attn_desc: 6 x int32, 3 x int64, int32 + float = 56 bytes; cf_attn_buffers: 14 pointers
    assert ctypes.sizeof(cf.AttnDesc) == 56
    assert cf.AttnDesc.n.offset == 24 and cf.AttnDesc.w_layout.offset == 48 and cf.AttnDesc.scale.offset == 52
    assert ctypes.sizeof(cf.AttnBuffers) == 14 * ctypes.sizeof(ctypes.c_void_p)


def test_backward_granularity_and_attention_bad_arguments(lib):
    A, B, C, D = 0x1000, 0x2000, 0x3000, 0x4000            # fake, aligned, never dereferenced
    # weight gradient
    assert _status(cf.wgrad_step, cf.layer_desc(2, 0, 64, 64, 64, "f32", "f32"), 0, A, B, C)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.wgrad_step, cf.layer_desc(2, 0, 64, 64, 64), 2, A, B, C)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.wgrad_step, cf.layer_desc(2, 0, 64, 64, 64), 0, None, B, C)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.wgrad_step, cf.layer_desc(2, 0, 64, 64, 64), 0, A + 8, B, C)[0] == cf.CF_ERR_MISALIGNED
    # slicing granularity
    assert _status(cf.rs_step, cf.layer_desc(2, 0, 30, 64, 64, m=4), 0, A, B, None, D)[0] == cf.CF_ERR_INVALID_ARG
    d = cf.layer_desc(2, 0, 32, 64, 64, m=2)
    assert _status(cf.rs_step, d, 4, A, B, C, D)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, d, 1, A, B, C, D)[0] == cf.CF_ERR_NULL_PTR          # the first hop receives nothing
    assert _status(cf.rs_step, d, 2, A, B, None, D)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.rs_pair_step, d, 0, A, B, None, None, D)[0] == cf.CF_ERR_UNSUPPORTED
    assert [cf.subslice_index(cf.CF_KIND_RS, 4, 2, 1, j) for j in range(8)] == [0, 1, 6, 7, 4, 5, 2, 3]
    assert _status(cf.subslice_index, cf.CF_KIND_RS_PAIR, 4, 2, 1, 0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.subslice_index, cf.CF_KIND_RS, 4, 0, 1, 0)[0] == cf.CF_ERR_INVALID_ARG
    # attention
    ok = cf.attn_desc(2, 0, 1, 1, 128, 128, 64, 0.1)
    assert _status(cf.attn_slice, cf.attn_desc(2, 0, 1, 1, 128, 64, 64, 0.1), 0, A, B, C, D)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.attn_slice, cf.attn_desc(3, 0, 1, 1, 128, 128, 64, 0.1), 0, A, B, C, D)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.attn_slice, ok, 2, A, B, C, D)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.attn_slice, ok, 0, A, None, C, D)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.attn_slice, cf.attn_desc(2, 0, 1, 1, 128, 128, 64, 0.0), 0, A, B, C, D)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.attn_rs_step, ok, 0, A, B, C, D, 0x5000, 0x6000, 0x7000)[0] == cf.CF_ERR_NULL_PTR   # recv at step 0
    assert _status(cf.attn_rs_step, ok, 1, A, B, C, D, None, 0x6000, 0x7000)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.attn_rs_step, ok, 1, A, B, C, D, 0x6000, 0x6000, 0x7000)[0] == cf.CF_ERR_INVALID_ARG


def test_version(lib):
    assert cf.version() >= 100


@pytest.mark.parametrize("p", [1, 2, 3, 8])
def test_chunk_index_matches_the_algorithms(lib, p):
    for r in range(p):
        rs = [cf.chunk_index(cf.CF_KIND_RS, p, r, i) for i in range(p)]
        ag = [cf.chunk_index(cf.CF_KIND_AG, p, r, i) for i in range(p)]
        dp = [cf.chunk_index(cf.CF_KIND_DP, p, r, i) for i in range(p)]
        assert sorted(rs) == list(range(p)) and sorted(ag) == list(range(p))
        assert rs[-1] == r and ag[0] == r and dp == rs
        for i in range(p):
            assert rs[i] == (r - i - 1 + p) % p        # Alg. 2 index line
            assert ag[i] == (r - i + p) % p            # Alg. 1 index line


@pytest.mark.parametrize("p", [2, 4, 6, 8, 12, 16])
def test_pairwise_partner_is_a_tournament(lib, p):
    """Appendix A(a): every round is a perfect matching and every pair meets exactly once."""
    import oracle
    met = set()
    for t in range(1, p):
        for r in range(p):
            q = cf.pair_partner(p, r, t)
            assert q == oracle.pair_partner(p, r, t)
            assert q != r and cf.pair_partner(p, q, t) == r
            met.add((min(r, q), max(r, q)))
    assert len(met) == p * (p - 1) // 2
    for r in range(p):
        ls = [cf.chunk_index(cf.CF_KIND_RS_PAIR, p, r, i) for i in range(p)]
        assert ls == [cf.chunk_index(cf.CF_KIND_DP_PAIR, p, r, i) for i in range(p)]
        assert sorted(ls) == list(range(p)) and ls[-1] == r
        assert ls[:-1] == [cf.pair_partner(p, r, t) for t in range(1, p)]
    if p == 4:                                            # the appendix's printed rounds
        assert [cf.pair_partner(4, 0, t) for t in (1, 2, 3)] == [1, 2, 3]
        assert [cf.pair_partner(4, 1, t) for t in (1, 2, 3)] == [0, 3, 2]


def test_pairwise_bad_arguments(lib):
    A, W, R, O, ACC = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000
    assert _status(cf.pair_partner, 3, 0, 1)[0] == cf.CF_ERR_INVALID_ARG        # odd p
    assert _status(cf.pair_partner, 4, 0, 0)[0] == cf.CF_ERR_INVALID_ARG        # rounds are 1-based
    assert _status(cf.pair_partner, 4, 0, 4)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.pair_partner, 4, 4, 1)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.chunk_index, cf.CF_KIND_RS_PAIR, 5, 0, 0)[0] == cf.CF_ERR_INVALID_ARG
    assert cf.chunk_index(cf.CF_KIND_RS_PAIR, 1, 0, 0) == 0
    good = cf.layer_desc(4, 1, 16, 32, 64)
    assert _status(cf.rs_pair_step, cf.layer_desc(3, 0, 16, 32, 64), 0, A, W, None, ACC, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_pair_step, good, 0, A, W, R, ACC, O)[0] == cf.CF_ERR_NULL_PTR      # nothing received at step 0
    assert _status(cf.rs_pair_step, good, 1, A, W, None, ACC, O)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.rs_pair_step, good, 2, A, W, R, None, O)[0] == cf.CF_ERR_NULL_PTR     # p > 2 needs acc
    assert _status(cf.rs_pair_step, good, 2, A, W, R, ACC, ACC)[0] == cf.CF_ERR_INVALID_ARG  # in place before the last step
    assert _status(cf.rs_pair_step, good, 3, A, W, R, ACC, R)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_pair_step, good, 2, A, W, ACC, ACC, O)[0] == cf.CF_ERR_INVALID_ARG  # recv == acc only at step 1
    assert _status(cf.rs_pair_step, cf.layer_desc(4, 1, 16, 32, 64, ldo=40), 2, A, W, R, ACC, O)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.dp_pair_step, 3, 0, 1, A, 16, R)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.dp_pair_step, 4, 0, 1, None, 16, R)[0] == cf.CF_ERR_NULL_PTR
    cf.dp_pair_step(4, 0, 0, None, 16, None)             # step 0 enqueues nothing
    assert _status(cf.rs_pair_step, good, 3, A, W, None, None, O)[0] == cf.CF_ERR_NULL_PTR   # the last step cannot defer
    assert _status(cf.rs_pair_last_step, good, A, W, [], O)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.rs_pair_last_step, good, A, W, [R, None, ACC], O)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.rs_pair_last_step, good, A, W, [R, O, ACC], O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_pair_last_step, cf.layer_desc(3, 0, 16, 32, 64), A, W, [R, ACC], O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_pair_last_step, cf.layer_desc(4, 1, 16, 32, 64, ldo=40), A, W, [R, ACC, 0x6000], O)[0] == cf.CF_ERR_UNSUPPORTED


def _status(fn, *a):
    with pytest.raises(cf.CommFuseError) as e:
        fn(*a)
    return e.value.status, str(e.value)


def test_bad_arguments_are_rejected_on_the_host(lib):
    A, W, R, O = 0x1000, 0x2000, 0x3000, 0x4000            # fake, aligned, never dereferenced
    good = cf.layer_desc(4, 1, 16, 32, 64)
    assert _status(cf.chunk_index, 0, 0, 0, 0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.chunk_index, 7, 4, 0, 0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, cf.layer_desc(0, 0, 16, 32, 64), 0, A, W, None, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, cf.layer_desc(4, 4, 16, 32, 64), 0, A, W, None, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, good, 4, A, W, R, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, good, -1, A, W, R, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, good, 0, None, W, None, O)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.rs_step, good, 0, A, W, R, O)[0] == cf.CF_ERR_NULL_PTR       # recv at step 0
    assert _status(cf.rs_step, good, 1, A, W, None, O)[0] == cf.CF_ERR_NULL_PTR    # no recv at step 1
    assert _status(cf.rs_step, good, 1, A, W, O, O)[0] == cf.CF_ERR_INVALID_ARG    # aliasing
    assert _status(cf.rs_step, good, 1, A + 2, W, R, O)[0] == cf.CF_ERR_MISALIGNED
    assert _status(cf.rs_step, cf.layer_desc(4, 1, 16, 32, 60), 1, A, W, R, O)[0] == cf.CF_ERR_MISALIGNED
    assert _status(cf.rs_step, cf.layer_desc(4, 1, 16, 34, 64, "f32"), 1, A, W, R, O)[0] == cf.CF_ERR_MISALIGNED
    assert _status(cf.rs_step, cf.layer_desc(4, 1, 16, 32, 64, lda=32), 1, A, W, R, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.rs_step, cf.layer_desc(4, 1, 16, 32, 64, in_dtype=5), 1, A, W, R, O)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.ag_step, cf.layer_desc(4, 1, 16, 32, 64, "f32", "bf16"), 1, A, W, O)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.ag_step, good, 0, A, None, O)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.ag_step, good, 9, A, W, O)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.dp_reduce_step, 4, 0, 1, None, 16, R)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.dp_reduce_step, 4, 0, 5, A, 16, R)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.dp_reduce_step, 4, 0, 1, A, -1, R)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.dp_reduce_step, 4, 0, 1, A + 1, 16, R)[0] == cf.CF_ERR_MISALIGNED
    st, text = _status(cf.rs_step, good, 7, A, W, R, O)
    assert "step" in text and cf.last_error() in text
    # step 0 of the gradient path computes nothing and enqueues nothing: succeeds without a GPU
    cf.dp_reduce_step(4, 0, 0, None, 16, None)


def test_schedule_argument_checks(lib):
    d = cf.layer_desc(4, 0, 16, 32, 64)
    t = [0x1000, 0x2000, 0x3000]
    ok = cf.make_buffers(0x100, 0x200, 0x300, t, (0x400, 0x500), (0x600, 0x700))
    assert _status(cf.run_schedule, d, 9, ok, None, None, 0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, ok, None, None, 1 << 9)[0] == cf.CF_ERR_INVALID_ARG
    bad = cf.make_buffers(0x100, 0x200, None, t, (0x400, 0x500), (0x600, 0x700))
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, bad, None, None, 0)[0] == cf.CF_ERR_NULL_PTR
    bad = cf.make_buffers(0x100, 0x200, 0x300, t, (0x400, 0x400), (0x600, 0x700))
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, bad, None, None, 0)[0] == cf.CF_ERR_INVALID_ARG
    bad = cf.make_buffers(0x100, 0x200, 0x300, t, (0x400, 0x500), (None, None))
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, bad, None, None, 0)[0] == cf.CF_ERR_NULL_PTR
    bad = cf.make_buffers(0x100, 0x200, 0x300, [0x1000, None, 0x3000], (0x400, 0x500), (0x600, 0x700))
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, bad, None, None, 0)[0] == cf.CF_ERR_NULL_PTR
    # a B_out buffer per sending step: every entry set, aligned, distinct from O, the landing buffers and each other
    each = [0x4000, 0x5000, 0x6000]
    se = lambda tab, **kw: cf.make_buffers(0x100, 0x200, 0x300, t, (0x400, 0x500), (None, None), None, kw.get("each"), tab)
    PS = cf.CF_PERSISTENT | cf.CF_SERIAL
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, se([0x7000, None, 0x9000]), None, None, 0)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, se([0x7000, 0x300, 0x9000]), None, None, 0)[0] == cf.CF_ERR_NULL_PTR
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, se([0x7000, 0x8008, 0x9000]), None, None, 0)[0] == cf.CF_ERR_MISALIGNED
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, se([0x7000, 0x8000, 0x7000]), None, None, 0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, se([0x7000, 0x5000, 0x9000], each=each), None, None, PS)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, se(None, each=each), None, None, PS)[0] == cf.CF_ERR_INVALID_ARG
    strided = cf.layer_desc(4, 0, 16, 32, 64, ldo=40)
    assert _status(cf.run_schedule, strided, cf.CF_KIND_RS_PAIR, ok, None, None, 0)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, ok, None, None, cf.CF_GRAPH)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.run_schedule, d, cf.CF_KIND_RS, ok, None, None, cf.CF_FUSED_COPY | cf.CF_POISON)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.run_schedule, cf.layer_desc(4, 0, 16, 32, 64, "f32"), cf.CF_KIND_RS, ok, None, None, cf.CF_FUSED_COPY)[0] == cf.CF_ERR_UNSUPPORTED
    assert _status(cf.run_schedule, cf.layer_desc(4, 0, 16, 0, 0), cf.CF_KIND_DP, ok, None, None, cf.CF_FUSED_COPY)[0] == cf.CF_ERR_UNSUPPORTED
    # 64 KiB of arrival counters + 8 partial tiles of m_chunk x n fp32; none for the gradient path / fp32
    assert cf.workspace_bytes(d, cf.CF_KIND_RS) == 64 * 1024 + 8 * 16 * 32 * 4
    assert cf.workspace_bytes(d, cf.CF_KIND_DP) == 0
    assert cf.workspace_bytes(cf.layer_desc(4, 0, 16, 32, 64, "f32"), cf.CF_KIND_AG) == 0
    assert _status(cf.set_workspace, 0x1008, 1 << 20)[0] == cf.CF_ERR_MISALIGNED
    assert _status(cf.set_workspace, 0x1000, 1024)[0] == cf.CF_ERR_INVALID_ARG
    cf.set_workspace(None)


def test_binding_has_no_fallback():
    src = open(os.path.join(ROOT, "paper_2604_24013_amd", "binding.py")).read()
    assert "import oracle" not in src and "from oracle" not in src
    assert "torch.matmul" not in src and "@" not in src.replace("@pytest", "")

"""Pins for the CPU oracle: it is checked against what the paper prints and what
the mathematics fixes, never against itself.  CPU only."""
import itertools
import os
import re

import numpy as np
import pytest

import oracle


# ----------------------------------------------------------------------------
# helpers: symbolic one-hot encoding of "term x_c" = device x, slice c
# ----------------------------------------------------------------------------
DEV = "abcd"


def onehot_problem(p):
    """A row-parallel problem whose partial product for (device q, slice c) is the
    one-hot vector e_{q*p+c}: X^q slice c is e_c (1 x p), W^q row k is e_{q*p+k}."""
    X_list, W_list = [], []
    for q in range(p):
        X_list.append(np.eye(p))                       # slice c (one row) = e_c
        W = np.zeros((p, p * p))
        for k in range(p):
            W[k, q * p + k] = 1.0
        W_list.append(W)
    return X_list, W_list


def decode(vec, p):
    """Multiset of (device, slice) terms encoded in a 1 x p*p vector."""
    v = np.asarray(vec).reshape(-1)
    terms = []
    for idx, cnt in enumerate(v):
        assert cnt == int(cnt) and cnt >= 0
        terms += [(idx // p, idx % p)] * int(cnt)
    return sorted(terms)


def parse_terms(expr):
    out = []
    for t in re.split(r"[+\s]+", expr.strip()):
        if t:
            out.append((DEV.index(t[0]), int(t[1:]) - 1))     # slices are printed 1-based
    return sorted(out)


def read_golden(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


# ----------------------------------------------------------------------------
# P1: the paper's worked all-gather / reduce-scatter examples (Sec. 3.1)
# ----------------------------------------------------------------------------

def test_all_gather_paper_example(golden_dir):
    lines = dict(ln.split(":", 1) for ln in read_golden(golden_dir, "collective_examples.txt"))
    sym = {s: float(10 + n) for n, s in enumerate("abcd")}
    ins = [np.array([[sym[t.strip()]]]) for t in lines["all_gather in"].split("|")]
    outs = [[sym[s] for s in t.split()] for t in lines["all_gather out"].split("|")]
    got = oracle.all_gather(ins)
    assert len(got) == 4
    for r in range(4):
        assert got[r].reshape(-1).tolist() == outs[r]


def test_reduce_scatter_paper_example(golden_dir):
    lines = dict(ln.split(":", 1) for ln in read_golden(golden_dir, "collective_examples.txt"))
    # distinct powers of two: every subset sum is unique, so a wrong term shows
    names = [t.split() for t in lines["reduce_scatter in"].split("|")]
    val = {}
    for q, row in enumerate(names):
        for c, nm in enumerate(row):
            val[nm] = float(2 ** (4 * q + c))
    ins = [[np.array([val[nm]]) for nm in row] for row in names]
    want = [sum(val[t] for t in e.strip().split("+")) for e in lines["reduce_scatter out"].split("|")]
    got = oracle.reduce_scatter(ins)
    assert [float(g[0]) for g in got] == want


# ----------------------------------------------------------------------------
# P2: Appendix A(b) circular-P2P trace pins who computes which slice when
# ----------------------------------------------------------------------------

def test_appendix_circular_trace(golden_dir):
    p = 4
    rounds = {}
    for ln in read_golden(golden_dir, "appendix_a_circular_p2p_trace.txt"):
        if ln.startswith("round"):
            head, body = ln.split(":", 1)
            t = int(head.split()[1])
            rounds[t] = [parse_terms(b.split("=", 1)[1]) for b in body.split(";")]
    assert sorted(rounds) == [1, 2, 3, 4]
    X_list, W_list = onehot_problem(p)
    O, received, sent = oracle.fuse_rs_lockstep(X_list, W_list)
    prev = [[] for _ in range(p)]
    for t in range(1, p + 1):
        i = t - 1
        for c in range(p):                       # buffer m_{c+1}
            terms = rounds[t][c]
            assert all(sl == c for _, sl in terms), "buffer m_c only ever holds slice c"
            new = [x for x in terms if x not in prev[c]]
            assert len(new) == 1, "exactly one new term per buffer per round"
            holder = new[0][0]                   # the device whose own term was just added
            held = sent[holder][i] if i < p - 1 else O[holder]
            assert decode(held, p) == terms, (t, c)
            if i > 0:                            # what it received is last round's buffer
                assert decode(received[holder][i], p) == prev[c]
            prev[c] = terms
    # after the last round device c holds the full sum of slice c and nothing is sent
    for r in range(p):
        assert decode(O[r], p) == [(q, r) for q in range(p)]
        assert sent[r][p - 1] is None
        assert received[r][0] is None


def test_appendix_send_lists(golden_dir):
    """Running example of the appendix: device x contributes slice c to device c, for
    every c other than its own -- the terms that leave x in the ring are exactly those."""
    p = 4
    X_list, W_list = onehot_problem(p)
    _, _, sent = oracle.fuse_rs_lockstep(X_list, W_list)
    for ln in read_golden(golden_dir, "appendix_a_circular_p2p_trace.txt"):
        if not ln.startswith("sends"):
            continue
        head, body = ln.split(":", 1)
        q = DEV.index(head.split()[1].lower())
        want = sorted((DEV.index(t[0]), int(t[1:]) - 1) for t in body.split())
        own_terms = sorted(
            term for i in range(p - 1) for term in decode(sent[q][i], p) if term[0] == q
        )
        assert own_terms == want


# ----------------------------------------------------------------------------
# P3: closed-form invariants of the index functions (Alg. 1, Alg. 2)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("p", [1, 2, 3, 4, 5, 8, 16])
def test_index_invariants(p):
    for r in range(p):
        ls_rs = [oracle.slice_index_rs(p, r, i) for i in range(p)]
        ls_ag = [oracle.slice_index_ag(p, r, i) for i in range(p)]
        assert sorted(ls_rs) == list(range(p)) and sorted(ls_ag) == list(range(p))
        assert ls_rs[p - 1] == r, "reduce-scatter: own slice is computed last"
        assert ls_ag[0] == r, "all-gather: own slice is computed first"
        assert oracle.send_rank(p, oracle.recv_rank(p, r)) == r
        nxt = oracle.send_rank(p, r)
        for i in range(p - 1):
            # what r works on at step i is what its successor works on at step i+1
            assert oracle.slice_index_rs(p, nxt, i + 1) == ls_rs[i]
            assert oracle.slice_index_ag(p, nxt, i + 1) == ls_ag[i]


# ----------------------------------------------------------------------------
# P4: exactness claim -- decomposed + fused == dense then collective
# ----------------------------------------------------------------------------

def _rand_problem(rng, p, mc, n, k, integer):
    if integer:
        g = lambda *s: rng.integers(-4, 5, size=s).astype(np.float64)
    else:
        g = lambda *s: rng.standard_normal(size=s)
    return g


@pytest.mark.parametrize("p,mc,n,k", [(1, 3, 4, 5), (2, 2, 3, 4), (3, 1, 5, 2), (4, 3, 7, 6), (8, 2, 5, 3)])
@pytest.mark.parametrize("integer", [True, False])
def test_rs_exactness(p, mc, n, k, integer):
    rng = np.random.default_rng(100 * p + mc + (7 if integer else 0))
    g = _rand_problem(rng, p, mc, n, k, integer)
    A = [g(p * mc, k) for _ in range(p)]
    W = [g(k, n) for _ in range(p)]
    want = oracle.rs_definition(A, W)
    got, _, _ = oracle.fuse_rs_lockstep(A, W)
    # independent statement of the definition with a library routine
    Y = sum(np.matmul(A[q], W[q]) for q in range(p))
    for r in range(p):
        if integer:
            assert np.array_equal(got[r], want[r])
            assert np.array_equal(got[r], Y[r * mc:(r + 1) * mc])
        else:
            np.testing.assert_allclose(got[r], want[r], rtol=0, atol=1e-12 * max(1.0, np.abs(want[r]).max()))
            np.testing.assert_allclose(got[r], Y[r * mc:(r + 1) * mc], rtol=0, atol=1e-12 * max(1.0, np.abs(Y).max()))


@pytest.mark.parametrize("p,mc,n,k", [(1, 3, 4, 5), (2, 2, 3, 4), (3, 1, 5, 2), (4, 3, 7, 6), (8, 2, 5, 3)])
@pytest.mark.parametrize("integer", [True, False])
def test_ag_exactness(p, mc, n, k, integer):
    rng = np.random.default_rng(200 * p + mc + (7 if integer else 0))
    g = _rand_problem(rng, p, mc, n, k, integer)
    X = [g(mc, k) for _ in range(p)]
    W = [g(k, n) for _ in range(p)]
    want = oracle.ag_definition(X, W)
    got, held = oracle.fuse_ag_lockstep(X, W)
    full = np.concatenate(X, axis=0)
    for r in range(p):
        lib = np.matmul(full, W[r])
        if integer:
            assert np.array_equal(got[r], want[r]) and np.array_equal(got[r], lib)
        else:
            np.testing.assert_allclose(got[r], want[r], rtol=0, atol=1e-12 * max(1.0, np.abs(lib).max()))
            np.testing.assert_allclose(got[r], lib, rtol=0, atol=1e-12 * max(1.0, np.abs(lib).max()))
        # ring order: at step i rank r holds the slice that started on rank r-i
        for i in range(p):
            assert np.array_equal(held[r][i], X[(r - i) % p])


@pytest.mark.parametrize("p,c", [(1, 5), (2, 4), (4, 3), (8, 6)])
def test_dp_exactness(p, c):
    rng = np.random.default_rng(300 + p)
    g = [rng.integers(-50, 51, size=p * c).astype(np.float64) for _ in range(p)]
    want = oracle.dp_definition(g)
    got, _, _ = oracle.fuse_dp_lockstep(g)
    tot = np.sum(np.stack(g), axis=0)
    for r in range(p):
        assert np.array_equal(got[r], want[r])
        assert np.array_equal(got[r], tot[r * c:(r + 1) * c])


# ----------------------------------------------------------------------------
# P5 / P7 / P8: the arithmetic pieces
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (17, 9, 33), (64, 48, 100), (0, 4, 3), (4, 0, 3)])
def test_gemm_vs_numpy(M, N, K):
    rng = np.random.default_rng(M * 1000 + N * 10 + K)
    X = rng.standard_normal((M, K))
    W = rng.standard_normal((K, N))
    got = oracle.gemm(X, W)
    want = np.matmul(X, W)
    assert got.shape == (M, N)
    if M and N:
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-13 * K * max(1.0, np.abs(want).max()))


def test_gemm_is_not_transposed():
    X = np.array([[1.0, 2.0, 3.0]])            # 1 x 3
    W = np.array([[1.0, 10.0], [100.0, 1000.0], [1e4, 1e5]])   # 3 x 2
    assert oracle.gemm(X, W).tolist() == [[1 + 200 + 3e4, 10 + 2000 + 3e5]]
    assert oracle.dot_element(X, W, 0, 1) == 10 + 2000 + 3e5


def test_gemm_bruteforce_python():
    rng = np.random.default_rng(5)
    M, N, K = 5, 4, 6
    X = rng.integers(-9, 10, size=(M, K)).astype(np.float64)
    W = rng.integers(-9, 10, size=(K, N)).astype(np.float64)
    got = oracle.gemm(X, W)
    for i, j in itertools.product(range(M), range(N)):
        s = 0.0
        for k in range(K):
            s += X[i, k] * W[k, j]
        assert got[i, j] == s
        assert oracle.dot_element(X, W, i, j) == s


def test_gemm_strided_views_are_handled():
    rng = np.random.default_rng(6)
    big = rng.standard_normal((12, 10))
    X = big[2:9, 1:7]                            # non-contiguous view
    W = rng.standard_normal((6, 3))
    np.testing.assert_allclose(oracle.gemm(X, W), np.matmul(X, W), atol=1e-13)


def test_add_vs_numpy():
    rng = np.random.default_rng(7)
    a = rng.standard_normal(1001)
    b = rng.standard_normal(1001)
    assert np.array_equal(oracle.add(a, b), np.add(a, b))


def test_round_to_bf16_known_values():
    # bf16 keeps 8 significant bits: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0)
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0, 3.0e38])
    got = oracle.round_to_bf16(x)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -2.5, 0.0, 2.9908533 * 1e38])
    np.testing.assert_allclose(got[:6], want[:6], rtol=0, atol=0)
    # every output is representable with an 8-bit significand
    m, _ = np.frexp(got[got != 0])
    assert np.all(m * 256 == np.round(m * 256))
    # rounding error bounded by half an ulp = 2^-9 relative
    assert np.all(np.abs(got - x) <= np.abs(x) * 2.0 ** -8)


# ----------------------------------------------------------------------------
# one-rank views agree with the lock-step runs when fed the mailbox contents
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("p", [1, 2, 4, 8])
def test_rank_views_match_lockstep(p):
    rng = np.random.default_rng(400 + p)
    mc, n, k = 3, 5, 4
    A = [rng.integers(-4, 5, size=(p * mc, k)).astype(np.float64) for _ in range(p)]
    W = [rng.integers(-4, 5, size=(k, n)).astype(np.float64) for _ in range(p)]
    O, received, sent = oracle.fuse_rs_lockstep(A, W)
    X = [rng.integers(-4, 5, size=(mc, k)).astype(np.float64) for _ in range(p)]
    Oag, held = oracle.fuse_ag_lockstep(X, W)
    g = [rng.integers(-50, 51, size=p * mc).astype(np.float64) for _ in range(p)]
    Odp, rdp, _ = oracle.fuse_dp_lockstep(g)
    Ydef = oracle.rs_definition(A, W)
    for r in range(p):
        outs = oracle.rs_rank_steps(A[r], W[r], received[r], p, r)
        for i in range(p - 1):
            assert np.array_equal(outs[i], sent[r][i])
        assert np.array_equal(outs[p - 1], O[r]) and np.array_equal(outs[p - 1], Ydef[r])
        assert np.array_equal(oracle.ag_rank(X[r], held[r], W[r], p, r), Oag[r])
        b = oracle.dp_rank(g[r], rdp[r], p, r)
        assert np.array_equal(b[r * mc:(r + 1) * mc], Odp[r])
        # linearity of the epilogue: out(R) - out(0) == R exactly
        if p > 1:
            zero = [None] + [np.zeros((mc, n))] * (p - 1)
            outs0 = oracle.rs_rank_steps(A[r], W[r], zero, p, r)
            for i in range(1, p):
                assert np.array_equal(outs[i] - outs0[i], received[r][i])
                assert np.array_equal(outs0[i], np.matmul(oracle.split_rows(A[r], p)[(r - i - 1) % p], W[r]))


def test_dp_rank_touches_only_scheduled_slices():
    p, c, r = 4, 5, 2
    rng = np.random.default_rng(9)
    bucket = rng.standard_normal(p * c)
    R = [None] + [rng.standard_normal(c) for _ in range(p - 1)]
    out = oracle.dp_rank(bucket, R, p, r)
    touched = {(r - i - 1) % p: i for i in range(1, p)}
    for l in range(p):
        sl = slice(l * c, (l + 1) * c)
        if l in touched:
            assert np.array_equal(out[sl], bucket[sl] + R[touched[l]])
        else:
            assert np.array_equal(out[sl], bucket[sl])
    # the slice sent at step 0 is (r-1) mod p and is left alone
    assert (r - 1) % p not in touched


def test_pair_matches_definition_up_to_bf16_handover():
    p, mc, d, f = 4, 4, 8, 6
    rng = np.random.default_rng(10)
    X = [rng.integers(-2, 3, size=(mc, d)).astype(np.float64) for _ in range(p)]
    Wup = rng.integers(-2, 3, size=(d, f)).astype(np.float64)
    Wdn = rng.integers(-2, 3, size=(f, d)).astype(np.float64)
    r = 1
    S = [None] + [X[(r - i) % p] for i in range(1, p)]
    R = [None] + [rng.integers(-5, 6, size=(mc, d)).astype(np.float64) for _ in range(p - 1)]
    H, outs = oracle.mlp_pair_rank(X[r], S, Wup, Wdn, R, p, r)
    Hdef = np.matmul(np.concatenate(X, axis=0), Wup)      # small integers: bf16 rounding is exact
    assert np.array_equal(H, Hdef)
    for i in range(p):
        l = (r - i - 1) % p
        want = np.matmul(Hdef[l * mc:(l + 1) * mc], Wdn) + (R[i] if i else 0)
        assert np.array_equal(outs[i], want)


# ----------------------------------------------------------------------------
# planted mistakes: each must be caught by a pin above (run on the CPU only)
# ----------------------------------------------------------------------------

def _pins_fail(monkeypatch_fn, golden_dir):
    failed = 0
    for t in (lambda: test_appendix_circular_trace(golden_dir),
              lambda: test_rs_exactness(4, 3, 7, 6, True),
              lambda: test_ag_exactness(4, 3, 7, 6, True),
              lambda: test_index_invariants(4),
              lambda: test_gemm_is_not_transposed()):
        try:
            t()
        except AssertionError:
            failed += 1
        except Exception:
            failed += 1
    return failed


@pytest.mark.parametrize("mistake", ["rs_index_sign", "rs_index_no_minus_one", "ag_index_sign", "send_backwards", "drop_add"])
def test_planted_mistakes_are_caught(monkeypatch, golden_dir, mistake):
    if mistake == "rs_index_sign":
        monkeypatch.setattr(oracle, "slice_index_rs", lambda p, r, i: (r + i + 1) % p)
    elif mistake == "rs_index_no_minus_one":
        monkeypatch.setattr(oracle, "slice_index_rs", lambda p, r, i: (r - i) % p)
    elif mistake == "ag_index_sign":
        monkeypatch.setattr(oracle, "slice_index_ag", lambda p, r, i: (r + i) % p)
    elif mistake == "send_backwards":
        monkeypatch.setattr(oracle, "send_rank", lambda p, r: (r - 1) % p)
    elif mistake == "drop_add":
        monkeypatch.setattr(oracle, "add", lambda a, b: np.asarray(b, dtype=np.float64))
    assert _pins_fail(None, golden_dir) >= 1


# ----------------------------------------------------------------------------
# pairwise bidirectional schedule (Appendix A(a))
# ----------------------------------------------------------------------------

def test_pairwise_rounds_match_the_paper(golden_dir):
    rounds = {}
    for ln in read_golden(golden_dir, "appendix_a_pairwise_rounds.txt"):
        head, body = ln.split(":", 1)
        rounds[int(head.split()[1])] = [tuple(sorted("ABCD".index(x.strip()) for x in pr.split("<->"))) for pr in body.split(";")]
    assert sorted(rounds) == [1, 2, 3]
    for t, pairs in rounds.items():
        got = sorted({tuple(sorted((r, oracle.pair_partner(4, r, t)))) for r in range(4)})
        assert got == sorted(pairs), t
    # with the one-hot problem: what travels in round t is the sender's partial of the RECEIVER's slice
    X_list, W_list = onehot_problem(4)
    O, received, sent = oracle.fuse_rs_pairwise_lockstep(X_list, W_list)
    for t, pairs in rounds.items():
        for a, b in pairs:
            assert decode(received[a][t], 4) == [(b, a)] and decode(received[b][t], 4) == [(a, b)]
    for r in range(4):
        assert decode(O[r], 4) == [(q, r) for q in range(4)]
        assert sent[r][3] is None


def test_pairwise_send_lists_match_the_running_example(golden_dir):
    """Appendix running example: A sends a2, a3, a4 to B, C, D etc. -- each device's sends are its
    partials of the other devices' slices, one to each owner."""
    X_list, W_list = onehot_problem(4)
    _, _, sent = oracle.fuse_rs_pairwise_lockstep(X_list, W_list)
    for ln in read_golden(golden_dir, "appendix_a_circular_p2p_trace.txt"):
        if not ln.startswith("sends"):
            continue
        head, body = ln.split(":", 1)
        q = DEV.index(head.split()[1].lower())
        want = sorted((DEV.index(t[0]), int(t[1:]) - 1) for t in body.split())
        got = sorted(term for i in range(3) for term in decode(sent[q][i], 4))
        assert got == want


@pytest.mark.parametrize("p", [2, 4, 6, 8, 10, 12, 16])
def test_pairwise_is_a_round_robin_tournament(p):
    met = set()
    for t in range(1, p):
        seen = set()
        for r in range(p):
            q = oracle.pair_partner(p, r, t)
            assert q != r and 0 <= q < p
            assert oracle.pair_partner(p, q, t) == r, "pairing must be symmetric"
            seen.add(r)
            met.add((min(r, q), max(r, q)))
        assert len(seen) == p
    assert len(met) == p * (p - 1) // 2, "every pair meets exactly once"
    for r in range(p):
        ls = [oracle.slice_index_pair(p, r, i) for i in range(p)]
        assert sorted(ls) == list(range(p)) and ls[-1] == r


@pytest.mark.parametrize("p", [3, 5])
def test_pairwise_rejects_odd_p(p):
    with pytest.raises(ValueError):
        oracle.pair_partner(p, 0, 1)


@pytest.mark.parametrize("p,mc,n,k", [(2, 2, 3, 4), (4, 3, 7, 6), (6, 1, 5, 2), (8, 2, 5, 3)])
@pytest.mark.parametrize("integer", [True, False])
def test_pairwise_exactness(p, mc, n, k, integer):
    rng = np.random.default_rng(500 * p + mc + (7 if integer else 0))
    g = _rand_problem(rng, p, mc, n, k, integer)
    A = [g(p * mc, k) for _ in range(p)]
    W = [g(k, n) for _ in range(p)]
    want = oracle.rs_definition(A, W)
    got, received, sent = oracle.fuse_rs_pairwise_lockstep(A, W)
    Y = sum(np.matmul(A[q], W[q]) for q in range(p))
    for r in range(p):
        if integer:
            assert np.array_equal(got[r], want[r]) and np.array_equal(got[r], Y[r * mc:(r + 1) * mc])
        else:
            np.testing.assert_allclose(got[r], Y[r * mc:(r + 1) * mc], rtol=0, atol=1e-12 * max(1.0, np.abs(Y).max()))
        outs = oracle.rs_pair_rank_steps(A[r], W[r], received[r], p, r)
        for i in range(p - 1):
            assert np.array_equal(outs[i], sent[r][i])
        assert np.array_equal(outs[p - 1], got[r])


def test_pairwise_dp_rank():
    p, c, r = 4, 5, 2
    rng = np.random.default_rng(12)
    g = [rng.integers(-50, 51, size=p * c).astype(np.float64) for _ in range(p)]
    O, received, _ = oracle.fuse_rs_pairwise_lockstep(g, [None] * p, compute=lambda x, _w: np.asarray(x, dtype=np.float64).copy())
    want = oracle.dp_definition(g)
    for q in range(p):
        assert np.array_equal(O[q], want[q])
    out = oracle.dp_pair_rank(g[r], received[r], p, r)
    assert np.array_equal(out[r * c:(r + 1) * c], want[r])
    mask = np.ones(p * c, dtype=bool)
    mask[r * c:(r + 1) * c] = False
    assert np.array_equal(out[mask], g[r][mask])


# ----------------------------------------------------------------------------
# slicing granularity m > 1 (Sec. 3.2)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("p,m", [(1, 3), (2, 2), (3, 2), (4, 1), (4, 3), (8, 2)])
def test_granularity_index_invariants(p, m):
    S = m * p
    for r in range(p):
        rs = [oracle.subslice_index_rs(p, m, r, j) for j in range(S)]
        ag = [oracle.subslice_index_ag(p, m, r, j) for j in range(S)]
        assert sorted(rs) == list(range(S)) and sorted(ag) == list(range(S))
        assert rs[-m:] == [r * m + s for s in range(m)], "own sub-slices are computed in the last hop"
        assert ag[:m] == [r * m + s for s in range(m)], "own sub-slices are computed in the first hop"
        nxt = oracle.send_rank(p, r)
        for j in range(S - m):            # what r handles at sub-step j, its successor handles one hop later
            assert oracle.subslice_index_rs(p, m, nxt, j + m) == rs[j]
            assert oracle.subslice_index_ag(p, m, nxt, j + m) == ag[j]
        if m == 1:
            assert rs == [oracle.slice_index_rs(p, r, i) for i in range(p)]
            assert ag == [oracle.slice_index_ag(p, r, i) for i in range(p)]


@pytest.mark.parametrize("p,m,mc,n,k", [(2, 2, 4, 3, 5), (3, 2, 2, 5, 2), (4, 3, 6, 7, 6), (8, 2, 2, 5, 3), (1, 4, 8, 3, 2)])
@pytest.mark.parametrize("integer", [True, False])
def test_granularity_exactness(p, m, mc, n, k, integer):
    rng = np.random.default_rng(900 * p + m + (7 if integer else 0))
    g = _rand_problem(rng, p, mc, n, k, integer)
    A = [g(p * mc, k) for _ in range(p)]
    W = [g(k, n) for _ in range(p)]
    want = oracle.rs_definition(A, W)
    got, received, sent = oracle.fuse_rs_lockstep_m(A, W, m)
    base, _, base_sent = oracle.fuse_rs_lockstep(A, W)
    for r in range(p):
        # rows are independent, so cutting a slice into m row blocks changes no value at all
        assert np.array_equal(got[r], base[r])
        if integer:
            assert np.array_equal(got[r], want[r])
        else:
            np.testing.assert_allclose(got[r], want[r], rtol=0, atol=1e-12 * max(1.0, np.abs(want[r]).max()))
        for i in range(p - 1):
            joined = np.concatenate([sent[r][i * m + s] for s in range(m)], axis=0)
            assert np.array_equal(joined, base_sent[r][i])
        assert all(sent[r][j] is None for j in range((p - 1) * m, p * m)), "nothing is sent in the last hop"
        assert all(received[r][j] is None for j in range(m)), "nothing is received in the first hop"
        # one-rank view fed with what the lock-step run delivered
        R = [None] + [np.concatenate([received[r][i * m + s] for s in range(m)], axis=0) for i in range(1, p)]
        outs = oracle.rs_rank_steps_m(A[r], W[r], R, p, r, m)
        for j in range(m * p):
            ref = sent[r][j] if j < (p - 1) * m else got[r][(j % m) * (mc // m):(j % m + 1) * (mc // m)]
            assert np.array_equal(outs[j], ref)
    # all-gather side
    X = [g(mc, k) for _ in range(p)]
    Wc = [g(k, n) for _ in range(p)]
    wantg = oracle.ag_definition(X, Wc)
    gotg, held = oracle.fuse_ag_lockstep_m(X, Wc, m)
    baseg, _ = oracle.fuse_ag_lockstep(X, Wc)
    for r in range(p):
        assert np.array_equal(gotg[r], baseg[r])
        if integer:
            assert np.array_equal(gotg[r], wantg[r])
        S_in = [None] + [np.concatenate([held[r][i * m + s] for s in range(m)], axis=0) for i in range(1, p)]
        assert np.array_equal(oracle.ag_rank_m(X[r], S_in, Wc[r], p, r, m), gotg[r])
        for i in range(p):          # the slice in hand at hop i is rank (r - i)'s input
            joined = np.concatenate([held[r][i * m + s] for s in range(m)], axis=0)
            assert np.array_equal(joined, X[(r - i) % p])


def test_granularity_dp_rank():
    p, m, c, r = 4, 2, 6, 1
    rng = np.random.default_rng(31)
    g = [rng.integers(-50, 51, size=p * c).astype(np.float64) for _ in range(p)]
    O, received, _ = oracle.fuse_rs_lockstep_m(g, [None] * p, m, compute=lambda x, _w: np.asarray(x, dtype=np.float64).copy())
    want = oracle.dp_definition(g)
    for q in range(p):
        assert np.array_equal(O[q], want[q])
    R = [None] + [np.concatenate([received[r][i * m + s] for s in range(m)]) for i in range(1, p)]
    out = oracle.dp_rank_m(g[r], R, p, r, m)
    assert np.array_equal(out[r * c:(r + 1) * c], want[r])
    assert np.array_equal(out, oracle.dp_rank(g[r], R, p, r)), "granularity changes no value of the gradient path"


# ----------------------------------------------------------------------------
# backward pass: gradients against central finite differences of the forward definition
# ----------------------------------------------------------------------------

def _fd_grad(f, x, eps=1e-6):
    """Central finite differences of the scalar function f at x (flat loop; tiny inputs only)."""
    g = np.zeros_like(x)
    flat, gf = x.reshape(-1), g.reshape(-1)
    for idx in range(flat.size):
        old = flat[idx]
        flat[idx] = old + eps
        up = f()
        flat[idx] = old - eps
        dn = f()
        flat[idx] = old
        gf[idx] = (up - dn) / (2 * eps)
    return g


@pytest.mark.parametrize("p,mc,n,k", [(2, 2, 3, 2), (3, 1, 2, 3), (4, 2, 2, 2)])
def test_backward_matches_finite_differences(p, mc, n, k):
    rng = np.random.default_rng(70 + p)
    # all-gather layer: X^r [mc x k], W^r [k x n], Y^r [p*mc x n]
    X = [rng.standard_normal((mc, k)) for _ in range(p)]
    W = [rng.standard_normal((k, n)) for _ in range(p)]
    C = [rng.standard_normal((p * mc, n)) for _ in range(p)]          # dL/dY^r for L = sum <Y^r, C^r>
    loss = lambda: sum(float(np.sum(y * c)) for y, c in zip(oracle.ag_layer_forward(X, W), C))
    dX, dW = oracle.ag_layer_backward_definition(X, W, C)
    fX, fW = oracle.fuse_ag_layer_backward(X, W, C)
    for r in range(p):
        np.testing.assert_allclose(dX[r], _fd_grad(loss, X[r]), rtol=0, atol=1e-6)
        np.testing.assert_allclose(dW[r], _fd_grad(loss, W[r]), rtol=0, atol=1e-6)
        np.testing.assert_allclose(fX[r], dX[r], rtol=0, atol=1e-12)
        np.testing.assert_allclose(fW[r], dW[r], rtol=0, atol=1e-12)
    # reduce-scatter layer: A^r [p*mc x k], W^r [k x n], Y^r [mc x n]
    A = [rng.standard_normal((p * mc, k)) for _ in range(p)]
    C = [rng.standard_normal((mc, n)) for _ in range(p)]
    loss = lambda: sum(float(np.sum(y * c)) for y, c in zip(oracle.rs_layer_forward(A, W), C))
    dA, dW = oracle.rs_layer_backward_definition(A, W, C)
    fA, fW = oracle.fuse_rs_layer_backward(A, W, C)
    for r in range(p):
        np.testing.assert_allclose(dA[r], _fd_grad(loss, A[r]), rtol=0, atol=1e-6)
        np.testing.assert_allclose(dW[r], _fd_grad(loss, W[r]), rtol=0, atol=1e-6)
        np.testing.assert_allclose(fA[r], dA[r], rtol=0, atol=1e-12)
        np.testing.assert_allclose(fW[r], dW[r], rtol=0, atol=1e-12)


@pytest.mark.parametrize("p", [1, 2, 4, 8])
def test_backward_fused_is_exact_on_integers(p):
    mc, n, k = 3, 4, 5
    rng = np.random.default_rng(80 + p)
    g = lambda *s: rng.integers(-4, 5, size=s).astype(np.float64)
    X, W, G = [g(mc, k) for _ in range(p)], [g(k, n) for _ in range(p)], [g(p * mc, n) for _ in range(p)]
    dX, dW = oracle.ag_layer_backward_definition(X, W, G)
    fX, fW = oracle.fuse_ag_layer_backward(X, W, G)
    Xf = np.concatenate(X)
    for r in range(p):
        assert np.array_equal(fX[r], dX[r]) and np.array_equal(fW[r], dW[r])
        assert np.array_equal(dW[r], Xf.T @ G[r])                     # against the library product
        assert np.array_equal(dX[r], sum(G[q] @ W[q].T for q in range(p))[r * mc:(r + 1) * mc])
        # one-rank view of the weight-gradient loop, fed what Alg. 1 hands the rank
        moving = [X[(r - i) % p] for i in range(p)]
        assert np.array_equal(oracle.wgrad_rank_steps(moving, G[r], p, r, True)[-1], dW[r])
    A, G2 = [g(p * mc, k) for _ in range(p)], [g(mc, n) for _ in range(p)]
    dA, dW = oracle.rs_layer_backward_definition(A, W, G2)
    fA, fW = oracle.fuse_rs_layer_backward(A, W, G2)
    Gf = np.concatenate(G2)
    for r in range(p):
        assert np.array_equal(fA[r], dA[r]) and np.array_equal(fW[r], dW[r])
        assert np.array_equal(dW[r], A[r].T @ Gf) and np.array_equal(dA[r], Gf @ W[r].T)
        moving = [G2[(r - i) % p] for i in range(p)]
        assert np.array_equal(oracle.wgrad_rank_steps(moving, A[r], p, r, False)[-1], dW[r])


# ----------------------------------------------------------------------------
# query-split attention (Alg. 4)
# ----------------------------------------------------------------------------

def _brute_attention(Q, K, V, scale):
    """Pure-Python loops: softmax(Q K^T * scale) V for [S x Dh] operands."""
    import math
    S, Dh = len(Q), len(Q[0])
    out = [[0.0] * Dh for _ in range(S)]
    for i in range(S):
        logits = [scale * sum(Q[i][d] * K[j][d] for d in range(Dh)) for j in range(len(K))]
        m = max(logits)
        e = [math.exp(x - m) for x in logits]
        z = sum(e)
        for d in range(Dh):
            out[i][d] = sum(e[j] / z * V[j][d] for j in range(len(K)))
    return out


def test_attention_slice_against_brute_force_and_closed_forms():
    rng = np.random.default_rng(200)
    B, h, S, Dh, N = 2, 3, 8, 4, 4
    Q, K, V = (rng.standard_normal((B, h, S, Dh)) for _ in range(3))
    scale = 1.0 / np.sqrt(Dh)
    for l in range(N):
        got = oracle.attention_slice(Q, K, V, l, N, scale)
        c = S // N
        assert got.shape == (B * c, h * Dh)
        for b in range(B):
            for a in range(h):
                want = _brute_attention(Q[b, a, l * c:(l + 1) * c].tolist(), K[b, a].tolist(), V[b, a].tolist(), scale)
                np.testing.assert_allclose(got[b * c:(b + 1) * c, a * Dh:(a + 1) * Dh], np.array(want), rtol=0, atol=1e-12)
    # zero queries: every key weighs 1/S, the output is the mean of V
    got = oracle.attention_slice(np.zeros_like(Q), K, V, 0, 1, scale)
    np.testing.assert_allclose(got.reshape(B, S, h, Dh), np.broadcast_to(V.mean(axis=2)[:, None], (B, S, h, Dh)), atol=1e-12)
    # one key far more similar than the rest: the output is that key's value row
    Kh = np.zeros((1, 1, S, Dh)); Kh[0, 0, 5] = 1.0
    Qh = np.full((1, 1, S, Dh), 50.0)
    got = oracle.attention_slice(Qh, Kh, V[:1, :1], 0, 1, 1.0)
    np.testing.assert_allclose(got, np.broadcast_to(V[0, 0, 5], (S, Dh)), atol=1e-9)
    # keys and values permuted together: nothing changes; the scale matters (a dropped scale is caught)
    perm = rng.permutation(S)
    a0 = oracle.attention_slice(Q, K, V, 1, 2, scale)
    np.testing.assert_allclose(oracle.attention_slice(Q, K[:, :, perm], V[:, :, perm], 1, 2, scale), a0, atol=1e-12)
    assert np.abs(oracle.attention_slice(Q, K, V, 1, 2, 1.0) - a0).max() > 1e-3
    w = oracle.softmax_rows(rng.standard_normal((5, 7)) * 30)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-12)


@pytest.mark.parametrize("p", [1, 2, 4])
def test_query_split_attention_exactness(p):
    """Alg. 4 decomposed == every rank's full attention + projection, reduce-scattered == the unsharded layer."""
    rng = np.random.default_rng(210 + p)
    B, h, S, Dh, D = 2, 2, 8, 4, 6
    scale = 0.5
    Q, K, V = ([rng.standard_normal((B, h, S, Dh)) for _ in range(p)] for _ in range(3))
    Wo = [rng.standard_normal((h * Dh, D)) for _ in range(p)]
    want = oracle.attn_rs_definition(Q, K, V, Wo, scale)
    got, received, sent = oracle.fuse_attn_rs_lockstep(Q, K, V, Wo, scale)
    # the unsharded layer: all p*h heads on one device, one projection with the stacked W_o
    Qa, Ka, Va = (np.concatenate(x, axis=1) for x in (Q, K, V))
    full = oracle.attention_slice(Qa, Ka, Va, 0, 1, scale) @ np.concatenate(Wo, axis=0)          # tokens (b, s)
    c = S // p
    for r in range(p):
        np.testing.assert_allclose(got[r], want[r], rtol=0, atol=1e-12)
        rows = [b * S + r * c + s for b in range(B) for s in range(c)]
        np.testing.assert_allclose(got[r], full[rows], rtol=0, atol=1e-11)
        outs = oracle.attn_rs_rank_steps(Q[r], K[r], V[r], Wo[r], received[r], p, r, scale, round_attn=False)
        for i in range(p - 1):
            np.testing.assert_allclose(outs[i], sent[r][i], rtol=0, atol=1e-12)
        np.testing.assert_allclose(outs[p - 1], got[r], rtol=0, atol=1e-12)
        assert sent[r][p - 1] is None and received[r][0] is None

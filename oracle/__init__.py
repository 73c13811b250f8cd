"""CommFuse CPU oracle (TEST INFRASTRUCTURE ONLY -- never on the product path).

A plain, slow, fp64 statement of what the decomposed, ring-ordered, fused
computation of the paper must produce.  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; the GPU library
and its Python binding never do, and this package imports neither of them.

Two levels are provided.

* Definitions (Sec. 3.1, "Common collective communications"; Sec. 4.1 and 4.2):
  the undecomposed result -- a dense product followed by a reduce-scatter, an
  all-gather followed by a dense product, a reduce-scatter of gradients.
  The paper states its method is exact, so these ARE the expected values.
* Lock-step simulations of Alg. 1 (FuseAllGather) and Alg. 2 / Alg. 3
  (FuseReduceScatter, row-parallel projection) for all ``p`` ranks with an
  in-memory mailbox standing for the P2P transfers, in the algorithms' own
  order and notation (``r`` rank, ``i`` step, ``j`` send-to, ``k`` recv-from,
  ``l`` slice index, ``B_in`` / ``B_out`` buffers).  They are checked against
  the definitions; they also yield what every rank receives at every step,
  which is what the one-rank views below take as their ``R_i`` / ``S_i``.
* One-rank views: what a single rank ``r`` computes at each step when the
  data delivered by rank ``r-1`` is handed in as an input.

Readings of the paper taken here (each is listed in the design notes):
the slice list of Alg. 2 is the input ``X^r`` cut into ``N`` equal row blocks;
Alg. 3's compute line uses slice ``l`` (not the send rank ``j``);
``compute_partial_output(X, W) = X @ W`` with activations on the left;
``N = T = p`` (slicing granularity ``m = 1``); a receive posted at step ``i-1``
is complete before ``B_in`` is read at step ``i``.

Pins (see tests): the paper's 4-rank all-gather / reduce-scatter examples,
the Appendix A(b) round-by-round trace, the exactness claim, closed-form
index invariants, numpy.matmul on special cases, and a pure-Python brute
force.  Nothing in this file is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcf_oracle.so")
_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(
        os.path.join(_HERE, "cf_oracle.c")
    ):
        from . import build as _b

        _b.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    dp = ctypes.POINTER(ctypes.c_double)
    i64 = ctypes.c_int64
    lib.cfo_gemm_f64.argtypes = [dp, i64, dp, i64, dp, i64, i64, i64, i64]
    lib.cfo_gemm_f64.restype = None
    lib.cfo_dot_f64.argtypes = [dp, i64, dp, i64, i64, i64, i64]
    lib.cfo_dot_f64.restype = ctypes.c_double
    lib.cfo_add_f64.argtypes = [dp, dp, dp, i64]
    lib.cfo_add_f64.restype = None
    lib.cfo_num_threads.argtypes = []
    lib.cfo_num_threads.restype = ctypes.c_int
    _lib = lib
    return lib


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def num_threads() -> int:
    """Threads the C loops use (OpenMP's max threads)."""
    return int(_load().cfo_num_threads())


# ---------------------------------------------------------------------------
# Elementary pieces
# ---------------------------------------------------------------------------

def gemm(X, W) -> np.ndarray:
    """``compute_partial_output`` of a linear projection: ``X @ W`` in fp64.

    Sec. 4.1 (row-sharded projection) and Sec. 4.2 (column-sharded projection);
    activations on the left, ``X[M x K]``, ``W[K x N]``.  Triple loop in C.
    """
    X = _f64(X)
    W = _f64(W)
    if X.ndim != 2 or W.ndim != 2 or X.shape[1] != W.shape[0]:
        raise ValueError(f"gemm shape mismatch {X.shape} @ {W.shape}")
    M, K = X.shape
    N = W.shape[1]
    O = np.empty((M, N), dtype=np.float64)
    if M and N:
        _load().cfo_gemm_f64(_dptr(X), max(K, 1), _dptr(W), max(N, 1), _dptr(O), N, M, N, K)
    return O


def dot_element(X, W, i: int, j: int) -> float:
    """One element ``(X @ W)[i, j]`` from its definition (for sampled checks)."""
    X = _f64(X)
    W = _f64(W)
    return float(_load().cfo_dot_f64(_dptr(X), X.shape[1], _dptr(W), W.shape[1], i, j, X.shape[1]))


def add(a, b) -> np.ndarray:
    """``B_in + O`` of Alg. 2, element by element in fp64."""
    a = _f64(a)
    b = _f64(b)
    if a.shape != b.shape:
        raise ValueError("add shape mismatch")
    out = np.empty_like(a)
    if a.size:
        _load().cfo_add_f64(_dptr(a), _dptr(b), _dptr(out), a.size)
    return out


def round_to_bf16(x) -> np.ndarray:
    """Round fp64 values to the nearest bfloat16 (ties to even), returned as fp64.

    Used only for the chained AG-GEMM -> GEMM-RS pair, where the intermediate
    activations are handed over in bf16.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


# ---------------------------------------------------------------------------
# Index functions of the two algorithms
# ---------------------------------------------------------------------------

def send_rank(p: int, r: int) -> int:
    """``j = (r + 1) mod N`` (Alg. 1 and Alg. 2)."""
    return (r + 1) % p


def recv_rank(p: int, r: int) -> int:
    """``k = (r - 1 + N) mod N`` (Alg. 1 and Alg. 2)."""
    return (r - 1 + p) % p


def slice_index_ag(p: int, r: int, i: int) -> int:
    """``l = (r - i + N) mod N`` (Alg. 1): own slice first."""
    return (r - i + p) % p


def slice_index_rs(p: int, r: int, i: int) -> int:
    """``l = (r - i - 1 + N) mod N`` (Alg. 2): own slice last."""
    return (r - i - 1 + p) % p


def split_rows(X, p: int) -> List[np.ndarray]:
    """``init_sequence_as_sequence_list(X, N)``: N equal blocks along the sequence (row) axis."""
    X = np.asarray(X)
    if X.shape[0] % p:
        raise ValueError("rows not divisible by p")
    mc = X.shape[0] // p
    return [X[c * mc:(c + 1) * mc] for c in range(p)]


# ---------------------------------------------------------------------------
# Collectives, by definition (Sec. 3.1)
# ---------------------------------------------------------------------------

def all_gather(per_rank: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Every rank ends with the concatenation, in rank order, of all ranks' data."""
    full = np.concatenate([np.asarray(x) for x in per_rank], axis=0)
    return [full.copy() for _ in per_rank]


def reduce_scatter(per_rank_slices: Sequence[Sequence[np.ndarray]]) -> List[np.ndarray]:
    """Rank ``c`` ends with the sum over ranks ``q`` of slice ``c`` of rank ``q``."""
    p = len(per_rank_slices)
    out = []
    for c in range(p):
        acc = np.zeros_like(np.asarray(per_rank_slices[0][c], dtype=np.float64))
        for q in range(p):
            acc = acc + np.asarray(per_rank_slices[q][c], dtype=np.float64)
        out.append(acc)
    return out


# ---------------------------------------------------------------------------
# Definitions of the three paths (undecomposed)
# ---------------------------------------------------------------------------

def rs_definition(A_list: Sequence[np.ndarray], W_list: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Row-parallel projection then reduce-scatter (Sec. 4.1 with Sec. 3.1).

    Rank ``q`` holds ``A^q[M x K_q]`` and ``W^q[K_q x N]``; the full partial
    product ``A^q @ W^q`` is cut into ``p`` row blocks and reduce-scattered.
    """
    p = len(A_list)
    partial = [split_rows(gemm(A_list[q], W_list[q]), p) for q in range(p)]
    return reduce_scatter(partial)


def ag_definition(X_list: Sequence[np.ndarray], W_list: Sequence[np.ndarray]) -> List[np.ndarray]:
    """All-gather of sequence shards, then column-parallel projection (Sec. 4.2)."""
    gathered = all_gather([_f64(x) for x in X_list])
    return [gemm(gathered[r], W_list[r]) for r in range(len(X_list))]


def dp_definition(g_list: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Reduce-scatter of the gradient buckets of ``p`` data-parallel ranks (Sec. 3.1, Zero-DP)."""
    p = len(g_list)
    return reduce_scatter([split_rows(np.asarray(g, dtype=np.float64), p) for g in g_list])


# ---------------------------------------------------------------------------
# Lock-step simulation of the algorithms over all p ranks
# ---------------------------------------------------------------------------

Compute = Callable[[np.ndarray, np.ndarray], np.ndarray]


def fuse_rs_lockstep(
    X_list: Sequence[np.ndarray],
    W_list: Sequence[Optional[np.ndarray]],
    compute: Optional[Compute] = None,
) -> Tuple[List[np.ndarray], List[List[Optional[np.ndarray]]], List[List[Optional[np.ndarray]]]]:
    """Alg. 2 (FuseReduceScatter) run by all ranks in lock-step.

    Returns ``(O, received, sent)``: ``O[r]`` is rank ``r``'s result;
    ``received[r][i]`` is the content of ``B_in`` that rank ``r`` adds at step
    ``i`` (``None`` at ``i = 0``); ``sent[r][i]`` is ``B_out`` after step ``i``
    (``None`` at the last step, where nothing is sent).
    """
    if compute is None:
        compute = gemm
    N = len(X_list)
    X_s = [split_rows(X_list[r], N) for r in range(N)]
    B_in: List[Optional[np.ndarray]] = [None] * N
    O: List[Optional[np.ndarray]] = [None] * N
    received = [[None] * N for _ in range(N)]
    sent = [[None] * N for _ in range(N)]
    for i in range(N):
        in_flight: List[Optional[np.ndarray]] = [None] * N
        for r in range(N):
            j = send_rank(N, r)
            l = slice_index_rs(N, r, i)
            O[r] = compute(X_s[r][l], W_list[r])
            if i > 0:
                received[r][i] = B_in[r]
                O[r] = add(B_in[r], O[r])
            if i < N - 1:
                B_out = O[r].copy()
                sent[r][i] = B_out
                in_flight[j] = B_out          # p2p_send to j == p2p_recv at j from its k
        B_in = in_flight                        # transfers of step i land before step i+1 reads
    return [o for o in O], received, sent


def fuse_ag_lockstep(
    X_list: Sequence[np.ndarray],
    W_list: Sequence[np.ndarray],
    compute: Optional[Compute] = None,
) -> Tuple[List[np.ndarray], List[List[Optional[np.ndarray]]]]:
    """Alg. 1 (FuseAllGather) run by all ranks in lock-step.

    Returns ``(O, held)``: ``O[r]`` is the concatenated output of rank ``r``;
    ``held[r][i]`` is the slice in ``B_out`` that rank ``r`` multiplies at step ``i``
    (its own ``X^r`` at ``i = 0``, then what rank ``r-1`` forwarded).
    """
    if compute is None:
        compute = gemm
    N = len(X_list)
    B_out = [_f64(X_list[r]) for r in range(N)]
    O_s: List[List[Optional[np.ndarray]]] = [[None] * N for _ in range(N)]
    held = [[None] * N for _ in range(N)]
    for i in range(N):
        B_in: List[Optional[np.ndarray]] = [None] * N
        for r in range(N):
            j = send_rank(N, r)
            l = slice_index_ag(N, r, i)
            if i < N - 1:
                B_in[j] = B_out[r]              # send what is in hand, neighbour receives it
            held[r][i] = B_out[r]
            O_s[r][l] = compute(B_out[r], W_list[r])
        if i < N - 1:
            B_out = B_in                         # after the wait: forward the received slice
    O = [np.concatenate(O_s[r], axis=0) for r in range(N)]
    return O, held


def fuse_dp_lockstep(g_list: Sequence[np.ndarray]):
    """Alg. 2 with ``compute_partial_output`` = "take slice ``l`` of the local gradient bucket".

    The paper gives no separate data-parallel algorithm; this is the reading
    used for the gradient path.  Returns ``(O, received, sent)`` as :func:`fuse_rs_lockstep`.
    """
    return fuse_rs_lockstep(g_list, [None] * len(g_list), compute=lambda x, _w: _f64(x).copy())


# ---------------------------------------------------------------------------
# One-rank views: rank r alone, neighbour traffic handed in
# ---------------------------------------------------------------------------

def rs_rank_steps(A, W, R: Sequence[Optional[np.ndarray]], p: int, r: int) -> List[np.ndarray]:
    """What rank ``r`` holds after each step of Alg. 2 / Alg. 3.

    ``A[p*M_c x K]`` local activations, ``W[K x N]`` row shard, ``R[i]`` the
    partial sum received for step ``i`` (``R[0]`` is ignored).  ``out[i]`` is
    ``B_out`` for ``i < p-1`` and the result ``O^r`` for ``i = p-1``.
    """
    X_s = split_rows(_f64(A), p)
    outs = []
    for i in range(p):
        l = slice_index_rs(p, r, i)
        O = gemm(X_s[l], W)
        if i > 0:
            O = add(_f64(R[i]), O)
        outs.append(O)
    return outs


def ag_rank(X_own, S: Sequence[Optional[np.ndarray]], W, p: int, r: int) -> np.ndarray:
    """Rank ``r``'s output of Alg. 1: slice ``l_i`` of ``O`` is ``T_i @ W`` with
    ``T_0 = X^r`` and ``T_i = S[i]`` (the slice received for step ``i``)."""
    O_s: List[Optional[np.ndarray]] = [None] * p
    for i in range(p):
        l = slice_index_ag(p, r, i)
        T = _f64(X_own) if i == 0 else _f64(S[i])
        O_s[l] = gemm(T, W)
    return np.concatenate(O_s, axis=0)


def dp_rank(bucket, R: Sequence[Optional[np.ndarray]], p: int, r: int) -> np.ndarray:
    """Gradient bucket of rank ``r`` after its ``p`` steps: at step ``i >= 1`` slice
    ``l_i = (r-i-1) mod p`` becomes ``R[i] + slice``; step 0 only sends."""
    out = _f64(bucket).copy()
    n = out.shape[0]
    if n % p:
        raise ValueError("bucket length not divisible by p")
    c = n // p
    for i in range(1, p):
        l = slice_index_rs(p, r, i)
        out[l * c:(l + 1) * c] = add(_f64(R[i]), out[l * c:(l + 1) * c])
    return out


def mlp_pair_rank(X_own, S, W_up, W_down, R, p: int, r: int):
    """Chained pair on rank ``r``: AG-GEMM (up) producing ``H``, rounded to bf16 for
    the hand-over, then GEMM-RS (down) on ``H``.  No activation function and no
    gate sit between them (the paper states none).  Returns ``(H_bf16, outs)``."""
    H = round_to_bf16(ag_rank(X_own, S, W_up, p, r))
    return H, rs_rank_steps(H, W_down, R, p, r)


# ---------------------------------------------------------------------------
# Pairwise bidirectional P2P schedule (Appendix A, subsection (a))
# ---------------------------------------------------------------------------
# The appendix decomposes the n(n-1) sends of a reduce-scatter into n-1 rounds of n/2 simultaneous
# bidirectional exchanges ("round-robin tournament"): in every round each device sends its partial
# of the PARTNER's slice straight to the partner (its owner) and receives the partner's partial of
# its own slice.  The paper prints the pairing only for four devices:
#   round 1 (A,B)(C,D); round 2 (A,C)(B,D); round 3 (A,D)(B,C).
# Reading taken for general even n: for n a power of two, partner = rank XOR round (this reproduces
# the printed table); for other even n the circle method of round-robin tournaments.  Odd n is not
# defined by the paper ("completion in n-1 rounds (for even n)") and is rejected.
# The computes are ordered like Alg. 2's: the partials that travel first are computed first, the
# rank's own slice last, so that nothing is left to send after the last compute.

def pair_partner(p: int, r: int, t: int) -> int:
    """Partner of rank ``r`` in round ``t`` (1 .. p-1) of the pairwise schedule."""
    if p < 2 or p % 2 or not (1 <= t <= p - 1) or not (0 <= r < p):
        raise ValueError("pairwise schedule needs even p >= 2, round in [1, p-1], rank in [0, p)")
    if p & (p - 1) == 0:
        return r ^ t
    a = t - 1                                   # circle method: rank p-1 is fixed, the others rotate
    if r == p - 1:
        return a
    if r == a:
        return p - 1
    return (2 * a - r) % (p - 1)


def slice_index_pair(p: int, r: int, i: int) -> int:
    """Slice computed at step ``i``: the partner of round ``i+1`` for ``i < p-1``, the own slice last."""
    if p == 1:
        return 0
    return r if i == p - 1 else pair_partner(p, r, i + 1)


def fuse_rs_pairwise_lockstep(X_list, W_list, compute: Optional[Compute] = None):
    """All ranks run the pairwise schedule in lock-step.

    Returns ``(O, received, sent)``: ``O[r]`` the reduced slice ``r``; ``received[r][t]`` what rank
    ``r`` receives in round ``t`` (index 0 unused); ``sent[r][i]`` the partial computed at step ``i``
    and sent in round ``i+1`` (``None`` at the last step).
    """
    if compute is None:
        compute = gemm
    N = len(X_list)
    X_s = [split_rows(X_list[r], N) for r in range(N)]
    sent = [[None] * N for _ in range(N)]
    received = [[None] * N for _ in range(N)]
    acc: List[Optional[np.ndarray]] = [None] * N
    O: List[Optional[np.ndarray]] = [None] * N
    for i in range(N):
        for r in range(N):                      # step i: every rank computes one partial
            l = slice_index_pair(N, r, i)
            part = compute(X_s[r][l], W_list[r])
            if i < N - 1:
                sent[r][i] = part               # goes to its owner l in round i+1
            else:
                O[r] = part if acc[r] is None else add(acc[r], part)   # own slice: add what was received
        if i < N - 1:
            t = i + 1                           # round t: exchange with the partner
            for r in range(N):
                q = pair_partner(N, r, t)
                got = sent[q][i]                # q computed its partial of slice r at step i
                received[r][t] = got
                acc[r] = got.copy() if acc[r] is None else add(acc[r], got)
    return O, received, sent


def rs_pair_rank_steps(A, W, R: Sequence[Optional[np.ndarray]], p: int, r: int):
    """One-rank view of the pairwise schedule: ``outs[i]`` is the partial sent after step ``i``
    (``i < p-1``) and ``outs[p-1]`` the result ``X_s[r] @ W + sum_t R[t]`` (``R[t]``: received in round t)."""
    X_s = split_rows(_f64(A), p)
    outs = []
    acc = None
    for i in range(p):
        if i >= 1:
            acc = _f64(R[i]).copy() if acc is None else add(acc, _f64(R[i]))
        part = gemm(X_s[slice_index_pair(p, r, i)], W)
        outs.append(part if (i < p - 1 or acc is None) else add(acc, part))
    return outs


def dp_pair_rank(bucket, R: Sequence[Optional[np.ndarray]], p: int, r: int) -> np.ndarray:
    """Gradient bucket of rank ``r`` after the pairwise schedule: its own slice ``r`` has received
    ``R[1] .. R[p-1]``; the other slices (sent away) are untouched."""
    out = _f64(bucket).copy()
    c = out.shape[0] // p
    for t in range(1, p):
        out[r * c:(r + 1) * c] = add(_f64(R[t]), out[r * c:(r + 1) * c])
    return out


# ---------------------------------------------------------------------------
# Slicing granularity m > 1 (Sec. 3.2, last sentences of its first paragraph)
# ---------------------------------------------------------------------------
# The sequence is cut into m * T slices for T ranks; the paper sets m = 1 and prints no index
# formulas for m > 1 (Alg. 1 / Alg. 2 use one "N" for both the ranks and the slices).
# Reading taken: the ring and its T hops stay as they are; the slice a rank handles at hop i
# (index l of Alg. 1 / Alg. 2) is cut into m sub-slices that are processed, aggregated and sent on
# one after the other, sub-step j = i*m + s handling sub-slice c = l*m + s of the m*T.  What is
# received for sub-step j is what the predecessor produced at sub-step j - m.

def subslice_index_rs(p: int, m: int, r: int, j: int) -> int:
    return slice_index_rs(p, r, j // m) * m + (j % m)


def subslice_index_ag(p: int, m: int, r: int, j: int) -> int:
    return slice_index_ag(p, r, j // m) * m + (j % m)


def fuse_rs_lockstep_m(X_list, W_list, m: int, compute: Optional[Compute] = None):
    """Alg. 2 with slicing granularity ``m``, all ranks in lock-step.

    Returns ``(O, received, sent)``; ``O[r]`` is the rank's result (its ``m`` sub-slices joined);
    ``received[r][j]`` / ``sent[r][j]`` per sub-step ``j`` in ``[0, m*T)`` (``None`` where nothing
    is received / sent: the first and the last hop).
    """
    if compute is None:
        compute = gemm
    T = len(X_list)
    S = m * T
    X_s = [split_rows(X_list[r], S) for r in range(T)]
    mailbox = [dict() for _ in range(T)]                 # per rank: sub-step -> arrived partial
    received = [[None] * S for _ in range(T)]
    sent = [[None] * S for _ in range(T)]
    final = [[None] * m for _ in range(T)]
    for j in range(S):
        i, s = divmod(j, m)
        posted = []
        for r in range(T):
            c = subslice_index_rs(T, m, r, j)
            O = compute(X_s[r][c], W_list[r])
            if i > 0:
                received[r][j] = mailbox[r].pop(j)
                O = add(received[r][j], O)
            if i < T - 1:
                sent[r][j] = O.copy()
                posted.append((send_rank(T, r), j + m, sent[r][j]))   # needed there one hop later
            else:
                final[r][s] = O
        for dst, when, buf in posted:
            mailbox[dst][when] = buf
    assert all(not mb for mb in mailbox), "every transfer was consumed"
    return [np.concatenate(f, axis=0) for f in final], received, sent


def fuse_ag_lockstep_m(X_list, W_list, m: int, compute: Optional[Compute] = None):
    """Alg. 1 with slicing granularity ``m``.  Returns ``(O, held)``; ``held[r][j]`` is the
    sub-slice rank ``r`` multiplies at sub-step ``j``."""
    if compute is None:
        compute = gemm
    T = len(X_list)
    S = m * T
    own = [split_rows(X_list[r], m) for r in range(T)]
    mailbox = [dict() for _ in range(T)]
    held = [[None] * S for _ in range(T)]
    O_s = [[None] * S for _ in range(T)]
    for j in range(S):
        i, s = divmod(j, m)
        posted = []
        for r in range(T):
            in_hand = own[r][s] if i == 0 else mailbox[r].pop(j)
            held[r][j] = in_hand
            if i < T - 1:
                posted.append((send_rank(T, r), j + m, in_hand))
            O_s[r][subslice_index_ag(T, m, r, j)] = compute(in_hand, W_list[r])
        for dst, when, buf in posted:
            mailbox[dst][when] = buf
    assert all(not mb for mb in mailbox)
    return [np.concatenate(O_s[r], axis=0) for r in range(T)], held


def rs_rank_steps_m(A, W, R: Sequence[Optional[np.ndarray]], p: int, r: int, m: int) -> List[np.ndarray]:
    """One-rank view with granularity ``m``: ``R[i]`` (hop ``i >= 1``) holds the ``m`` sub-partials of
    that hop stacked by rows; returns the output of every sub-step."""
    X_s = split_rows(_f64(A), m * p)
    outs = []
    for j in range(m * p):
        i, s = divmod(j, m)
        O = gemm(X_s[subslice_index_rs(p, m, r, j)], W)
        if i > 0:
            O = add(split_rows(_f64(R[i]), m)[s], O)
        outs.append(O)
    return outs


def ag_rank_m(X_own, S_in: Sequence[Optional[np.ndarray]], W, p: int, r: int, m: int) -> np.ndarray:
    """One-rank view of Alg. 1 with granularity ``m``: ``S_in[i]`` is the slice delivered for hop ``i``."""
    blocks = [None] * (m * p)
    for j in range(m * p):
        i, s = divmod(j, m)
        src = _f64(X_own) if i == 0 else _f64(S_in[i])
        blocks[subslice_index_ag(p, m, r, j)] = gemm(split_rows(src, m)[s], W)
    return np.concatenate(blocks, axis=0)


def dp_rank_m(bucket, R: Sequence[Optional[np.ndarray]], p: int, r: int, m: int) -> np.ndarray:
    out = _f64(bucket).copy()
    c = out.shape[0] // (m * p)
    for j in range(m, m * p):
        i, s = divmod(j, m)
        k = subslice_index_rs(p, m, r, j)
        out[k * c:(k + 1) * c] = add(_f64(R[i])[s * c:(s + 1) * c], out[k * c:(k + 1) * c])
    return out


# ---------------------------------------------------------------------------
# Backward pass of the two TPSP layers
# ---------------------------------------------------------------------------
# The paper states that TPSP involves reduce-scatter and all-gather in the forward AND the backward
# pass (Sec. 1) and prints no backward algorithm.  Reading taken: the textbook gradients of the two
# layers, each collective of which is decomposed by the same two loops:
#   all-gather layer   Y^r = AG(X) W^r :  dX^r = RS_r( G^r (W^r)^T )      -> Alg. 2 with W^T
#                                         dW^r = AG(X)^T G^r              -> Alg. 1's loop, the slice in hand
#                                                                            multiplied (transposed) into dW
#   reduce-scatter layer Y^r = RS_r(A^q W^q): dA^r = AG(G) (W^r)^T        -> Alg. 1 with W^T
#                                         dW^r = (A^r)^T AG(G)            -> Alg. 1's loop over the arriving G
# with G^r = dL/dY^r.  The weight gradient is a sum over the sequence slices; it is accumulated in the
# order in which Alg. 1 meets them (l = (r - i) mod N).

def ag_layer_forward(X_list, W_list):
    return ag_definition(X_list, W_list)


def rs_layer_forward(A_list, W_list):
    return rs_definition(A_list, W_list)


def ag_layer_backward_definition(X_list, W_list, G_list):
    """Gradients of the all-gather layer, dense: returns ``(dX, dW)`` per rank."""
    N = len(X_list)
    X_full = np.concatenate([_f64(x) for x in X_list], axis=0)
    dX_full = None
    for r in range(N):
        term = gemm(_f64(G_list[r]), np.ascontiguousarray(_f64(W_list[r]).T))
        dX_full = term if dX_full is None else add(dX_full, term)
    dX = split_rows(dX_full, N)
    dW = [gemm(np.ascontiguousarray(X_full.T), _f64(G_list[r])) for r in range(N)]
    return dX, dW


def rs_layer_backward_definition(A_list, W_list, G_list):
    """Gradients of the reduce-scatter layer, dense: returns ``(dA, dW)`` per rank."""
    N = len(A_list)
    G_full = np.concatenate([_f64(g) for g in G_list], axis=0)
    dA = [gemm(G_full, np.ascontiguousarray(_f64(W_list[r]).T)) for r in range(N)]
    dW = [gemm(np.ascontiguousarray(_f64(A_list[r]).T), G_full) for r in range(N)]
    return dA, dW


def fuse_ag_layer_backward(X_list, W_list, G_list):
    """The same gradients through the decomposed loops, all ranks in lock-step."""
    N = len(X_list)
    dX, _, _ = fuse_rs_lockstep(G_list, [np.ascontiguousarray(_f64(w).T) for w in W_list])
    # weight gradient: Alg. 1's loop; the compute on the slice in hand adds its contribution to dW
    _, held = fuse_ag_lockstep(X_list, [None] * N, compute=lambda x, _w: x)
    dW = []
    for r in range(N):
        G_s = split_rows(_f64(G_list[r]), N)
        acc = None
        for i in range(N):
            l = slice_index_ag(N, r, i)
            term = gemm(np.ascontiguousarray(_f64(held[r][i]).T), G_s[l])
            acc = term if acc is None else add(acc, term)
        dW.append(acc)
    return dX, dW


def fuse_rs_layer_backward(A_list, W_list, G_list):
    N = len(A_list)
    dA, held = fuse_ag_lockstep(G_list, [np.ascontiguousarray(_f64(w).T) for w in W_list])
    dW = []
    for r in range(N):
        A_s = split_rows(_f64(A_list[r]), N)
        acc = None
        for i in range(N):
            l = slice_index_ag(N, r, i)
            term = gemm(np.ascontiguousarray(A_s[l].T), _f64(held[r][i]))
            acc = term if acc is None else add(acc, term)
        dW.append(acc)
    return dA, dW


def wgrad_rank_steps(moving: Sequence[np.ndarray], local, p: int, r: int, moving_is_left: bool) -> List[np.ndarray]:
    """One-rank view of the weight-gradient loop.  ``moving[i]`` is the slice in hand at step ``i``
    (own slice first, then the deliveries); ``local`` is the rank's full ``[p*m_chunk x .]`` operand.
    ``moving_is_left``: dW += moving^T local[l]  (all-gather layer), else dW += local[l]^T moving
    (reduce-scatter layer).  Returns dW after every step."""
    L_s = split_rows(_f64(local), p)
    outs, acc = [], None
    for i in range(p):
        l = slice_index_ag(p, r, i)
        mv = _f64(moving[i])
        left, right = (mv, L_s[l]) if moving_is_left else (L_s[l], mv)
        term = gemm(np.ascontiguousarray(left.T), right)
        acc = term if acc is None else add(acc, term)
        outs.append(acc)
    return outs


# ---------------------------------------------------------------------------
# FuseReduceScatter with query-split attention (Alg. 4, Sec. 4.3)
# ---------------------------------------------------------------------------
# compute_partial_output of Alg. 2 becomes: attention of ONE query slice against the rank's full keys
# and values (the rank holds a/T heads over the whole sequence), then the row-shard output projection.
# Readings: Alg. 4 writes Softmax(Q K^T) with no scaling and no mask; a scale factor is an argument
# here (1/sqrt(D_h) in the tests, 1 gives the printed form), and no mask is applied, as printed.
# Tensors: Q, K, V [B, h, S, D_h] (h = local heads); a slice is rows [l*S/N, (l+1)*S/N) of the sequence
# of every batch element; its tokens are ordered (b, s) and its features (head, d), so that
# O~ [B*S/N x h*D_h] is the left operand of the projection W_o^r [h*D_h x D].
# The attention output is rounded to bf16 before the projection when ``round_attn`` is set (the GPU
# path hands it to the bf16 GEMM), as the up-projection output of the MLP pair is.

def softmax_rows(x: np.ndarray) -> np.ndarray:
    x = _f64(x)
    e = np.exp(x - np.max(x, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_slice(Q, K, V, l: int, N: int, scale: float) -> np.ndarray:
    """Attention output of query slice ``l`` of ``N``: ``[B*S/N x h*D_h]``, tokens (b, s), features (head, d)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, h, S, Dh = Q.shape
    c = S // N
    out = np.zeros((B, c, h, Dh))
    for b in range(B):
        for a in range(h):
            q = Q[b, a, l * c:(l + 1) * c, :]
            scores = gemm(q, np.ascontiguousarray(K[b, a].T))
            w = softmax_rows(scores * scale)
            out[b, :, a, :] = gemm(w, V[b, a])
    return out.reshape(B * c, h * Dh)


def attn_rs_definition(Q_list, K_list, V_list, Wo_list, scale: float, round_attn: bool = False):
    """Dense definition: every rank runs full attention over its heads and projects; the partial outputs
    are reduce-scattered along the sequence.  Returns the per-rank results ``[B*S/N x D]`` (tokens (b, s))."""
    N = len(Q_list)
    per_rank_slices = []
    for r in range(N):
        parts = []
        for l in range(N):
            o = attention_slice(Q_list[r], K_list[r], V_list[r], l, N, scale)
            if round_attn:
                o = round_to_bf16(o)
            parts.append(gemm(o, Wo_list[r]))
        per_rank_slices.append(parts)
    return reduce_scatter(per_rank_slices)


def fuse_attn_rs_lockstep(Q_list, K_list, V_list, Wo_list, scale: float, round_attn: bool = False):
    """Alg. 4 by all ranks in lock-step: Alg. 2 whose compute is attention of slice ``l`` then the projection."""
    N = len(Q_list)
    B_in = [None] * N
    O = [None] * N
    received = [[None] * N for _ in range(N)]
    sent = [[None] * N for _ in range(N)]
    for i in range(N):
        in_flight = [None] * N
        for r in range(N):
            l = slice_index_rs(N, r, i)
            o = attention_slice(Q_list[r], K_list[r], V_list[r], l, N, scale)
            if round_attn:
                o = round_to_bf16(o)
            O[r] = gemm(o, Wo_list[r])
            if i > 0:
                received[r][i] = B_in[r]
                O[r] = add(B_in[r], O[r])
            if i < N - 1:
                sent[r][i] = O[r].copy()
                in_flight[send_rank(N, r)] = sent[r][i]
        B_in = in_flight
    return O, received, sent


def attn_rs_rank_steps(Q, K, V, Wo, R: Sequence[Optional[np.ndarray]], p: int, r: int, scale: float,
                       round_attn: bool = True) -> List[np.ndarray]:
    """One-rank view of Alg. 4: the output of every step, ``R[i]`` being what the neighbour delivers for step i."""
    outs = []
    for i in range(p):
        o = attention_slice(Q, K, V, slice_index_rs(p, r, i), p, scale)
        if round_attn:
            o = round_to_bf16(o)
        out = gemm(o, Wo)
        if i > 0:
            out = add(_f64(R[i]), out)
        outs.append(out)
    return outs

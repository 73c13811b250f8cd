/*
 * commfuse.h -- C ABI of the CommFuse rank-step library for AMD MI355X (gfx950).
 *
 * One rank's share of the paper's decomposed, ring-ordered, fused replacement
 * of reduce-scatter after a row-parallel GEMM (FuseReduceScatter, Alg. 2 and
 * its row-parallel instantiation Alg. 3 / Sec. 4.1) and of all-gather before a
 * column-parallel GEMM (FuseAllGather, Alg. 1 / Sec. 4.2), plus the
 * data-parallel gradient reduce step (Alg. 2 with the identity as
 * compute_partial_output; Sec. 3.1, Zero-DP paragraph).
 *
 * Notation follows the paper: p = ring size (T = N, slicing granularity m = 1),
 * r = rank, i = step in [0, p), l = slice index computed at step i,
 * B_in / B_out = receive / send buffers.
 *
 * Conventions for every entry point
 *   - Plain C.  All tensor pointers are DEVICE pointers unless a comment says
 *     "host".  Descriptor structs and pointer tables are HOST memory.
 *   - Row-major tensors with explicit row strides in elements (0 = packed).
 *   - The caller owns every buffer and every stream.  Nothing here allocates
 *     device memory.  No call synchronises the device: work is enqueued on the
 *     given HIP stream(s) (hipStream_t passed as void*; NULL = default stream)
 *     and the call returns.
 *   - Errors: a negative cf_status is returned and nothing is enqueued; the
 *     text of the last error of the calling thread is kept for
 *     commfuse_last_error().  The library never aborts or throws.
 *   - Alignment: every tensor base pointer must be 16-byte aligned; k, n and
 *     all row strides must be multiples of 8 elements for bf16 operands and of
 *     4 elements for fp32 operands (CF_ERR_MISALIGNED otherwise).
 */
#ifndef COMMFUSE_H
#define COMMFUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CF_OK = 0,
    CF_ERR_INVALID_ARG = -1,  /* p, rank, step, sizes or flags out of range     */
    CF_ERR_NULL_PTR = -2,     /* a required pointer is NULL (or recv misplaced) */
    CF_ERR_UNSUPPORTED = -3,  /* dtype / layout combination not implemented     */
    CF_ERR_MISALIGNED = -4,   /* pointer or stride alignment rule violated      */
    CF_ERR_HIP = -5           /* a HIP runtime call failed (see last_error)     */
} cf_status;

typedef enum { CF_BF16 = 0, CF_F32 = 1 } cf_dtype;
typedef enum {
    CF_KIND_RS = 0,       /* FuseReduceScatter on the ring (Alg. 2 / Alg. 3)                      */
    CF_KIND_AG = 1,       /* FuseAllGather on the ring (Alg. 1)                                   */
    CF_KIND_DP = 2,       /* gradient reduce on the ring (Alg. 2, identity compute)               */
    CF_KIND_RS_PAIR = 3,  /* FuseReduceScatter, pairwise bidirectional schedule (Appendix A(a))   */
    CF_KIND_DP_PAIR = 4,  /* gradient reduce, pairwise bidirectional schedule                     */
    CF_KIND_WGRAD_X = 5,  /* weight gradient of the all-gather layer: the [m x k] operand travels  */
    CF_KIND_WGRAD_G = 6   /* weight gradient of the reduce-scatter layer: the [m x n] one travels  */
} cf_kind;

/* Memory order of the weight shard W^r.
 *   CF_W_KN: W[k x n], row-major, n contiguous -- the paper's W_o^r in R^{D/T x D}
 *            multiplied from the right (Alg. 3 parameters line).
 *   CF_W_NK: the same matrix stored transposed, [n x k] with k contiguous (the
 *            order in which linear layers commonly keep their weights). */
typedef enum { CF_W_KN = 0, CF_W_NK = 1 } cf_wlayout;

/* One tensor-parallel layer on one rank (Alg. 1 / Alg. 2 "Input", "Parameters",
 * "Output" lines).  HOST struct. */
typedef struct {
    int32_t p;         /* ring size T (= N, m = 1), >= 1                         */
    int32_t rank;      /* r in [0, p)                                            */
    int64_t m_chunk;   /* rows per sequence slice, B*S/p                         */
    int64_t n;         /* output features of this rank's weight shard            */
    int64_t k;         /* contraction length of this rank's weight shard         */
    int64_t lda;       /* row stride of the activations / slice (0 = k)          */
    int64_t ldw;       /* row stride of W (0 = n for CF_W_KN, k for CF_W_NK)      */
    int64_t ldo;       /* row stride of outputs, partial sums and B_in (0 = n)   */
    int32_t in_dtype;  /* cf_dtype of activations and W                          */
    int32_t out_dtype; /* cf_dtype of the all-gather path's output O; partial
                          sums, B_in, B_out and the reduce-scatter result are
                          always fp32                                            */
    int32_t w_layout;  /* cf_wlayout                                             */
    int32_t m;         /* slicing granularity (Sec. 3.2): the sequence is cut into m*p
                          slices, i.e. every ring hop into m sub-steps; 0 or 1 = the
                          paper's default m = 1.  m must divide m_chunk.  See below. */
} cf_layer_desc;

/* Slicing granularity m > 1.  The paper fixes m = 1 and prints no indices for m > 1;
 * reading taken: the ring and its p hops are unchanged, and the slice l handled at hop
 * i is cut into m row blocks that are computed, aggregated and sent on one after the
 * other.  `step` then counts SUB-STEPS j in [0, m*p): hop i = j / m, block s = j % m,
 * sub-slice c = l*m + s of the m*p (rows [c*m_chunk/m, (c+1)*m_chunk/m) of the
 * sequence).  Every per-step tensor (recv, out, the slice in hand, the slots of
 * cf_buffers) then has m_chunk/m rows, "step == 0" conditions become "hop == 0", and
 * a delivery for sub-step j is what the neighbour produced at sub-step j - m.
 * The pairwise kinds need m = 1. */

/* Slice index l of step i: Alg. 2 "l = (r - i - 1 + N) mod N" for CF_KIND_RS and
 * CF_KIND_DP, Alg. 1 "l = (r - i + N) mod N" for CF_KIND_AG; for the pairwise kinds
 * the partner of round i+1 while i < p-1 and the rank's own slice at i = p-1.
 * Host-only arithmetic.  Returns a negative cf_status on bad arguments. */
int commfuse_chunk_index(int kind, int p, int rank, int step);

/* The same for slicing granularity m >= 1: sub-slice index c in [0, m*p) of sub-step
 * `step` in [0, m*p) (ring kinds only). */
int commfuse_subslice_index(int kind, int p, int m, int rank, int step);

/* Pairwise bidirectional schedule (Appendix A(a)): the reduce-scatter's p(p-1) sends
 * are p-1 rounds of p/2 simultaneous two-way exchanges, each partial going straight
 * to the owner of its slice.  Partner of `rank` in round t in [1, p-1], p even:
 *   p a power of two: rank XOR t -- for four devices the appendix's table
 *     (A,B)(C,D) / (A,C)(B,D) / (A,D)(B,C);
 *   other even p: the circle method of round-robin tournaments (rank p-1 fixed,
 *     the others rotate): in round t, p-1 meets t-1 and a meets b when
 *     a + b = 2(t-1) mod (p-1).
 * Host-only arithmetic.  Negative cf_status for odd p or arguments out of range. */
int commfuse_pair_partner(int p, int rank, int round);

/* One iteration i of Alg. 2 / Alg. 3 (compute, aggregate, stage for sending):
 *     out = A[l*m_chunk : (l+1)*m_chunk, :] @ W  (+ recv  if step > 0)
 * fused in one kernel: the chunk GEMM accumulates in fp32 and its epilogue adds
 * B_in and stores B_out.
 *   A    [p*m_chunk x k]  local activations X^r, in_dtype; the call selects slice l
 *   W    weight shard, in_dtype, layout desc->w_layout
 *   recv B_in [m_chunk x n] fp32, row stride ldo; must be NULL iff step == 0
 *   out  [m_chunk x n] fp32, row stride ldo: B_out for step < p-1, the rank's
 *        result O^r for step == p-1.  May not alias recv.
 */
cf_status commfuse_rs_step(const cf_layer_desc *desc, int step, const void *A, const void *W,
                           const float *recv, float *out, void *hip_stream);

/* commfuse_rs_step for callers that cannot allocate device memory and have no workspace to register: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and the same result as commfuse_rs_step; the split-K scratch (arrival counters and fp32 partial
 * tiles) is a file-scope device array inside the library instead of the workspace registered with
 * commfuse_set_workspace, which this call ignores.  The call allocates nothing: no hipMalloc, no hipFree, no
 * allocating library routine.
 *   Limit: (m_chunk / m) * n <= 2,097,152 elements per step (8 k-splits of such a step's fp32 output fill the
 *     64 MiB of partial tiles; 64 KiB of counters beside them); larger steps get CF_ERR_INVALID_ARG and
 *     nothing is enqueued.  Every GPU the library is used on holds its own 64 MiB + 64 KiB array from the
 *     moment the library's code is loaded there until the process ends.
 *   First call on a device: looks up the device address of that GPU's array once (with that device current)
 *     and zeroes the arrival counters with a small fill kernel on `hip_stream`; make that first call outside
 *     graph capture.  The kernels leave the counters at zero, and the partial tiles are written before they
 *     are read, so nothing else needs clearing between calls.
 *   All calls on one GPU share that GPU's array: two calls whose kernels overlap in time on one GPU (different
 *     streams, or one stream of a graph with parallel branches) race.  Calls on one stream are safe. */
cf_status commfuse_rs_step_noalloc(const cf_layer_desc *desc, int step, const void *A, const void *W,
                                   const float *recv, float *out, void *hip_stream);

/* One iteration i of the pairwise schedule (Appendix A(a)), p even or 1.  The
 * partials that travel first are computed first and the rank's own slice last, as
 * in Alg. 2, so nothing is left to send after the last compute:
 *     step >= 1:    acc (+)= recv      (what the partner of round `step` sent: its
 *                                       partial of THIS rank's slice; the first
 *                                       arrival initialises acc)
 *     step <  p-1:  out = A[l] @ W     (l = partner of round step+1; sent to l)
 *     step == p-1:  out = acc + A[rank] @ W        (the reduced slice O^r)
 *   recv [m_chunk x n] fp32; NULL at step 0.  At step 1 recv may equal acc
 *        ("received in place"): then nothing is copied.  At 1 <= step < p-1, recv and
 *        acc both NULL defers the aggregation to commfuse_rs_pair_last_step.
 *   acc  [m_chunk x n] fp32 accumulator of received partials, required when p > 2
 *        (for p == 2 it is ignored: out = recv + A[rank] @ W).  The accumulate is a
 *        separate elementwise kernel enqueued before the GEMM and needs ldo == n.
 *   out  [m_chunk x n] fp32; at step p-1 it may equal acc (recv when p == 2): in place.
 */
cf_status commfuse_rs_pair_step(const cf_layer_desc *desc, int step, const void *A, const void *W,
                                const float *recv, float *acc, float *out, void *hip_stream);

/* The last iteration (step p-1) of the pairwise schedule with the aggregation deferred
 * to the end (Sec. 3.2 leaves open whether the received buffers are summed at the end
 * or incrementally inside the loop): every round's arrival was kept in a buffer of its
 * own, and
 *     out = ((recv_each[0] + recv_each[1]) + ... + recv_each[p-2]) + A[rank] @ W
 * -- the same order of fp32 additions as the incremental form, so both give the same
 * bits.  For bf16 operands the sum runs in the GEMM's epilogue (each received buffer
 * is read once and nothing is written in between); otherwise `out` serves as the
 * accumulator of elementwise passes before an in-place GEMM.
 *   recv_each HOST array of p-1 DEVICE pointers, [m_chunk x n] fp32 each, row stride
 *             ldo (ldo == n required when p > 2), in round order; unused when p == 1.
 *             None may alias out.
 * The steps before it are commfuse_rs_pair_step calls with recv = acc = NULL. */
cf_status commfuse_rs_pair_last_step(const cf_layer_desc *desc, const void *A, const void *W,
                                     const float *const *recv_each, float *out, void *hip_stream);

/* One iteration i of Alg. 1 (the compute on the slice in hand):
 *     O[l*m_chunk : (l+1)*m_chunk, :] = shard @ W
 *   shard B_out [m_chunk x k], in_dtype, row stride lda: X^r when step == 0,
 *         afterwards the slice received from rank r-1
 *   O     [p*m_chunk x n], out_dtype (fp32, or bf16 rounded to nearest even from
 *         the fp32 accumulator), row stride ldo; the concatenation of Alg. 1's
 *         last line is done in place by writing slice l at its row offset.
 */
cf_status commfuse_ag_step(const cf_layer_desc *desc, int step, const void *shard, const void *W,
                           void *O, void *hip_stream);

/* Data-parallel gradient path: iteration i of Alg. 2 with compute_partial_output
 * = "take slice l of the local gradient bucket":
 *     bucket[l*chunk_elems : (l+1)*chunk_elems] += recv      (step in [1, p))
 * step 0 computes nothing (its slice is only sent) and enqueues nothing.
 *   bucket fp32 [p*chunk_elems], updated in place;  recv fp32 [chunk_elems].
 *   (Granularity m > 1 changes nothing for an elementwise sum but the size of the
 *   pieces: call with p*m "ranks' worth" of pieces through commfuse_run_schedule, which
 *   honours desc->m for this kind too.)
 *   chunk_elems may be any non-negative number and the pointers need only be
 *   4-byte aligned; the 16-byte vector kernel runs when both the slice start
 *   and recv are 16-byte aligned (a scalar kernel handles the rest).
 */
cf_status commfuse_dp_reduce_step(int p, int rank, int step, float *bucket, int64_t chunk_elems,
                                  const float *recv, void *hip_stream);

/* Backward pass.  The paper names reduce-scatter and all-gather in the backward pass
 * of TPSP (Sec. 1) without printing an algorithm; the gradients of the two layers
 * decompose with the same two loops:
 *   all-gather layer  Y^r = AG(X) W^r:   dX^r = RS_r(G^r (W^r)^T) is commfuse_rs_step on
 *     A = G^r with the weight pointer unchanged and the OTHER w_layout (W^r stored
 *     [k x n] is (W^r)^T stored [n' x k'] with n' = k, k' = n);
 *   reduce-scatter layer Y^r = RS_r(A^q W^q):  dA^r = AG(G) (W^r)^T is commfuse_ag_step
 *     in the same way;
 *   both weight gradients are sums over the sequence slices, accumulated in the order in
 *   which Alg. 1's loop meets them -- one call of commfuse_wgrad_step per iteration:
 *       dW (+)= left^T @ right          (accumulates iff step > 0)
 *     left  [m_chunk x k] bf16, row stride lda;  right [m_chunk x n] bf16, row stride ldw
 *     dW    [k x n] fp32, row stride ldo, updated in place
 *     desc: p, rank, m_chunk (rows contracted per step), k, n as above; in_dtype must be
 *     CF_BF16 (CF_ERR_UNSUPPORTED otherwise, and for operands of 2 GiB or more);
 *     w_layout and out_dtype are ignored.  The caller passes the slice in hand and
 *     rows l = (r - step) mod p of its local operand (commfuse_chunk_index(CF_KIND_AG)).
 * In cf_buffers for CF_KIND_WGRAD_X / CF_KIND_WGRAD_G: A_or_own_shard = the rank's own
 * slice of the travelling operand, W = its full local operand [p*m_chunk x .] (the
 * other factor), O = dW, peer_stage / slot / peer_sink as for CF_KIND_AG. */
cf_status commfuse_wgrad_step(const cf_layer_desc *desc, int step, const void *left, const void *right,
                              float *dW, void *hip_stream);

/* Gradient path under the pairwise schedule: every round's arrival is a peer's copy
 * of THIS rank's slice, so for step in [1, p)
 *     bucket[rank*chunk_elems : (rank+1)*chunk_elems] += recv
 * and step 0 enqueues nothing.  p even or 1; pointer rules as above. */
cf_status commfuse_dp_pair_step(int p, int rank, int step, float *bucket, int64_t chunk_elems,
                                const float *recv, void *hip_stream);

/* Buffers of a whole emulated rank step.  HOST struct holding DEVICE pointers.
 * Peer traffic is emulated: what rank r-1 would deliver for step i (i = 1..p-1)
 * sits in peer_stage[i-1] and is copied into slot[i % 2] on the copy stream.
 * With granularity m > 1, peer_stage[i-1] / peer_sink[i] still hold one whole hop (the
 * m blocks stacked by rows); block s of hop i is delivered for sub-step j = i*m + s into
 * slot[j % 2] (m_chunk/m rows are used of each slot and send slot).
 * Slices and partial sums keep the descriptor's row strides everywhere (slices of the
 * all-gather path: lda, of the weight-gradient path: lda / ldw, partial sums: ldo), in
 * peer_stage, slot, send_slot, peer_sink and recv_each alike; a delivery copies a row
 * block with its padding.  The pairwise kinds need packed partial sums (ldo == n). */
typedef struct {
    const void *A_or_own_shard;   /* RS: A [p*m_chunk x k]; AG: X^r [m_chunk x k]; DP: unused */
    const void *W;                /* weight shard (unused for DP)                             */
    void *O;                      /* RS: O^r [m_chunk x n] fp32; AG: O [p*m_chunk x n]; DP: bucket */
    const void *const *peer_stage;/* host array of p-1 device pointers (may be NULL if p == 1) */
    void *slot[2];                /* B_in double buffer: RS fp32 [m_chunk x n]; AG in_dtype
                                     [m_chunk x k]; DP fp32 [chunk_elems]                      */
    float *send_slot[2];          /* RS: B_out double buffer fp32 [m_chunk x n]; else unused   */
    void *const *peer_sink;       /* optional host array of p-1 device pointers receiving the
                                     emulated sends of steps 0..p-2 (RS: B_out, AG: the slice
                                     in hand, DP: slice l); NULL = sends are not copied        */
    void *const *recv_each;       /* optional (NULL = use slot[]): host array of p-1 device
                                     buffers shaped like slot[], one per hop / round; slot[] is
                                     then unused.  Ring kinds (RS, AG, weight gradient): hop i's
                                     delivery lands in recv_each[i-1]; no buffer is reused inside
                                     the call, so no delivery waits for a kernel, and with
                                     CF_DEVICE_WAIT and no peer_sink the compute stream carries
                                     nothing but the step kernels.  CF_KIND_RS_PAIR: round t's
                                     delivery lands in recv_each[t-1], no step accumulates, and
                                     the last step adds them all in its epilogue
                                     (commfuse_rs_pair_last_step).  Bucket kinds (CF_KIND_DP,
                                     CF_KIND_DP_PAIR): with CF_PERSISTENT only.                  */
    float *const *send_each;      /* reduce-scatter kinds, optional (NULL = use send_slot[]): host
                                     array of p-1 device buffers [m_chunk x n] fp32, row stride ldo,
                                     one per sending step: the B_out of step i < p-1 (Alg. 2
                                     "B_out <- O"; with m > 1 the m blocks of hop i stacked by rows)
                                     is stored to send_each[i] and stays there, send_slot[] is then
                                     unused, and peer_sink[i], if given, is copied from it.  No
                                     send buffer is reused inside the call, so no step waits for an
                                     earlier send to drain.  Required with CF_PERSISTENT when
                                     p > 1: the steps of that launch run side by side and each
                                     needs a B_out of its own.  None may alias O or a landing
                                     buffer.                                                      */
} cf_buffers;

enum {
    CF_NO_COPY = 1u,     /* enqueue the kernels only (slots keep whatever they hold)   */
    CF_NO_COMPUTE = 2u,  /* enqueue the copies only                                    */
    CF_SERIAL = 4u,      /* one stream, copy i+1 strictly after kernel i: no overlap   */
    CF_POISON = 8u,      /* debug: fill each B_in slot with NaN bytes before its copy  */
    CF_GRAPH = 16u,      /* capture the schedule once into a HIP graph, replay after   */
    CF_FUSED_COPY = 32u, /* bf16 RS / AG only (bucket kinds: with CF_PERSISTENT only, see
                            there): the delivery for step i+1 is carried by
                            extra workgroups of step i's kernel launch instead of a
                            hipMemcpyAsync on copy_stream: one stream, no events
                            (copy_stream is unused; not with CF_POISON)               */
    CF_PERSISTENT = 128u,/* bf16 CF_KIND_RS / CF_KIND_AG / CF_KIND_RS_PAIR / CF_KIND_WGRAD_* (and the fp32 bucket kinds, see
                            the end), at most 16 (sub-)steps: ONE kernel
                            launch runs all steps of the rank step.  Its work items (step, output tile) are
                            dealt out step-major to a grid that fills the chip once; tiles of different
                            steps run side by side (the chunk GEMMs do not depend on each other -- only
                            the add of B_in / the arrival of the slice does), nothing is launched or
                            drained between steps, and because a step no longer has to fill the chip
                            alone the tiles can be larger.  Needs cf_buffers.recv_each (every hop's
                            delivery stays where it landed), for the reduce-scatter kinds
                            cf_buffers.send_each (every step stores the B_out of Alg. 2 into a
                            buffer of its own; peer_sink, if given, is copied from those after the
                            launch).  With CF_SERIAL the
                            deliveries are enqueued before the kernel on the compute stream -- a
                            kernel that holds its compute units for the whole rank step starves
                            concurrent blit copies.  Without CF_SERIAL (CF_KIND_RS / CF_KIND_AG only, two
                            streams; the other kinds need CF_SERIAL): the rank step is a few launches, each a
                            group of consecutive (sub-)steps that fills the chip about once, and the
                            deliveries of a group are copied on copy_stream under the launches of the
                            groups before it, one event per group ordering the two streams.
                            (The kernel can also wait for per-step delivery flags on the device; on a real ring, where a delivery is a remote DMA
                            write that needs no compute unit here, that is how it would overlap.)
                            CF_KIND_RS_PAIR: every arrival is kept (recv_each) and the last step adds
                            them all, as commfuse_rs_pair_last_step does.
                            Weight-gradient kinds: recv_each must be in GATHERED order -- with
                            blk = m_chunk rows of the moving operand, the own slice is row block `rank`
                            of one buffer and recv_each[i-1] its row block (rank - i) mod p (the block
                            the local operand pairs hop i with); else CF_ERR_UNSUPPORTED.  The p chunk
                            GEMMs dW += slice^T local_slice are then one GEMM whose contraction runs
                            over all p*m_chunk rows: dW is written once, not read and written p times
                            (the sum runs in row-block order, not in step order).
                            Results are deterministic for a given launch, but not bit-identical to the
                            one-kernel-per-step modes: with eight or sixteen (sub-)steps the workgroups of
                            each XCD start their k loops at a different k-tile and wrap around, so the fp32
                            sum over k is taken in a rotated order.
                            Bucket kinds (CF_KIND_DP, CF_KIND_DP_PAIR; fp32): there is no GEMM to fuse
                            into; the flag buys the deliveries of all hops as ONE batched copy launch
                            into recv_each, followed by the same add kernels in the same order.  With
                            CF_FUSED_COPY no copy is launched: the add kernels read the arrivals from
                            the neighbours' buffers (peer_stage) and store them on to recv_each in the
                            same pass (same sums, bit for bit).
                            With CF_FUSED_COPY (CF_KIND_RS, CF_KIND_AG): the delivery is carried by the
                            consumer -- no copy is launched, the emulated transfer runs inside the kernel,
                            under its main loop.  Reduce-scatter: the waves that need B_in read it from the
                            neighbour's buffer (peer_stage), add it in mid-sum, and store it to the landing
                            buffer (recv_each).  All-gather: the kernel takes the gathered slices from the
                            neighbours' buffers as its left operand, and every k-tile that comes in is
                            stored on to the landing buffer by one of the workgroups that load it.  (A row
                            block lands without the padding of its rows.)  A reduce-scatter launch that
                            cannot do that (a tile other than 256x256, a k range under 18 k-tiles of 64, or
                            20 with a ragged last one; the projection of the attention layer) reads B_in
                            from the neighbour's buffer in its epilogue, and the same work item copies its
                            tile's part of it to the landing buffer beside its GEMM (packed partial sums,
                            ldo == n).  Otherwise (all-gather: k not a multiple of 64; the other kinds) the
                            flag changes nothing: the deliveries are enqueued in front.
                            With CF_FUSED_COPY (CF_KIND_RS_PAIR) and a registered workspace: the work items
                            of step t-1 land the arrival of round t (peer_stage[t-1] -> recv_each[t-1]), each
                            its own output tile's part, and count the tile up; the step that sums the
                            arrivals waits per tile (bounded spin: commfuse_device_status reports a
                            time-out).  Same sums, bit for bit.  Without a workspace the flag changes nothing.
                            Not with CF_DEVICE_WAIT.                                                  */
    CF_DEVICE_WAIT = 64u /* bf16 RS / AG only, needs a registered workspace: the compute
                            stream does not wait for the copy stream between steps;
                            each delivery is followed by a flag write and the step
                            kernel waits for its flag on the device (before its first
                            operand load for AG, before the B_in add for RS, as in
                            Alg. 2 where the transfer is needed by the add only).  The
                            wait is a bounded spin: on time-out the kernel finishes
                            with invalid results and commfuse_device_status() reports it.
                            The two streams must be able to progress independently, and
                            the mode cannot be combined with CF_GRAPH: a graph holds no
                            edge from a flag write to the kernel polling that flag, so a
                            replay may queue the writer behind the waiting kernel          */
};

/* A whole rank step: the p iterations of Alg. 1 (CF_KIND_AG) or Alg. 2
 * (CF_KIND_RS, CF_KIND_DP) with the paper's overlap: while the kernel of step i
 * runs on compute_stream, the delivery for step i+1 is copied on copy_stream;
 * p kernels, p-1 deliveries, nothing after the last kernel.  Ordering between
 * the two streams uses HIP events owned by the library.  On return
 * compute_stream has been made to wait for everything enqueued, so one
 * hipStreamSynchronize(compute_stream) by the caller suffices.
 * For CF_KIND_DP, desc->m_chunk is the number of elements per slice and n, k,
 * dtypes are ignored.  Overlapping calls that share slots race.
 * Pairwise kinds (CF_KIND_RS_PAIR, CF_KIND_DP_PAIR; p even or 1): peer_stage[t-1] is
 * what the partner of round t delivers (its partial / copy of this rank's slice);
 * CF_KIND_RS_PAIR accumulates in O itself (the delivery of round 1 lands in O, later
 * ones in slot[t % 2] and are added to O before the step's GEMM; the last GEMM adds
 * its product to O in place), or, with recv_each set, keeps every arrival and sums
 * them in the last GEMM's epilogue; peer_sink[i] receives what step i sends to the
 * partner of round i+1.  CF_DEVICE_WAIT is not available for them, CF_FUSED_COPY with
 * CF_PERSISTENT only. */
cf_status commfuse_run_schedule(const cf_layer_desc *desc, int kind, const cf_buffers *bufs,
                                void *compute_stream, void *copy_stream, uint32_t flags);

/* Query-split attention (Alg. 4, Sec. 4.3): FuseReduceScatter whose compute_partial_output
 * is the attention of ONE query slice against the rank's full keys and values, followed by
 * the row-shard output projection W_o^r; aggregation and staging for sending as in Alg. 2.
 * The rank holds `heads` = a/T attention heads over the whole sequence.
 *   Q, K, V   [batch, heads, seq, head_dim] bf16, contiguous (Alg. 4 "Input" line)
 *   slice l   = queries [l*seq/p, (l+1)*seq/p) of every batch element; its seq/p * batch
 *               tokens are ordered (batch element, position), its features (head, d)
 *   attn_out  [batch*seq/p x heads*head_dim] bf16, caller-owned scratch: the attention
 *               output of the slice, rounded to bf16, the left operand of the projection
 *   Wo        [heads*head_dim x n] (CF_W_KN) or its transpose (CF_W_NK), bf16
 *   recv/out  [batch*seq/p x n] fp32, as for commfuse_rs_step
 * Readings: Alg. 4 prints Softmax(Q K^T) with neither scale nor mask: `scale` multiplies
 * the scores (1/sqrt(head_dim) is the usual choice, 1 the printed form) and no mask is
 * applied.  The softmax runs in fp32; the probabilities are rounded to bf16 for the
 * product with V (the row sum is taken over the rounded values).  head_dim must be 128
 * and p must divide seq (CF_ERR_UNSUPPORTED / CF_ERR_INVALID_ARG otherwise). */
typedef struct {
    int32_t p, rank;
    int32_t batch, heads, seq, head_dim;
    int64_t n;          /* output features D of W_o^r                                  */
    int64_t ldw;        /* row stride of Wo (0 = packed)                               */
    int64_t ldo;        /* row stride of partial sums and outputs (0 = n)              */
    int32_t w_layout;   /* cf_wlayout of Wo                                            */
    float scale;        /* factor on Q K^T before the softmax                          */
} cf_attn_desc;

/* The attention of query slice `slice` alone (the first half of a step). */
cf_status commfuse_attn_slice(const cf_attn_desc *desc, int slice, const void *Q, const void *K, const void *V,
                              void *attn_out, void *hip_stream);

/* One iteration i of Alg. 4: attention of slice l = (r - i - 1) mod p into attn_out, then
 *     out = attn_out @ Wo (+ recv if step > 0)       (two kernels on `hip_stream`) */
cf_status commfuse_attn_rs_step(const cf_attn_desc *desc, int step, const void *Q, const void *K, const void *V,
                                const void *Wo, const float *recv, float *out, void *attn_out, void *hip_stream);

/* Buffers of a whole emulated rank step of Alg. 4 (HOST struct, DEVICE pointers); the
 * delivery / sending fields mean what they mean in cf_buffers for CF_KIND_RS. */
typedef struct {
    const void *Q, *K, *V, *Wo;
    void *attn_out;                 /* one slice's attention output [batch*seq/p x heads*head_dim] bf16; with
                                       CF_PERSISTENT p times that: the outputs of all p slices, slice l in row
                                       block l                                                               */
    float *O;                       /* O^r [batch*seq/p x n] fp32 */
    const void *const *peer_stage;
    void *slot[2];
    float *send_slot[2];
    void *const *peer_sink;
    void *const *recv_each;
    float *const *send_each;
} cf_attn_buffers;

/* A whole rank step of Alg. 4 with the overlap and the flags of commfuse_run_schedule.
 * CF_PERSISTENT (with CF_SERIAL and recv_each, m = 1): the deliveries, then the attention of ALL p query slices
 * in one launch (a slice's attention depends on nothing that travels; the grid then fills the chip without a
 * key split), then the projections with their B_in adds as one persistent launch over attn_out. */
cf_status commfuse_run_attn_schedule(const cf_attn_desc *desc, const cf_attn_buffers *bufs, void *compute_stream,
                                     void *copy_stream, uint32_t flags);

/* Synchronises `hip_stream` and reports whether any step kernel since the last call gave up a
 * bounded device-side wait -- CF_DEVICE_WAIT, or CF_KIND_RS_PAIR with CF_PERSISTENT | CF_FUSED_COPY -- (CF_ERR_HIP;
 * the status word in the workspace is cleared).  CF_OK if none did
 * or no workspace is registered.  This is the one entry point that synchronises. */
cf_status commfuse_device_status(void *hip_stream);

/* Text of the calling thread's last error ("" if none).  Host pointer, valid
 * until the thread's next failing call. */
const char *commfuse_last_error(void);

/* Split-K workspace.  The per-step grids of the chunk GEMMs (one sequence slice of
 * Alg. 1 / Alg. 2 at a time) are small against 256 compute units; with a workspace
 * the bf16 kernels may split the k range of an output tile over several
 * workgroups, which park fp32 partial tiles there and are summed in a fixed order
 * by the last one to finish.  Optional: without one every tile is computed by a
 * single workgroup.
 *   commfuse_workspace_bytes: size that lets every split choice be used for this
 *     layer (0 if the kind / dtype never splits).  Host-only arithmetic.
 *   commfuse_set_workspace: registers a caller-owned DEVICE buffer (16-byte
 *     aligned), or clears a registration (NULL / 0).  With hip_stream == NULL the
 *     buffer serves all later calls of this process; with a stream it serves the
 *     work enqueued on THAT stream (for commfuse_run_schedule: the compute stream)
 *     and takes precedence there -- two layers in flight on two streams each
 *     register a workspace of their own.  The first 64 KiB (arrival counters,
 *     delivery flags, a status word) are zeroed on `hip_stream` (this is the one
 *     call that enqueues a memset; do not capture it into a graph).  The caller
 *     keeps the buffer alive and unmodified while registered.  Steps that
 *     overlap in time on the GPU must not share a workspace.
 *     commfuse_device_status(stream) reads the status word of the workspace that
 *     serves `stream`.  Clear a stream's registration before destroying the stream
 *     (a later stream may get the same handle).
 */
size_t commfuse_workspace_bytes(const cf_layer_desc *desc, int kind);
cf_status commfuse_set_workspace(void *device_ptr, size_t bytes, void *hip_stream);

/* Destroys the events and graphs the library created lazily.  Call with no
 * work of this library in flight. */
void commfuse_destroy_cache(void);

/* Library version, e.g. 100 = 1.0.0. */
int commfuse_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COMMFUSE_H */

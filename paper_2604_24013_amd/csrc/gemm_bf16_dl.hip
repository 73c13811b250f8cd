// bf16 x bf16 -> fp32 chunk GEMM for gfx950, direct-to-LDS variant.
//
//  * Operand tiles go from global memory straight into LDS (buffer_load ... lds,
//    16 bytes per lane) without passing through registers.
//  * A [k x n] weight tile stays in its natural order in LDS and is read back
//    with the transposing LDS read (ds_read_b64_tr_b16); a [n x k] weight tile
//    and the activations are read with plain 16-byte reads.
//  * k-tiles of 64 (full 128-byte lines of the k-contiguous operands) in NS = 2..4
//    LDS stages (as many as the tile shape leaves room for in 160 KiB).  A k-tile is consumed in four 16-wide slices; fragments are
//    double-buffered in registers and the LDS reads of slice s+1 are issued under
//    the first MFMAs of slice s.  The one barrier per k-tile sits before the last
//    slice: by then every wave has read all of the tile, so the freed stage's
//    next tile can be requested, and the next tile (requested NS-1 barriers
//    earlier) is published; its first fragments are fetched under the MFMAs of
//    the last slice, so the matrix pipe does not drain at tile boundaries.
//  * The direct loads of a tile are not issued as one burst: each wave issues one
//    after every few MFMAs.  A burst fills the address queue of the texture unit
//    and the wave -- which issues in order -- then cannot feed the matrix pipe
//    until its last load has been accepted.
//  * Same fused epilogue as the register-staged kernel: Alg. 2 "O <- B_in + O",
//    "B_out <- O", or Alg. 1's in-place slice store -- here with bounds-checked
//    buffer loads/stores, so all B_in loads of a row block are in flight at once.
//
// Layout in LDS (per stage):
//   activations / [n x k] weights: 128-byte rows (64 k) of eight 16-byte chunks,
//     two rows per 256-byte line; chunk index and line half are XOR-ed with row
//     bits 1..3 so that the 16-byte fragment reads of 16 consecutive rows hit 16
//     different bank groups.  A wave-wide direct load fills 1 KiB of contiguous
//     LDS (8 rows); the swizzle is applied by choosing which global chunk each
//     lane fetches.
//   [k x n] weights: one k-row of BN bf16 after the other; the 64-byte groups of
//     a row are XOR-ed with (k & 3) so that the four rows a transposing read
//     touches fall into different banks.
// Rows / columns beyond the matrix and the k tail read as zero through the
// buffer bounds check (such a lane is given an offset beyond num_records).
#include "cf_internal.h"

#include <cstdio>
#include <cstdlib>
#include <type_traits>

namespace cf {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

constexpr int BK = 64;                    // k extent of one LDS stage
constexpr int KS = BK / 16;               // 16-wide k-slices (one MFMA deep) per stage
constexpr unsigned OOB = 0x80000000u;     // byte offset beyond any buffer this kernel accepts

// Byte offset of 16-byte chunk kc (0..7) of tile row `row` (128-byte rows).  Only row bits
// 0..3 enter the swizzle, so rows 32 apart differ by a constant 4096 bytes, and the chunk
// pair of k-slice ks is reached by XOR-ing (ks << 5) into the offset of slice 0.
__device__ __forceinline__ int swz_row(int row, int kc)
{
    const int r0 = row & 1, r1 = (row >> 1) & 1, r2 = (row >> 2) & 1, r3 = (row >> 3) & 1;
    const int half = r0 ^ r3;
    const int kcp = kc ^ ((r1 << 2) | (r2 << 1) | r3);
    return ((row >> 1) << 8) + (half << 7) + (kcp << 4);
}

// Inverse: which (row, kc) lives at bytes [pos, pos+16) of a tile.
__device__ __forceinline__ void unswz_row(int pos, int &row, int &kc)
{
    const int rp = pos >> 8, half = (pos >> 7) & 1, kcp = (pos >> 4) & 7;
    const int r1 = rp & 1, r2 = (rp >> 1) & 1, r3 = (rp >> 2) & 1;
    row = (rp << 1) | (half ^ r3);
    kc = kcp ^ ((r1 << 2) | (r2 << 1) | r3);
}

// Raw buffer descriptor: base, stride 0, num_records bytes, 32-bit raw data format.
__device__ __forceinline__ i32x4_t make_rsrc(const void *base, unsigned bytes)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    i32x4_t r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(a & 0xFFFFFFFFull));
    r[1] = __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xFFFFull));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// One wave-wide 16-byte-per-lane load from global memory straight into LDS:
// lane L's 16 bytes land at LDS byte address lds_addr + 16 L.  Issued as inline
// assembly so that the compiler does not order later LDS reads of OTHER stages
// behind it; completion is awaited explicitly (vmcnt) before the barrier that
// publishes the stage.
__device__ __forceinline__ void direct_load_16(i32x4_t rsrc, unsigned voffset, int soffset, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "buffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory");   // M0 is written here and used by nothing else in this kernel
}

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// One 16-byte-per-lane load from global memory into registers whose completion the CALLER awaits (vmcnt): issued
// as inline assembly so that the compiler, which cannot count the requests between a load in one trip of a loop
// and its use in the next, does not drain the whole request queue in front of the use.
__device__ __forceinline__ u32x4_t load_16_unawaited(i32x4_t rsrc, unsigned voffset, int soffset)
{
    u32x4_t v;
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(v) : "v"(voffset), "s"(rsrc), "s"(soffset) : "memory");
    return v;
}

// Scheduling hint for one slice phase: after each MFMA up to RPM LDS reads, until REMAIN reads are placed.
template <int REMAIN, int RPM>
__device__ __forceinline__ void interleave_mfma_reads()
{
    if constexpr (REMAIN > 0) {
        constexpr int now = REMAIN < RPM ? REMAIN : RPM;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, now, 0);   // `now` LDS reads
        interleave_mfma_reads<REMAIN - now, RPM>();
    }
}

__device__ __forceinline__ int xcd_remap(int pid, int total)
{
    constexpr int NXCD = 8;
    const int q = total / NXCD, rem = total % NXCD;
    const int xcd = pid % NXCD, idx = pid / NXCD;
    return xcd * q + (xcd < rem ? xcd : rem) + idx;
}

// A_T: the left operand is stored [K x M] (see GemmParams::a_t); its tile then lives in LDS like a
// [k x n] weight tile and is read with the transposing LDS read as well.
// PERSIST: one launch runs all steps of a rank step (GemmParams::n_steps, see the work-item loop below).
// RLDS: reduce-scatter variant of the SPREAD tile.  The received partial B_in does not wait for the epilogue: in
// sixteen k-tiles near the end of the k loop (the last before the final one; with a ragged K the two iterations that
// request the ragged k-tile come in between) it is brought in, one 32x32 sub-tile of every wave at a time,
// by direct loads into an LDS landing area (no register is held while the load is in flight) and added to the
// accumulators in mid-loop, so that the epilogue only stores.  The landing area takes the place of the third
// left-operand stage (see the schedule below).
// MF16: the 256x256 tile's main loop on v_mfma_f32_16x16x32_bf16 instead of v_mfma_f32_32x32x16_bf16 -- the same
// flops from twice as many instructions that each write a quarter of the accumulator registers, which costs the chip
// less power per flop (measured) and, where the launch is paced by the power limit, time.  A 32x32 sub-tile of the
// accumulators is then four 16x16 tiles: registers 4g .. 4g+3 with g = 2x + y hold rows 16x + (lane & 15), columns
// 16y + 4 (lane >> 4) .. + 3.  A k-tile is two 32-wide slices, each consumed in four quarter phases (one 32-row block
// of the wave tile per phase).
template <int BM, int BN, int WGM, int WGN, int NS, bool SPREAD, bool W_KN, bool OUT_BF16, bool A_T = false,
          bool PERSIST = false, bool RLDS = false, bool MF16 = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_dl_kernel(GemmParams P, int tiles_m, int tiles_n)
{
    static_assert(!MF16 || (SPREAD && !A_T && NS == 2 && !RLDS),
                  "16x16x32 main loop: 256x256 tile, left operand stored [m x k], B_in added in the epilogue");
    static_assert(!A_T || (W_KN && !OUT_BF16), "the transposed left operand comes with [k x n] weights and fp32 output");
    static_assert(!RLDS || (SPREAD && !OUT_BF16 && !A_T && NS == 2), "B_in through LDS: 256x256 tile, fp32 output");
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = (A_BYTES / 1024) / NW;     // 1 KiB wave-loads of the A tile per wave
    constexpr int B_LD = (B_BYTES / 1024) / NW;
    constexpr int LPT = A_LD + B_LD;                // direct loads per wave per k-tile
    static_assert(A_LD >= 1 && B_LD >= 1 && (A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "tile vs waves");
    // LDS: NSA stages of the left-operand tile, then NS stages of the weight tile.  The 256x256 tile (SPREAD)
    // fills the 160 KiB with THREE left-operand stages and two weight stages: its weight loads go out first
    // after the barrier that frees their stage and its left-operand loads one k-tile further ahead (see the
    // steady state below), which lengthens the time every load has to arrive.
    constexpr int NSA = SPREAD ? NS + 1 : NS;
    constexpr int W_BASE = NSA * A_BYTES;
    constexpr int R_BYTES = 0;
    // wave-private scratch of the epilogue's stores (4 KiB per wave): a left-operand stage that no load targets any
    // more -- RLDS: the stage that served as the landing area of B_in (land_stage below); else the third stage of the
    // 256x256 tile, else the first (after a barrier: every wave is done reading the stages)
    constexpr int E_SCR_BYTES = 4096;
    static_assert(NW * E_SCR_BYTES <= A_BYTES || !SPREAD, "epilogue scratch inside one left-operand stage");
    static_assert(NW * E_SCR_BYTES <= NSA * A_BYTES + NS * B_BYTES, "epilogue scratch inside the stages");
    static_assert(NS >= 2 && NS <= 4 && NSA * A_BYTES + NS * B_BYTES + R_BYTES <= 160 * 1024, "LDS budget");
    static_assert(KS == 4, "the slice schedule below is written for four slices per stage");
    constexpr int W_ROWB = BN * 2;                   // bytes of one k-row of a [k x n] weight tile
    constexpr int A_ROWB = BM * 2;                   // bytes of one k-row of a [k x m] left-operand tile

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NSA * A_BYTES + NS * B_BYTES + R_BYTES];

    const int tid0 = threadIdx.x;

    // Workgroups beyond the GEMM's own grid carry the emulated delivery of the NEXT step (what the ring
    // neighbour sends while this step computes): a streaming copy that shares the launch with the GEMM,
    // so that no second stream, event or inter-queue wait sits between two step kernels.
    const int gemm_wgs = tiles_m * tiles_n * P.splits;
    if (!PERSIST && (int)blockIdx.x >= gemm_wgs) {
        const u32x4_t *src = static_cast<const u32x4_t *>(P.cp_src);
        u32x4_t *dst = static_cast<u32x4_t *>(P.cp_dst);
        const size_t n16 = P.cp_bytes / 16;
        const size_t stride = (size_t)P.cp_wgs * (64 * NW);
        size_t i = (size_t)((int)blockIdx.x - gemm_wgs) * (64 * NW) + tid0;
        for (; i + 3 * stride < n16; i += 4 * stride) {
            const u32x4_t v0 = __builtin_nontemporal_load(&src[i]);
            const u32x4_t v1 = __builtin_nontemporal_load(&src[i + stride]);
            const u32x4_t v2 = __builtin_nontemporal_load(&src[i + 2 * stride]);
            const u32x4_t v3 = __builtin_nontemporal_load(&src[i + 3 * stride]);
            __builtin_nontemporal_store(v0, &dst[i]);
            __builtin_nontemporal_store(v1, &dst[i + stride]);
            __builtin_nontemporal_store(v2, &dst[i + 2 * stride]);
            __builtin_nontemporal_store(v3, &dst[i + 3 * stride]);
        }
        for (; i < n16; i += stride)
            __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
        return;
    }

    // Persistent mode (GemmParams::n_steps > 0): one launch runs ALL steps of a rank step.  The work items
    // (step, output tile) are dealt out round robin, step-major, to the workgroups of a grid that fills the
    // chip once; a workgroup goes on to its next item as soon as it is done with the last one, so tiles of
    // different steps run side by side (the chunk GEMMs of Alg. 1 / Alg. 2 do not depend on each other; only
    // the add of B_in / the arrival of the slice does, which the per-step delivery flag guards) and nothing
    // is launched, drained or refilled between steps.  Every workgroup's loop is finite: the kernel exits.
    const int tiles_per_step = tiles_m * tiles_n * P.splits;
    // XCD-per-step mapping (GemmParams::xcd_steps): XCD x (workgroups x, x+8, ...) runs the steps x, x+8, ...
    // whole, so a step's own operand (A of the step) passes through one L2 only, instead of through all
    // eight when every XCD holds a band of every step's tiles.  With GemmParams::xcd_bands = NB > 1 the XCDs form
    // 8 / NB step groups x NB column bands instead: XCD x runs the steps x / NB, x / NB + 8 / NB, ... on the tile
    // columns of band x % NB only -- fewer weight bands and more left-operand bands per L2, which is less traffic
    // where a step has few tile rows and many tile columns.
    const bool by_xcd = PERSIST && P.xcd_steps;
    const int xcd_nb = by_xcd ? P.xcd_bands : 1, xcd_groups = 8 / xcd_nb;
    const int xcd_grp = (int)(blockIdx.x & 7) / xcd_nb, xcd_band = (int)(blockIdx.x & 7) % xcd_nb;
    const int item_stride = by_xcd ? (int)(gridDim.x >> 3) : (int)gridDim.x;
    const int n_items = PERSIST ? (by_xcd ? (tiles_per_step * P.n_steps) >> 3 : tiles_per_step * P.n_steps) : 0;
    int item = by_xcd ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    do {
    // Lane and wave indices are taken anew for every work item: what is derived from them then lives
    // from its first use in this item, not across the whole loop.
    int tid = tid0;
    if constexpr (PERSIST)
        asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    // the XCD's items: all (step, tile row) pairs of one tile column, then the next column of its band
    const int rows_x = by_xcd ? (P.n_steps / xcd_groups) * tiles_m : 1;       // (step, tile row) pairs of this XCD
    const int step_i = PERSIST ? (by_xcd ? xcd_grp + xcd_groups * ((item % rows_x) / tiles_m) : item / tiles_per_step) : 0;
    const void *const cA = PERSIST ? P.A_step[step_i] : P.A;
    const float *const cRecv = PERSIST ? P.recv_step[step_i] : P.recv;
    void *const cLand = PERSIST ? P.land_step[step_i] : nullptr;   // where the delivery is to land, if this kernel carries it
    void *const cOut = PERSIST ? P.out_step[step_i] : P.out;
    const unsigned *const cFlag = PERSIST ? P.flag_step[step_i] : P.wait_flag;
    // further received partials (GemmParams::recv_more): in a persistent launch they belong to the last step only
    const int n_more = (!PERSIST || step_i == P.n_steps - 1) ? P.n_recv_more : 0;

    // Work item = (output tile, k-split); the splits of a tile are neighbours in the remapped order.
    const int splits = P.splits;
    const int work = by_xcd ? (xcd_band * (tiles_n / xcd_nb) + item / rows_x) * tiles_m + (item % rows_x) % tiles_m
                            : xcd_remap(PERSIST ? item % tiles_per_step : (int)blockIdx.x, tiles_per_step);
    const int tile = work / splits, split = work % splits;
    const int m0 = (tile % tiles_m) * BM;
    const int n0 = (tile / tiles_m) * BN;
    const int M = P.M, N = P.N, K = P.K;
    const int nk_all = (K + BK - 1) / BK;
    const int ktb = (int)(((long long)nk_all * split) / splits);          // first k-tile of this split
    const int nk = (int)(((long long)nk_all * (split + 1)) / splits) - ktb; // its number of k-tiles

    // Device-side wait for an emulated delivery: one lane polls the flag with device-coherent loads,
    // sleeping between polls, for at most spin_limit polls (every wave reaches the barrier either way).
    // The delivery was written by another kernel while this one was already running, possibly through
    // the L2 of another XCD: the caches this kernel reads through may hold older contents of those
    // addresses.  So what follows the wait is either an agent-scope acquire (operand loads: L1 and the
    // non-local L2 lines are invalidated once per workgroup) or loads with the device-coherent cache
    // policy (the B_in loads of the epilogue, which are read once anyway).
    auto wait_delivery = [&](bool acquire) __attribute__((always_inline)) {
        if (cFlag != nullptr) {
            if (tid == 0) {
                unsigned n = 0;
                while (__hip_atomic_load(cFlag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == 0u) {
                    if (++n >= P.spin_limit) {
                        __hip_atomic_fetch_or(P.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(32);
                }
            }
            __syncthreads();
            if (acquire)
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
    };
    if (P.wait_at_start)
        wait_delivery(true);

    // Buffer resources; all byte extents are below 2^31 (host-checked).
    const unsigned a_bytes = (unsigned)((A_T ? ((int64_t)(K - 1) * P.lda + M) : ((int64_t)(M - 1) * P.lda + K)) * 2);
    const unsigned w_bytes = (unsigned)((W_KN ? ((int64_t)(K - 1) * P.ldw + N) : ((int64_t)(N - 1) * P.ldw + K)) * 2);
    const i32x4_t a_rsrc = make_rsrc(cA, a_bytes);
    const i32x4_t w_rsrc = make_rsrc(P.W, w_bytes);
    const unsigned lds_base = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem);

    // Per-lane global byte offsets (k0 = 0) of every wave-load, and the k index of its chunk for the tail test.
    unsigned a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int j = 0; j < A_LD; ++j) {
        const int pos = (j * NW + wave) * 1024 + lane * 16;
        if constexpr (A_T) {
            const int k = pos / A_ROWB, inrow = pos % A_ROWB;
            const int q = (inrow >> 6) ^ (k & 3);
            const int gm = m0 + q * 32 + ((inrow >> 4) & 3) * 8;
            a_off[j] = gm < M ? (unsigned)(((int64_t)k * P.lda + gm) * 2) : OOB;
        } else {
            int row, kc;
            unswz_row(pos, row, kc);
            const int gm = m0 + row;
            a_off[j] = gm < M ? (unsigned)(((int64_t)gm * P.lda + kc * 8) * 2) : OOB;
        }
    }
#pragma unroll
    for (int j = 0; j < B_LD; ++j) {
        const int pos = (j * NW + wave) * 1024 + lane * 16;
        if constexpr (W_KN) {
            const int k = pos / W_ROWB, inrow = pos % W_ROWB;
            const int q = (inrow >> 6) ^ (k & 3);
            // (MF16: the two 32-byte halves of a 64-byte group change places in the rows with odd k / 16: the sixteen-lane
            // blocks of a transposing read then hold different 8-row groups of k for the SAME columns, and the two
            // blocks that are served together -- lanes 0..15 and 16..31: k / 8 = 0 and 2, or 1 and 3, see the
            // fragment addressing -- must not fall into the same banks)
            const int c4 = ((inrow >> 4) & 3) ^ (MF16 ? ((k >> 4) & 1) << 1 : 0);
            const int gn = n0 + q * 32 + c4 * 8;
            b_off[j] = gn < N ? (unsigned)(((int64_t)k * P.ldw + gn) * 2) : OOB;
        } else {
            int row, kc;
            unswz_row(pos, row, kc);
            const int gn = n0 + row;
            b_off[j] = gn < N ? (unsigned)(((int64_t)gn * P.ldw + kc * 8) * 2) : OOB;
        }
    }
    // k index (inside a k-tile) of the chunk wave-load j of a tile fetches for this lane: needed only where a
    // k-tile is ragged or beyond the range, so it is recomputed there (from an opaque copy of the lane index:
    // kept in registers across the main loop it costs eight of them)
    auto chunk_k = [&](int j, bool k_major, int rowb) __attribute__((always_inline)) {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int pos = (j * NW + wave) * 1024 + ln * 16;
        if (k_major)
            return pos / rowb;
        int row, kc;
        unswz_row(pos, row, kc);
        return kc * 8;
    };
    const int w_kstep = W_KN ? (int)(P.ldw * 2) : 2;   // bytes per unit of k along W
    const int a_kstep = A_T ? (int)(P.lda * 2) : 2;    // ... and along the left operand
    // MF16 (whole tiles only: no lane is out of range): wave-load j of a tile fetches, lane by lane, what wave-load 0
    // fetches 64 rows further on (a [k x n] weight tile: what wave-load j - 2 fetches 32 k-rows further on -- the
    // 32-byte halves change places every 16 k-rows), so one per-lane offset per operand (two for [k x n] weights) is
    // kept and the distance goes into the scalar part of the address
    constexpr int W_JP = (MF16 && W_KN) ? 2 : 1;     // wave-loads of a weight tile with an offset register of their own
    const int a_jstep = MF16 ? (int)(64 * P.lda * 2) : 0;
    const int w_jstep = MF16 ? (int)((W_KN ? 16 : 64) * P.ldw * 2) : 0;
    // per-lane offset register and scalar distance of weight wave-load j
    auto w_reg = [](int j) { return MF16 ? j % W_JP : j; };
    auto w_dist = [&](int j) __attribute__((always_inline)) { return (j - j % W_JP) * w_jstep; };

    // Direct load number `idx` (0 .. LPT-1: the A wave-loads, then the W wave-loads) of local k-tile
    // kt into `stage`.  A tile beyond the end of this split's k range is requested all the same, with
    // every lane out of range (it reads zeros and moves no data), so that the number of loads per
    // tile -- and with it every vmcnt below -- is the same in every iteration.
    // Persistent mode: the workgroups of step group g of G (XCD x of 8 without column bands) walk the k range
    // starting g/G of the way in and wrap around, so that the XCDs that read the same weight tiles -- and would ask
    // for the same lines at the same moment -- are spread over the k range (measured: 1 % of the pair's rank step).
    // The sum over k is taken in that rotated order: deterministic for a given launch, last-bit different between
    // step groups.
    const int rot = (PERSIST && P.k_rotate) ? (xcd_grp * nk_all) / xcd_groups : 0;
    auto ktile = [&](int kt) __attribute__((always_inline)) {                           // global k-tile of this item's local k-tile kt
        const int kk = ktb + kt + rot;
        return kk >= nk_all ? kk - nk_all : kk;
    };
    // With WHOLE_K (a k-tile known to be whole) the load is issued without any test: a
    // branch after every MFMA segment of the main loop costs more than it looks (measured: 4 - 6 % of the launch,
    // and a select on the offset still 1 %).  A tile beyond the end of the range is then fetched for real -- the
    // k-tile index wraps around (ktile), so it is a tile of the matrix -- into a stage that nobody reads.
    auto issue_load = [&](int kt, int stage_a, int stage_w, auto idx_tag, auto whole_k_tag) __attribute__((always_inline)) {
        constexpr int idx = decltype(idx_tag)::value;
        constexpr bool WHOLE_K = decltype(whole_k_tag)::value;
        const int k0 = ktile(kt) * BK;
        const unsigned sa = lds_base + stage_a * A_BYTES + wave * 1024;
        const unsigned sw = lds_base + W_BASE + stage_w * B_BYTES + wave * 1024;
        if constexpr (WHOLE_K) {
            if constexpr (idx < A_LD)
                direct_load_16(a_rsrc, a_off[MF16 ? 0 : idx], k0 * a_kstep + idx * a_jstep, sa + idx * NW * 1024);
            else
                direct_load_16(w_rsrc, b_off[w_reg(idx - A_LD)], k0 * w_kstep + w_dist(idx - A_LD), sw + (idx - A_LD) * NW * 1024);
            return;
        }
        const bool full = kt < nk && (k0 + BK) <= K;     // uniform: the common case needs no per-lane test
        if (full) {
            if constexpr (idx < A_LD)
                direct_load_16(a_rsrc, a_off[MF16 ? 0 : idx], k0 * a_kstep + idx * a_jstep, sa + idx * NW * 1024);
            else
                direct_load_16(w_rsrc, b_off[w_reg(idx - A_LD)], k0 * w_kstep + w_dist(idx - A_LD), sw + (idx - A_LD) * NW * 1024);
        } else {
            const bool none = kt >= nk;
            const int klim = none ? -1 : K;              // chunks at k >= klim read as zero
            const int ks0 = none ? 0 : k0;
            if constexpr (idx < A_LD) {
                const unsigned off = (k0 + chunk_k(idx, A_T, A_ROWB)) >= klim ? OOB : a_off[MF16 ? 0 : idx];
                direct_load_16(a_rsrc, off, ks0 * a_kstep + idx * a_jstep, sa + idx * NW * 1024);
            } else {
                constexpr int j = idx - A_LD;
                const unsigned off = (k0 + chunk_k(j, W_KN, W_ROWB)) >= klim ? OOB : b_off[w_reg(j)];
                direct_load_16(w_rsrc, off, ks0 * w_kstep + w_dist(j), sw + j * NW * 1024);
            }
        }
    };
    auto issue_range = [&](int kt, int stage_a, int stage_w, auto lo_tag, auto hi_tag) __attribute__((always_inline)) {   // loads [lo, hi) of a tile
        constexpr int lo = decltype(lo_tag)::value, hi = decltype(hi_tag)::value;
        static_assert(hi - lo <= 12, "at most twelve direct loads per tile and wave");
        const int k0 = ktile(kt) * BK;
        const unsigned sa = lds_base + stage_a * A_BYTES + wave * 1024;
        const unsigned sw = lds_base + W_BASE + stage_w * B_BYTES + wave * 1024;
        if (kt < nk && (k0 + BK) <= K) {                 // uniform: the common case, no per-lane test
#pragma unroll
            for (int idx = lo; idx < hi; ++idx) {
                if (idx < A_LD)
                    direct_load_16(a_rsrc, a_off[(!MF16 && idx < A_LD) ? idx : 0], k0 * a_kstep + idx * a_jstep, sa + idx * NW * 1024);
                else
                    direct_load_16(w_rsrc, b_off[idx >= A_LD ? w_reg(idx - A_LD) : 0], k0 * w_kstep + w_dist(idx - A_LD),
                                   sw + (idx - A_LD) * NW * 1024);
            }
        } else {
            if constexpr (lo + 0 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 0>{}, std::false_type{});
            if constexpr (lo + 1 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 1>{}, std::false_type{});
            if constexpr (lo + 2 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 2>{}, std::false_type{});
            if constexpr (lo + 3 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 3>{}, std::false_type{});
            if constexpr (lo + 4 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 4>{}, std::false_type{});
            if constexpr (lo + 5 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 5>{}, std::false_type{});
            if constexpr (lo + 6 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 6>{}, std::false_type{});
            if constexpr (lo + 7 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 7>{}, std::false_type{});
            if constexpr (lo + 8 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 8>{}, std::false_type{});
            if constexpr (lo + 9 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 9>{}, std::false_type{});
            if constexpr (lo + 10 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 10>{}, std::false_type{});
            if constexpr (lo + 11 < hi) issue_load(kt, stage_a, stage_w, std::integral_constant<int, lo + 11>{}, std::false_type{});
        }
    };

    // (MF16: the accumulators as the 16x16 tiles the MFMAs write, acc4[i][j][g] = registers 4g .. 4g+3 of sub-tile (i, j))
    f32x16_t acc[MF16 ? 1 : TM][MF16 ? 1 : TN];
    f32x4_t acc4[MF16 ? TM : 1][MF16 ? TN : 1][4];
    if constexpr (MF16) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    acc4[i][j][g] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    acc[i][j][e] = 0.0f;
    }
    // registers 4g .. 4g+3 of sub-tile (i, j)
    auto acc_get = [&](int i, int j, int g) __attribute__((always_inline)) {
        if constexpr (MF16) {
            return acc4[i][j][g];
        } else {
            f32x4_t o;
            o[0] = acc[i][j][4 * g + 0];
            o[1] = acc[i][j][4 * g + 1];
            o[2] = acc[i][j][4 * g + 2];
            o[3] = acc[i][j][4 * g + 3];
            return o;
        }
    };
    auto acc_set = [&](int i, int j, int g, f32x4_t v) __attribute__((always_inline)) {
        if constexpr (MF16) {
            acc4[i][j][g] = v;
        } else {
            acc[i][j][4 * g + 0] = v[0];
            acc[i][j][4 * g + 1] = v[1];
            acc[i][j][4 * g + 2] = v[2];
            acc[i][j][4 * g + 3] = v[3];
        }
    };

    // All-gather with the delivery carried by the consumer (GemmParams::land_step): the left operand comes in from the
    // neighbour's buffer, and each of its k-tiles is stored on to the landing buffer by ONE of the workgroups that
    // load it: the work item of tile column c takes the local k-tiles c, c + tiles_n, c + 2 tiles_n, ...  (All
    // items of a step and tile row walk k in the same order: the k rotation comes with whole steps per XCD.)
    // Every wave stores the 4 KiB it loaded itself -- it reads them back from the stage, whole 128-byte rows per
    // eight lanes, at the global offsets it fetched them from -- so its own vmcnt wait is all the ordering needed.
    constexpr bool CARRY_A = PERSIST && !RLDS && !A_T;
    int carry_at = (CARRY_A && cLand != nullptr && cRecv == nullptr) ? tile / tiles_m : 0x7fffffff;
    __amdgpu_buffer_rsrc_t la_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(cLand, 0, (CARRY_A && cLand != nullptr) ? (int)a_bytes : 0, 0x00020000);
    auto carry_tile = [&](int kt, int stage_a) __attribute__((always_inline)) {
        const int k0 = ktile(kt) * BK;
#pragma unroll
        for (int j = 0; j < A_LD; ++j) {
            const u32x4_t t = *reinterpret_cast<const u32x4_t *>(smem + stage_a * A_BYTES + (j * NW + wave) * 1024 + lane * 16);
            __builtin_amdgcn_raw_buffer_store_b128(t, la_rsrc, (int)a_off[MF16 ? 0 : j], k0 * 2 + j * a_jstep, 0);
        }
        carry_at += tiles_n;
    };

    // Fragment addressing (byte offsets inside a stage), fixed for the whole loop.  The swizzle
    // uses row bits 0..3 only, so the 32-row MFMA tiles of a wave differ by constants, and the
    // 16-wide k-slice ks is reached by XOR-ing (ks << 5) into the offset of slice 0.
    const int frow = lane & 31, fkc = lane >> 5;
    const int a_addr = swz_row(wm * WTM + frow, fkc);
    int a_addr_t[A_T ? TM : 1];
    if constexpr (A_T) {
        const int blk = lane >> 4, i16 = lane & 15;
        const int kl = (blk >> 1) * 8 + (i16 >> 2);
        const int ml = wm * WTM + (blk & 1) * 16 + (i16 & 3) * 4;        // row of tile i = 0
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int q = ((ml >> 5) + i) ^ (kl & 3);
            a_addr_t[i] = kl * A_ROWB + (q << 6) + (ml & 31) * 2;
        }
    } else {
        a_addr_t[0] = 0;
    }
    int w_addr[W_KN ? TN : 1];
    if constexpr (W_KN) {
        const int blk = lane >> 4, i16 = lane & 15;
        const int kl = (blk >> 1) * 8 + (i16 >> 2);                      // k of (ks = 0, h = 0)
        const int nl = wn * WTN + (blk & 1) * 16 + (i16 & 3) * 4;        // column of tile j = 0
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int q = ((nl >> 5) + j) ^ (kl & 3);
            w_addr[j] = W_BASE + kl * W_ROWB + (q << 6) + (nl & 31) * 2;
        }
    } else {
        w_addr[0] = W_BASE + swz_row(wn * WTN + frow, fkc);
    }

    // MF16: a fragment is 16 rows x 32 k: lane L holds row (L & 15) and one 16-byte chunk (8 k) of the 32-wide slice --
    // chunk 0, 2, 1, 3 for the lane blocks L >> 4 = 0, 1, 2, 3 (which eight k values sit in which slots of the
    // contraction is free as long as both operands agree; with this order the lanes L and L + 32 read an even and an
    // odd chunk, as they do in the 32x32x16 layout).  The second slice of a k-tile is reached by XOR-ing 64 into the
    // offset, 16-row tiles lie 2 KiB apart.  (The LDS bank-conflict counter shows 64 cycles per wave and k-tile for this
    // loop with either chunk order -- 2.5 % of a k-tile's time -- and none for the 32x32x16 loop.)
    constexpr int TN16 = WTN / 16;
    int a_addr16 = 0;
    // ([k x n] weights: one address per pair of 16-column tiles; the odd tile of a pair lies at that address ^ 32)
    int w_addr16[(MF16 && W_KN) ? TN16 / 2 : 1];
    if constexpr (MF16) {
        static_assert(!MF16 || (TM == 4 && TN == 2), "quarter phases are written for the 128x64 wave tile");
        const int kch = (((lane >> 4) & 1) << 1) | (lane >> 5);          // this lane's chunk of a slice
        a_addr16 = swz_row(wm * WTM + (lane & 15), kch);
        if constexpr (W_KN) {
            const int i16 = lane & 15;
            const int kl = kch * 8 + (i16 >> 2);                             // k of (slice 0, first half)
#pragma unroll
            for (int t = 0; t < TN16; t += 2) {
                const int nl = wn * WTN + t * 16 + (i16 & 3) * 4;
                const int q = (nl >> 5) ^ (kl & 3);
                w_addr16[t / 2] = W_BASE + kl * W_ROWB + (q << 6) + (((nl & 31) * 2) ^ (((kl >> 4) & 1) << 5));
            }
        } else {
            w_addr16[0] = W_BASE + swz_row(wn * WTN + (lane & 15), kch);
        }
    } else {
        w_addr16[0] = 0;
    }
    auto read_frags = [&](int stage_a, int stage_w, int ks, bf16x8_t (&af)[TM], bf16x8_t (&wf)[TN]) __attribute__((always_inline)) {
        const unsigned char *st = smem + stage_a * A_BYTES;
        const unsigned char *stw = smem + stage_w * B_BYTES;     // (w_addr holds the weight region's base)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (A_T) {
                const unsigned char *pa = st + a_addr_t[i] + ks * 16 * A_ROWB;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pa));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pa + 4 * A_ROWB));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                af[i] = __builtin_bit_cast(bf16x8_t, both);
            } else {
                af[i] = *reinterpret_cast<const bf16x8_t *>(st + (a_addr ^ (ks << 5)) + i * 32 * 128);
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (W_KN) {
                const unsigned char *pw = stw + w_addr[j] + ks * 16 * W_ROWB;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pw));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pw + 4 * W_ROWB));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                wf[j] = __builtin_bit_cast(bf16x8_t, both);
            } else {
                wf[j] = *reinterpret_cast<const bf16x8_t *>(stw + (w_addr[0] ^ (ks << 5)) + j * 32 * 128);
            }
        }
    };
    auto mfma_block = [&](const bf16x8_t (&af)[TM], const bf16x8_t (&wf)[TN]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
    };

    // One slice phase: the LDS reads of the NEXT slice's fragments (into afn, wfn), then the MFMAs of
    // the fragments in (afc, wfc) in NSEG segments.  The reads are interleaved with the MFMAs of the
    // first segment; after each segment one direct load of a later k-tile may be issued (load slots
    // LO .. LO+NSEG-1 of tile kt_l into stage_l), so that the wave never queues a burst of loads
    // behind which its MFMAs would wait.
    constexpr int NREAD = (A_T ? 2 * TM : TM) + (W_KN ? 2 * TN : TN);
    constexpr int NMFMA = TM * TN;
    constexpr int NSEG = NMFMA < 4 ? NMFMA : 4;
    constexpr int MPS = NMFMA / NSEG;                       // MFMAs per segment
    constexpr int LH = LPT < NSEG ? LPT : NSEG;             // loads issued in the first load phase
    static_assert(NMFMA % NSEG == 0 && (!SPREAD || LPT - LH <= NSEG), "segmenting");
    auto mfma_seg = [&](const bf16x8_t (&af)[TM], const bf16x8_t (&wf)[TN], auto seg_tag) __attribute__((always_inline)) {
        constexpr int seg = decltype(seg_tag)::value;
#pragma unroll
        for (int q = seg * MPS; q < (seg + 1) * MPS; ++q)
            acc[q / TN][q % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[q % TN], af[q / TN], acc[q / TN][q % TN], 0, 0, 0);
    };
    auto phase = [&](const bf16x8_t (&afc)[TM], const bf16x8_t (&wfc)[TN], bool do_read, int sa_n, int sw_n, int ks_n,
                     bf16x8_t (&afn)[TM], bf16x8_t (&wfn)[TN], int kt_l, int sa_l, int sw_l, auto lo_tag, auto n_tag,
                     auto whole_k_tag) __attribute__((always_inline)) {
        constexpr int LO = decltype(lo_tag)::value, NL = decltype(n_tag)::value;   // load slots of this phase
        if (do_read)
            read_frags(sa_n, sw_n, ks_n, afn, wfn);
        mfma_seg(afc, wfc, std::integral_constant<int, 0>{});
        interleave_mfma_reads<NREAD, (NREAD + MPS - 1) / MPS>();
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (NL > 0) issue_load(kt_l, sa_l, sw_l, std::integral_constant<int, LO>{}, whole_k_tag);
        if constexpr (NSEG > 1) {
            mfma_seg(afc, wfc, std::integral_constant<int, 1>{});
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NL > 1) issue_load(kt_l, sa_l, sw_l, std::integral_constant<int, LO + 1>{}, whole_k_tag);
        }
        if constexpr (NSEG > 2) {
            mfma_seg(afc, wfc, std::integral_constant<int, 2>{});
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NL > 2) issue_load(kt_l, sa_l, sw_l, std::integral_constant<int, LO + 2>{}, whole_k_tag);
        }
        if constexpr (NSEG > 3) {
            mfma_seg(afc, wfc, std::integral_constant<int, 3>{});
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NL > 3) issue_load(kt_l, sa_l, sw_l, std::integral_constant<int, LO + 3>{}, whole_k_tag);
        }
    };
    using c0 = std::integral_constant<int, 0>;
    using cLH = std::integral_constant<int, LH>;
    using cLR = std::integral_constant<int, LPT - LH>;
    using cLPT = std::integral_constant<int, LPT>;

    bf16x8_t af0[TM], wf0[TN], af1[TM], wf1[TN];

    // B_in prefetch (one workgroup per CU, fp32 output, no k-split): the epilogue's loads of the received
    // partial are issued pf_lead k-tiles before the end of the k loop and land in registers under the remaining
    // MFMAs, so that the epilogue only adds and stores.
    constexpr bool PF = !SPREAD && NS >= 3 && !OUT_BF16;
    constexpr int PFR = TM * TN * 4;                  // 16-byte loads per lane
    static_assert(!PF || (NS - 2) * LPT + PFR < 64, "vmcnt range");
    const unsigned r_bytes = (unsigned)(((int64_t)(M - 1) * P.ldo + N) * 4);
    const unsigned r_bytes_of_recv = r_bytes;
    __amdgpu_buffer_rsrc_t r_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(cRecv), 0, cRecv != nullptr ? (int)r_bytes : 0, 0x00020000);
    const int pf_at = nk - 1 - P.pf_lead;             // iteration after whose tile loads the prefetch is issued
    // Arrivals landed tile by tile by the work items of the steps before (GemmParams::tail_src): the last step's item
    // waits for its own tile's count before it reads them, in the epilogue.
    // (fp32 partial sums only, and never in the kernel that streams B_in: the launcher does not pick it for such a launch.)
    constexpr bool TAILS = PERSIST && !RLDS && !OUT_BF16;
    const bool wait_tiles = TAILS && P.tile_ready != nullptr && step_i == P.n_steps - 1;
    const bool pf_on = PF && cRecv != nullptr && splits == 1 && n_more == 0 && P.pf_lead > 0 && pf_at >= 0 && !wait_tiles;
    // The arrival that travels while this step computes (pairwise schedule: the partner's partial for the own slice):
    // this work item lands its own output tile's part of it -- from the sender's buffer to the landing buffer, written
    // through to memory (plain stores and a write-back of the L2 before the count take twice the whole launch's time)
    // -- and then counts the tile up for the step that sums the arrivals.  Every other workgroup of an XCD does so in
    // front of its main loop, the others behind their epilogue: the work items of a round run in lock step, and this
    // way one half copies while the other half multiplies instead of all 256 copying at once.
    constexpr int COHERENT_LD = 1 | 16;               // buffer cache-policy bits sc0 | sc1
    // The 16x16x32 main loop deals the copy over its k-tiles instead: one 16-byte load and the store of the one before
    // per lane and k-tile, behind the k-tile's barrier (the wait in front of the next barrier covers them: they are
    // older than the loads it lets pass), and what the k range leaves over is copied behind the epilogue.
    constexpr bool TL_STREAM = TAILS && MF16;
    constexpr int TL_CPR = WTN / 4, TL_RPI = 64 / TL_CPR, TL_N = WTM / TL_RPI;     // 16-byte chunks per row, rows and instructions per wave
    const float *const tl_src = TAILS ? P.tail_src[step_i] : nullptr;
    const bool tl_on = TL_STREAM && tl_src != nullptr;
    const bool tail_early = TAILS && !tl_on && (((int)blockIdx.x >> 3) & 1) != 0;
    const i32x4_t tl_srsrc = make_rsrc(tl_src, tl_src != nullptr ? r_bytes : 0u);
    __amdgpu_buffer_rsrc_t tl_drsrc = __builtin_amdgcn_make_buffer_rsrc(
        TAILS ? P.tail_dst[step_i] : nullptr, 0, tl_src != nullptr ? (int)r_bytes : 0, 0x00020000);
    const int tl_row0 = m0 + wm * WTM + lane / TL_CPR, tl_col = n0 + wn * WTN + (lane % TL_CPR) * 4;
    const int tl_voff = (tl_row0 < M && tl_col < N) ? (int)(((int64_t)tl_row0 * P.ldo + tl_col) * 4) : (int)OOB;
    const int tl_stride = (int)((int64_t)TL_RPI * P.ldo * 4);                      // bytes from one instruction's rows to the next's
    int tl_c = 0;                                    // instructions issued so far
    u32x4_t tl_v = {0u, 0u, 0u, 0u};
    auto tl_step = [&]() __attribute__((always_inline)) {
        if (tl_on) {
            if (tl_c > 0 && tl_c <= TL_N)
                __builtin_amdgcn_raw_buffer_store_b128(tl_v, tl_drsrc, tl_voff, (tl_c - 1) * tl_stride, COHERENT_LD);
            // (the load is awaited by the wait in front of the next k-tile's barrier: it is older than the four
            // left-operand loads that wait lets pass)
            if (tl_c < TL_N)
                tl_v = load_16_unawaited(tl_srsrc, (unsigned)tl_voff, tl_c * tl_stride);
            ++tl_c;
        }
    };
    auto land_arrival = [&](int first) __attribute__((always_inline)) {
        const float *const tsrc = tl_src;
        if (TAILS && tsrc != nullptr) {
            __amdgpu_buffer_rsrc_t ts_rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(tsrc), 0, (int)r_bytes, 0x00020000);
            __amdgpu_buffer_rsrc_t td_rsrc = __builtin_amdgcn_make_buffer_rsrc(P.tail_dst[step_i], 0, (int)r_bytes, 0x00020000);
            constexpr int CPR = WTN / 4;             // 16-byte chunks in a row of the wave's part
            constexpr int RPI = 64 / CPR;            // rows per instruction
            constexpr int TB = 16;                   // loads in flight per lane
            static_assert(64 % CPR == 0 && (WTM / RPI) % TB == 0, "whole batches");
            const int sn = n0 + wn * WTN + (lane % CPR) * 4;
#pragma unroll 1
            for (int b = first; b < WTM / RPI; b += TB) {
                u32x4_t v[TB];
                int off[TB];
#pragma unroll
                for (int u = 0; u < TB; ++u) {
                    const int sm = m0 + wm * WTM + (b + u) * RPI + lane / CPR;
                    off[u] = (b + u < WTM / RPI && sm < M && sn < N) ? (int)(((int64_t)sm * P.ldo + sn) * 4) : (int)OOB;
                    v[u] = __builtin_amdgcn_raw_buffer_load_b128(ts_rsrc, off[u], 0, 0);
                }
#pragma unroll
                for (int u = 0; u < TB; ++u)
                    __builtin_amdgcn_raw_buffer_store_b128(v[u], td_rsrc, off[u], 0, COHERENT_LD);
            }
            if (P.tile_ready != nullptr) {           // (nobody waits for a copy that only lands this step's own B_in)
                __builtin_amdgcn_s_waitcnt(0);       // this wave's stores are acknowledged
                __syncthreads();                     // ... and every wave's
                if (tid == 0)
                    __hip_atomic_fetch_add(&P.tile_ready[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };
    if (TAILS && tail_early)
        land_arrival(0);
    f32x4_t pre[PF ? TM : 1][PF ? TN : 1][4];
    auto prefetch_recv = [&](auto aux_tag) __attribute__((always_inline)) {
        constexpr int AUX = decltype(aux_tag)::value;
#pragma unroll
        for (int i = 0; i < (PF ? TM : 0); ++i) {
            const int m = m0 + wm * WTM + i * 32 + (lane & 31);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n0 + wn * WTN + j * 32 + g * 8 + (lane >> 5) * 4;
                    const unsigned e = (m < M && n < N) ? (unsigned)((int64_t)m * P.ldo + n) : OOB;
                    pre[i][j][g] = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                        r_rsrc, e == OOB ? (int)OOB : (int)(e * 4), 0, AUX));
                }
        }
    };

    // RLDS: is B_in streamed in under the main loop for this work item?  (Uniform.)  It needs sixteen k-tiles
    // before the last one (and before the iterations that test their loads), and one more for the change of
    // schedule in front of them; a step that waits for a delivery flag, sums several received partials or is a
    // k-split keeps the loads in the epilogue.
    constexpr int RQ = TM * TN;                       // 32x32 sub-tiles per wave, one in flight at a time
    // A ragged k tail (the launcher then leaves the k order unrotated: it is the last k-tile) is requested in the
    // last two iterations before the final tile; those test their loads and come after the streamed ones.
    const int tested = (RLDS && K % BK != 0) ? (nk - 1 < 2 ? nk - 1 : 2) : 0;
    const bool streamed = RLDS && cRecv != nullptr && cFlag == nullptr && !wait_tiles && n_more == 0 && splits == 1 &&
                          P.stream_recv && nk >= 2 * RQ + 2 + tested && (tested == 0 || rot == 0);
    // the left-operand stage whose memory serves as the wave-private scratch of the epilogue's stores (and, RLDS, as
    // the landing area of B_in before)
    int land_stage = SPREAD ? NSA - 1 : 0;
    if constexpr (SPREAD && MF16) {
        // The schedule of the 256x256 tile (see the variant below for its reasoning) on 16x16x32 MFMAs.  A k-tile is two
        // 32-wide slices; a slice is consumed in four quarter phases, phase p = the wave tile's 32-row block p:
        // 2 left-operand fragments (16-row tiles x = 0, 1) x 4 weight fragments = 8 MFMAs, in four segments of two
        // (segments 0, 1: x = 0; segments 2, 3: x = 1).  A phase is short (128 cycles of MFMA issue), so LDS reads and
        // direct loads are dealt out thinly -- at most one fragment read and one direct load per segment -- and every
        // fragment register is refilled as soon as its last MFMA has issued, a phase and a half before its next use:
        // the left-operand fragments live in two buffers that alternate by phase (afA: even phases), and phase q reads
        //     at segment 0: fragment x = 1 of phase q+1, into the other buffer (its last use was in phase q-1);
        //     at segment 2: fragment x = 0 of phase q+2, into its own buffer;
        // the weight fragments live in two buffers that alternate by slice; those of slice 1 are read one per phase in
        // phases 0 .. 3, those of slice 0 of the next tile two per phase in phases 6 and 7 (segments 1 and 3).
        //   steady state, tile kt (phases 0 .. 7 = slice 0 blocks 0 .. 3, slice 1 blocks 0 .. 3):
        //     phases 0 .. 3: + one left-operand load of tile kt+NS each, into the stage tile kt-1 vacated
        //     phase 6, after segment 0 (the last read of tile kt has been issued):
        //              wait: tile kt+1 complete; barrier: tile kt has been read by all;
        //              then the first reads of tile kt+1, and in phases 6 and 7 + two weight loads of tile kt+NS each
        static_assert(A_LD == 4 && B_LD == 4, "load slots below: four loads per operand, tile and wave");
        using p0_t = std::integral_constant<int, 0>;
        using p1_t = std::integral_constant<int, 1>;
        using p2_t = std::integral_constant<int, 2>;
        using p3_t = std::integral_constant<int, 3>;
        using c1 = std::integral_constant<int, 1>;
        using c2 = std::integral_constant<int, 2>;
        using on_t = std::true_type;
        using off_t = std::false_type;
        bf16x8_t afA[2], afB[2], wfA[4], wfB[4];
        // the two MFMAs of segment seg of a phase on block PB: 16-row tile x = seg / 2, 16-column tiles 2 (seg & 1) + {0, 1}
        auto mfma16_seg = [&](auto pb_tag, const bf16x8_t (&af)[2], const bf16x8_t (&wf)[4], auto seg_tag) __attribute__((always_inline)) {
            constexpr int PB = decltype(pb_tag)::value, seg = decltype(seg_tag)::value;
            constexpr int x = seg >> 1, j = seg & 1;
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const int g = 2 * x + y;
                acc4[MF16 ? PB : 0][MF16 ? j : 0][g] =
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[2 * j + y], af[x], acc4[MF16 ? PB : 0][MF16 ? j : 0][g], 0, 0, 0);
            }
        };
        auto frag_a16 = [&](int stage_a, int sl, int t16) __attribute__((always_inline)) {
            return *reinterpret_cast<const bf16x8_t *>(smem + stage_a * A_BYTES + (a_addr16 ^ (sl << 6)) + t16 * 2048);
        };
        auto frag_w16 = [&](int stage_w, int sl, auto t_tag) __attribute__((always_inline)) {
            constexpr int t = decltype(t_tag)::value;
            const unsigned char *stw = smem + stage_w * B_BYTES;
            if constexpr (W_KN) {
                const unsigned char *pw = stw + (w_addr16[(MF16 && W_KN) ? t / 2 : 0] ^ ((t & 1) << 5)) + sl * 32 * W_ROWB;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t *)(pw));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t *)(pw + 4 * W_ROWB));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(bf16x8_t, both);
            } else {
                return *reinterpret_cast<const bf16x8_t *>(stw + (w_addr16[0] ^ (sl << 6)) + t * 2048);
            }
        };
        constexpr int NRD_WF = W_KN ? 2 : 1;                 // LDS reads of one weight fragment
        auto nothing = [&]() __attribute__((always_inline)) {};
        // One quarter phase on block PB with the fragments (afc, wfc).
        //   r1: fragment x = 1 of (stage s1, slice l1, block b1) into afo[1] at segment 0;  mid(): between segments 0 and 1;
        //   nwf weight fragments w0, w0 + 1 of (stage sw, slice lw) into wfn at segments 1 and 3;
        //   r2: fragment x = 0 of (s2, l2, b2) into afc[0] at segment 2;
        //   ld1(), ld3(): direct loads issued at segments 1 and 3.
        auto phase16 = [&](auto pb_tag, bf16x8_t (&afc)[2], const bf16x8_t (&wfc)[4], bf16x8_t (&afo)[2], bf16x8_t (&wfn)[4],
                           auto r1_tag, int s1, int l1, int b1, auto mid, auto nwf_tag, int sw, int lw, auto w0_tag,
                           auto r2_tag, int s2, int l2, int b2, auto ld1, auto ld3) __attribute__((always_inline)) {
            constexpr bool R1 = decltype(r1_tag)::value, R2 = decltype(r2_tag)::value;
            constexpr int NWF = decltype(nwf_tag)::value, W0 = decltype(w0_tag)::value;
            if constexpr (R1)
                afo[1] = frag_a16(s1, l1, 2 * b1 + 1);
            mfma16_seg(pb_tag, afc, wfc, std::integral_constant<int, 0>{});
            interleave_mfma_reads<R1 ? 1 : 0, 1>();
            __builtin_amdgcn_sched_barrier(0);
            mid();
            if constexpr (NWF > 0)
                wfn[W0] = frag_w16(sw, lw, std::integral_constant<int, W0>{});
            ld1();
            mfma16_seg(pb_tag, afc, wfc, std::integral_constant<int, 1>{});
            interleave_mfma_reads<((NWF > 0) ? NRD_WF : 0), 1>();
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (R2)
                afc[0] = frag_a16(s2, l2, 2 * b2);
            mfma16_seg(pb_tag, afc, wfc, std::integral_constant<int, 2>{});
            interleave_mfma_reads<R2 ? 1 : 0, 1>();
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NWF > 1)
                wfn[W0 + 1] = frag_w16(sw, lw, std::integral_constant<int, W0 + 1>{});
            ld3();
            mfma16_seg(pb_tag, afc, wfc, std::integral_constant<int, 3>{});
            interleave_mfma_reads<((NWF > 1) ? NRD_WF : 0), 1>();
            __builtin_amdgcn_sched_barrier(0);
        };
        // Phases 0 .. 5 of a tile in stages (ca, cw); ldq(q): the direct load phase q (0 .. 3) issues (at its segment 1).
        auto front16 = [&](int ca, int cw, auto ld0, auto ld1_, auto ld2, auto ld3_, auto ph2) __attribute__((always_inline)) {
            phase16(p0_t{}, afA, wfA, afB, wfB, on_t{}, ca, 0, 1, nothing, c1{}, cw, 1, c0{}, on_t{}, ca, 0, 2, ld0, nothing);
            phase16(p1_t{}, afB, wfA, afA, wfB, on_t{}, ca, 0, 2, nothing, c1{}, cw, 1, c1{}, on_t{}, ca, 0, 3, ld1_, nothing);
            ph2(ld2);
            phase16(p3_t{}, afB, wfA, afA, wfB, on_t{}, ca, 1, 0, nothing, c1{}, cw, 1, std::integral_constant<int, 3>{}, on_t{}, ca, 1, 1, ld3_, nothing);
            phase16(p0_t{}, afA, wfB, afB, wfA, on_t{}, ca, 1, 1, nothing, c0{}, 0, 0, c0{}, on_t{}, ca, 1, 2, nothing, nothing);
            phase16(p1_t{}, afB, wfB, afA, wfA, on_t{}, ca, 1, 2, nothing, c0{}, 0, 0, c0{}, on_t{}, ca, 1, 3, nothing, nothing);
        };
        // phase 2 of a tile in stages (ca, cw) as a plain phase
        auto plain_ph2 = [&](int ca, int cw) __attribute__((always_inline)) {
            return [&, ca, cw](auto ld2) __attribute__((always_inline)) {
                phase16(p2_t{}, afA, wfA, afB, wfB, on_t{}, ca, 0, 3, nothing, c1{}, cw, 1, c2{}, on_t{}, ca, 1, 0, ld2, nothing);
            };
        };

    #pragma unroll
        for (int t = 0; t < NS; ++t)
            issue_range(t, t, t, c0{}, cLPT{});
        wait_vmcnt<(NS - 1) * LPT>();
        __syncthreads();
        afA[0] = frag_a16(0, 0, 0);
        afA[1] = frag_a16(0, 0, 1);
        afB[0] = frag_a16(0, 0, 2);
        wfA[0] = frag_w16(0, 0, std::integral_constant<int, 0>{});
        wfA[1] = frag_w16(0, 0, std::integral_constant<int, 1>{});
        wfA[2] = frag_w16(0, 0, std::integral_constant<int, 2>{});
        wfA[3] = frag_w16(0, 0, std::integral_constant<int, 3>{});
        __builtin_amdgcn_sched_barrier(0);

        int cur_a = 0, cur_w = 0;                        // stages of tile kt
        int prev_a = NSA - 1;                            // left-operand stage of tile kt-1 (= of tile kt+NS)
        auto body = [&](int kt, int ca, int cw, int pa, int na, int nw_, auto wk) __attribute__((always_inline)) {
            auto la = [&](auto idx_tag) __attribute__((always_inline)) {       // a left-operand load of tile kt+NS
                return [&, kt, pa](/*no args*/) __attribute__((always_inline)) { issue_load(kt + NS, pa, 0, decltype(idx_tag){}, wk); };
            };
            auto lw = [&](auto idx_tag) __attribute__((always_inline)) {       // a weight load of tile kt+NS
                return [&, kt, cw]() __attribute__((always_inline)) { issue_load(kt + NS, 0, cw, decltype(idx_tag){}, wk); };
            };
            front16(ca, cw, la(std::integral_constant<int, 0>{}), la(std::integral_constant<int, 1>{}),
                    la(std::integral_constant<int, 2>{}), la(std::integral_constant<int, 3>{}), plain_ph2(ca, cw));
            auto publish = [&]() __attribute__((always_inline)) {
                if (CARRY_A && kt == carry_at) {     // tile kt goes on to the landing buffer: its stores are the
                    carry_tile(kt, ca);              // youngest requests and need not be awaited here
                    wait_vmcnt<(NS - 2) * LPT + 2 * A_LD>();
                } else {
                    wait_vmcnt<(NS - 2) * LPT + A_LD>();
                }
                __syncthreads();
                if constexpr (TL_STREAM)
                    tl_step();
                __builtin_amdgcn_sched_barrier(0);
            };
            phase16(p2_t{}, afA, wfB, afB, wfA, on_t{}, ca, 1, 3, publish, c2{}, nw_, 0, c0{}, on_t{}, na, 0, 0,
                    lw(std::integral_constant<int, 4>{}), lw(std::integral_constant<int, 5>{}));
            phase16(p3_t{}, afB, wfB, afA, wfA, on_t{}, na, 0, 0, nothing, c2{}, nw_, 0, c2{}, on_t{}, na, 0, 1,
                    lw(std::integral_constant<int, 6>{}), lw(std::integral_constant<int, 7>{}));
        };
        // first iteration that tests its loads (all of them when K is a multiple of the k-tile: none does)
        const int tested_at = K % BK == 0 ? nk - 1 : ((rot == 0 && nk - 1 > NS) ? nk - 1 - NS : 0);
        int kt = 0;
        for (; kt < tested_at; ++kt) {
            const int nxt_a = (cur_a + 1 == NSA) ? 0 : cur_a + 1;
            const int nxt_w = (cur_w + 1 == NS) ? 0 : cur_w + 1;
            body(kt, cur_a, cur_w, prev_a, nxt_a, nxt_w, std::true_type{});
            prev_a = cur_a;
            cur_a = nxt_a;
            cur_w = nxt_w;
        }
        // the last tile of a work item: nothing follows it
        auto last16 = [&](int ca, int cw) __attribute__((always_inline)) {
            front16(ca, cw, nothing, nothing, nothing, nothing, plain_ph2(ca, cw));
            phase16(p2_t{}, afA, wfB, afB, wfA, on_t{}, ca, 1, 3, nothing, c0{}, 0, 0, c0{}, off_t{}, 0, 0, 0, nothing, nothing);
            if (CARRY_A && nk - 1 == carry_at)
                carry_tile(nk - 1, ca);
            phase16(p3_t{}, afB, wfB, afA, wfA, off_t{}, 0, 0, 0, nothing, c0{}, 0, 0, c0{}, off_t{}, 0, 0, 0, nothing, nothing);
        };
        for (; kt + 1 < nk; ++kt) {
            const int nxt_a = (cur_a + 1 == NSA) ? 0 : cur_a + 1;
            const int nxt_w = (cur_w + 1 == NS) ? 0 : cur_w + 1;
            body(kt, cur_a, cur_w, prev_a, nxt_a, nxt_w, std::false_type{});
            prev_a = cur_a;
            cur_a = nxt_a;
            cur_w = nxt_w;
        }
        if (nk > 0)
            last16(cur_a, cur_w);
    } else if constexpr (SPREAD) {
        // The left-operand tile has NS+1 stages, the weight tile NS (tile t lives in stages t mod (NS+1) and
        // t mod NS).  Loads return in issue order, so what is issued first must be what is needed first:
        //   prologue: tiles 0 .. NS-1 whole, in tile order; tile 0 is awaited, its first fragments fetched
        //   steady state, tile kt:
        //     slice 0: + the left-operand loads of tile kt+NS, into the stage tile kt-1 vacated
        //     slice 1, slice 2
        //     wait: tile kt+1 complete -- the loads of NS-2 later whole tiles and the left-operand loads
        //           just issued may be in flight; barrier: tile kt has been read by all
        //     slice 3: + the weight loads of tile kt+NS, into the stage tile kt vacated
        // A weight load thus has 1 to 1.25 k-tiles of MFMA time to arrive and a left-operand load 1.75 to 2
        // (with NS = 2; both NS-2 more otherwise).
        static_assert(A_LD == LH && LPT - LH == B_LD, "one load slot per MFMA segment and operand");
        using cALD = std::integral_constant<int, A_LD>;
    #pragma unroll
        for (int t = 0; t < NS; ++t)
            issue_range(t, t, t, c0{}, cLPT{});
        wait_vmcnt<(NS - 1) * LPT>();
        __syncthreads();
        read_frags(0, 0, 0, af0, wf0);
        __builtin_amdgcn_sched_barrier(0);

        // The steady state.  When K is a multiple of the k-tile every iteration is branch-free.  Otherwise (the
        // launcher then leaves the k order unrotated) the ragged k-tile is the last one of the range: the
        // iterations up to the one that requests it are branch-free too, and only the last NS ones test.
        int cur_a = 0, cur_w = 0;                        // stages of tile kt
        int prev_a = NSA - 1;                            // left-operand stage of tile kt-1 (= of tile kt+NS)
        auto body = [&](int kt, int ca, int cw, int pa, int na, int nw_, auto wk) __attribute__((always_inline)) {
            phase(af0, wf0, true, ca, cw, 1, af1, wf1, kt + NS, pa, 0, c0{}, cALD{}, wk);
            phase(af1, wf1, true, ca, cw, 2, af0, wf0, 0, 0, 0, c0{}, c0{}, wk);
            phase(af0, wf0, true, ca, cw, 3, af1, wf1, 0, 0, 0, c0{}, c0{}, wk);
            if (CARRY_A && kt == carry_at) {         // tile kt goes on to the landing buffer: its stores are the
                carry_tile(kt, ca);                  // youngest requests and need not be awaited here
                wait_vmcnt<(NS - 2) * LPT + 2 * A_LD>();
            } else {
                wait_vmcnt<(NS - 2) * LPT + A_LD>();
            }
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            phase(af1, wf1, true, na, nw_, 0, af0, wf0, kt + NS, 0, cw, cALD{}, cLR{}, wk);
        };
        // first iteration that tests its loads (all of them when K is a multiple of the k-tile: none does)
        const int tested_at = K % BK == 0 ? nk - 1 : ((rot == 0 && nk - 1 > NS) ? nk - 1 - NS : 0);
        // RLDS, a work item that streams B_in: the three-stage schedule runs up to the k-tile before the sixteen
        // streamed ones, the two-stage schedule with the landing area (below) takes over there
        const int change_at = nk - 1 - tested - 2 * RQ - 1;
        const int plain_end = (RLDS && streamed) ? change_at : tested_at;
        int kt = 0;
        for (; kt < plain_end; ++kt) {
            const int nxt_a = (cur_a + 1 == NSA) ? 0 : cur_a + 1;
            const int nxt_w = (cur_w + 1 == NS) ? 0 : cur_w + 1;
            body(kt, cur_a, cur_w, prev_a, nxt_a, nxt_w, std::true_type{});
            prev_a = cur_a;
            cur_a = nxt_a;
            cur_w = nxt_w;
        }
        if (!(RLDS && streamed)) {
            for (; kt + 1 < nk; ++kt) {
                const int nxt_a = (cur_a + 1 == NSA) ? 0 : cur_a + 1;
                const int nxt_w = (cur_w + 1 == NS) ? 0 : cur_w + 1;
                body(kt, cur_a, cur_w, prev_a, nxt_a, nxt_w, std::false_type{});
                prev_a = cur_a;
                cur_a = nxt_a;
                cur_w = nxt_w;
            }
            if (nk > 0) {                                    // last tile: nothing follows it
                using wk = std::true_type;
                phase(af0, wf0, true, cur_a, cur_w, 1, af1, wf1, 0, 0, 0, c0{}, c0{}, wk{});
                phase(af1, wf1, true, cur_a, cur_w, 2, af0, wf0, 0, 0, 0, c0{}, c0{}, wk{});
                phase(af0, wf0, true, cur_a, cur_w, 3, af1, wf1, 0, 0, 0, c0{}, c0{}, wk{});
                if (CARRY_A && nk - 1 == carry_at)
                    carry_tile(nk - 1, cur_a);
                phase(af1, wf1, false, 0, 0, 0, af0, wf0, 0, 0, 0, c0{}, c0{}, wk{});
            }
        }
        if constexpr (RLDS) {
          if (streamed) {
            // The streamed part: two stages of both operands and the landing area.  On entry (kt = change_at) tile
            // kt is complete and all of tile kt+1 is in flight; the left-operand tiles kt and kt+1 keep their
            // stages, later ones alternate between the two, and the third stage -- tile kt-1 has been read by all
            // -- becomes the landing area, 4 KiB per wave.  Weight tile t stays in stage t & 1.  Iteration kt:
            //     slice 0: + the weight loads of tile kt+1 (its stage was vacated at the barrier of iteration kt-1;
            //              not in the first iteration, where they are in flight already)
            //     slice 1 (X iterations: + the four B_in loads of one sub-tile), slice 2
            //     wait: tile kt+1 complete (X: the B_in loads just issued may still be in flight); barrier
            //     (Y iterations: the sub-tile is read from the landing area and added to its accumulators)
            //     slice 3: + the left-operand loads of tile kt+2, into the stage tile kt vacated
            // Loads return in issue order: the B_in loads of an X iteration are behind the weight loads of tile
            // kt+1 and ahead of everything tile kt+2 needs, so they have until the wait of the following (Y)
            // iteration, one and a half k-tiles of MFMA time, to arrive.  Each wave reads back only what it
            // loaded itself, so its own vmcnt wait is all the ordering the landing area needs.
            static_assert(A_LD <= NSEG && B_LD <= NSEG && NSEG == 4 && NS == 2, "one load slot per MFMA segment");
            const int nxt_a0 = (cur_a + 1 == NSA) ? 0 : cur_a + 1;
            const int a_of_parity[2] = {(kt & 1) ? nxt_a0 : cur_a, (kt & 1) ? cur_a : nxt_a0};
            land_stage = prev_a;                         // (the stage of tile kt-1; kt >= 1 here)
            const int a_ev = a_of_parity[0], a_od = a_of_parity[1];
            const i32x4_t rr = make_rsrc(cRecv, r_bytes_of_recv);
            __amdgpu_buffer_rsrc_t l_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                static_cast<float *>(cLand), 0, cLand != nullptr ? (int)r_bytes_of_recv : 0, 0x00020000);
            const int land_off = land_stage * A_BYTES + wave * 4096;
            const unsigned r_lds = lds_base + land_off;
            // byte offset of sub-tile q = (i, j) of this wave, row 0 / column 0 of the lane pattern
            auto r_soff = [&](int q) __attribute__((always_inline)) {
                const int i = q / TN, j = q % TN;
                return (int)((((int64_t)(m0 + wm * WTM + i * 32)) * P.ldo + n0 + wn * WTN + j * 32) * 4);
            };
            auto phase_x = [&](const bf16x8_t (&afc)[TM], const bf16x8_t (&wfc)[TN], int sa_n, int sw_n, int ks_n,
                               bf16x8_t (&afn)[TM], bf16x8_t (&wfn)[TN], int q) __attribute__((always_inline)) {
                const int so = __builtin_amdgcn_readfirstlane(r_soff(q));     // (uniform; kept in a scalar register)
                // a lane outside the matrix must not touch memory: the scalar part of the address is not covered
                // by the buffer's range check, so such a lane is given the out-of-range offset itself
                // (computed from an opaque copy of the lane index: otherwise the offsets of all eight sub-tiles are
                // hoisted out of the k loop and held in registers the main loop does not have)
                int ln = lane;
                asm volatile("" : "+v"(ln));
                // Plane g of the landing area (load g: columns 8g + 4 (lane >> 5) .. + 3) holds its rows permuted:
                // the lane fetches row (lane & 31) ^ (2g + (lane >> 5)), so that the eight 16-byte chunks of a row,
                // which lie 512 bytes apart across the planes, fall into different banks when the rows are read
                // back eight lanes to a row.
                const int half = ln >> 5;
                const int rn = n0 + wn * WTN + (q % TN) * 32 + half * 4;
                auto off_of = [&](int g) __attribute__((always_inline)) {
                    const int r = (ln & 31) ^ (2 * g + half);
                    const int rm = m0 + wm * WTM + (q / TN) * 32 + r;
                    return (rm < M && rn + 8 * g < N) ? (unsigned)((((int64_t)r) * P.ldo + half * 4) * 4) : OOB;
                };
                const unsigned v0 = off_of(0), v1 = off_of(1), v2 = off_of(2), v3 = off_of(3);
                read_frags(sa_n, sw_n, ks_n, afn, wfn);
                mfma_seg(afc, wfc, std::integral_constant<int, 0>{});
                interleave_mfma_reads<NREAD, (NREAD + MPS - 1) / MPS>();
                __builtin_amdgcn_sched_barrier(0);
                direct_load_16(rr, v0, so, r_lds);
                mfma_seg(afc, wfc, std::integral_constant<int, 1>{});
                __builtin_amdgcn_sched_barrier(0);
                direct_load_16(rr, v1, so + 32, r_lds + 1024);
                mfma_seg(afc, wfc, std::integral_constant<int, 2>{});
                __builtin_amdgcn_sched_barrier(0);
                direct_load_16(rr, v2, so + 64, r_lds + 2048);
                mfma_seg(afc, wfc, std::integral_constant<int, 3>{});
                __builtin_amdgcn_sched_barrier(0);
                direct_load_16(rr, v3, so + 96, r_lds + 3072);
            };
            auto add_landed = [&](auto q_tag) __attribute__((always_inline)) {          // "O <- B_in + O" for sub-tile q, in mid-sum
                constexpr int q = decltype(q_tag)::value;
                int ln = lane;
                asm volatile("" : "+v"(ln));
                const unsigned char *src = smem + land_off + (ln & 32) * 16;
                f32x4_t v[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    v[g] = *reinterpret_cast<const f32x4_t *>(src + g * 1024 + (((ln & 31) ^ (2 * g + (ln >> 5))) << 4));
                    acc[q / TN][q % TN][4 * g + 0] += v[g][0];
                    acc[q / TN][q % TN][4 * g + 1] += v[g][1];
                    acc[q / TN][q % TN][4 * g + 2] += v[g][2];
                    acc[q / TN][q % TN][4 * g + 3] += v[g][3];
                }
                // the delivery carried by the consumer: what just arrived from the neighbour's buffer is also stored to
                // this rank's landing buffer (a lane outside the matrix is given the out-of-range offset: store dropped)
                if (cLand != nullptr) {
                    // Whole 128-byte lines per store: the sub-tile is read from the landing area a second time, eight
                    // lanes to a row (chunk c of row r lies in plane c / 2 at lane slot (r ^ c) + 32 (c & 1)), so that
                    // one store instruction writes eight full rows instead of 32-byte pieces of thirty-two.
                    const int c = ln & 7, r8 = ln >> 3;
                    const unsigned char *base = smem + land_off + (c >> 1) * 1024 + (32 * (c & 1)) * 16;
                    const int rn = n0 + wn * WTN + (q % TN) * 32 + c * 4;
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4) {
                        const int row = 8 * s4 + r8;
                        const f32x4_t t = *reinterpret_cast<const f32x4_t *>(base + ((row ^ c) << 4));
                        const int rm = m0 + wm * WTM + (q / TN) * 32 + row;
                        const int boff = (rm < M && rn < N) ? (int)(((int64_t)rm * P.ldo + rn) * 4) : (int)OOB;
                        // (plain stores: non-temporal or write-through ones measured 10 - 30 % slower here)
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, t), l_rsrc, boff, 0, 0);
                    }
                }
            };
            // mode 0: plain; mode 1 (X): issues the B_in loads of sub-tile q; mode 2 (Y): adds sub-tile Q.
            // n_w: the number of weight loads slice 0 issues (none in the iteration that takes over)
            auto iteration_wk = [&](int kt_, auto mode_tag, int q, auto q_tag, auto wk, auto n_w) __attribute__((always_inline)) {
                constexpr int MODE = decltype(mode_tag)::value;
                const int cw = kt_ & 1, nw_ = cw ^ 1;
                const int ca = cw ? a_od : a_ev, na = cw ? a_ev : a_od;
                phase(af0, wf0, true, ca, cw, 1, af1, wf1, kt_ + 1, 0, nw_, cALD{}, n_w, wk);
                if constexpr (MODE == 1)
                    phase_x(af1, wf1, ca, cw, 2, af0, wf0, q);
                else
                    phase(af1, wf1, true, ca, cw, 2, af0, wf0, 0, 0, 0, c0{}, c0{}, wk);
                phase(af0, wf0, true, ca, cw, 3, af1, wf1, 0, 0, 0, c0{}, c0{}, wk);
                if constexpr (MODE == 1)
                    wait_vmcnt<4>();
                else
                    wait_vmcnt<0>();
                __syncthreads();
                if constexpr (MODE == 2)
                    add_landed(q_tag);
                __builtin_amdgcn_sched_barrier(0);
                phase(af1, wf1, true, na, nw_, 0, af0, wf0, kt_ + 2, ca, 0, c0{}, cALD{}, wk);
            };
            using m0_t = std::integral_constant<int, 0>;
            using m1_t = std::integral_constant<int, 1>;
            using m2_t = std::integral_constant<int, 2>;
            iteration_wk(kt, m0_t{}, 0, c0{}, std::true_type{}, c0{});       // the iteration that takes over
            ++kt;
            auto pair_of = [&](auto q_tag) __attribute__((always_inline)) {
                iteration_wk(kt, m1_t{}, decltype(q_tag)::value, c0{}, std::true_type{}, cLR{});
                iteration_wk(kt + 1, m2_t{}, 0, q_tag, std::true_type{}, cLR{});
                kt += 2;
            };
            static_assert(RQ == 8, "eight sub-tiles per wave");
            pair_of(std::integral_constant<int, 0>{});
            pair_of(std::integral_constant<int, 1>{});
            pair_of(std::integral_constant<int, 2>{});
            pair_of(std::integral_constant<int, 3>{});
            pair_of(std::integral_constant<int, 4>{});
            pair_of(std::integral_constant<int, 5>{});
            pair_of(std::integral_constant<int, 6>{});
            pair_of(std::integral_constant<int, 7>{});
            for (; kt + 1 < nk; ++kt)                        // the iterations that request the ragged k-tile
                iteration_wk(kt, m0_t{}, 0, c0{}, std::false_type{}, cLR{});
            {                                                // last tile: nothing follows it
                using wk = std::true_type;
                const int cw = (nk - 1) & 1, ca = cw ? a_od : a_ev;
                phase(af0, wf0, true, ca, cw, 1, af1, wf1, 0, 0, 0, c0{}, c0{}, wk{});
                phase(af1, wf1, true, ca, cw, 2, af0, wf0, 0, 0, 0, c0{}, c0{}, wk{});
                phase(af0, wf0, true, ca, cw, 3, af1, wf1, 0, 0, 0, c0{}, c0{}, wk{});
                phase(af1, wf1, false, 0, 0, 0, af0, wf0, 0, 0, 0, c0{}, c0{}, wk{});
            }
          }
        }
    } else {
        // Variant for the small tiles (few MFMAs per slice): a tile's loads go out together right
        // after the barrier that frees their stage, and the LDS reads of the next slice are
        // interleaved with all MFMAs of the current one.
        auto phase_b = [&](const bf16x8_t (&afc)[TM], const bf16x8_t (&wfc)[TN], bool do_read, int stage_n, int ks_n,
                           bf16x8_t (&afn)[TM], bf16x8_t (&wfn)[TN], auto rpm_tag) __attribute__((always_inline)) {
            constexpr int RPM = decltype(rpm_tag)::value;
            if (do_read)
                read_frags(stage_n, stage_n, ks_n, afn, wfn);
#pragma unroll
            for (int q = 0; q < NMFMA; ++q)
                acc[q / TN][q % TN] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfc[q % TN], afc[q / TN], acc[q / TN][q % TN], 0, 0, 0);
            interleave_mfma_reads<NREAD, RPM>();
            __builtin_amdgcn_sched_barrier(0);
        };
        constexpr int RPM_N = (NREAD + NMFMA - 1) / NMFMA;      // reads spread over the whole slice
        using rpm1 = std::integral_constant<int, RPM_N>;
        using rpm2 = std::integral_constant<int, 2 * RPM_N>;    // reads packed into its first half
#pragma unroll
        for (int t = 0; t < NS; ++t)
            issue_range(t, t, t, c0{}, cLPT{});
        wait_vmcnt<(NS - 1) * LPT>();
        __syncthreads();
        read_frags(0, 0, 0, af0, wf0);
        __builtin_amdgcn_sched_barrier(0);
        int cur = 0;
        for (int kt = 0; kt + 1 < nk; ++kt) {
            const int nxt = (cur + 1 == NS) ? 0 : cur + 1;
            phase_b(af0, wf0, true, cur, 1, af1, wf1, rpm1{});
            phase_b(af1, wf1, true, cur, 2, af0, wf0, rpm1{});
            phase_b(af0, wf0, true, cur, 3, af1, wf1, rpm2{});   // reads early: complete at the barrier
            // tile kt+1 complete, NS-2 later tiles may be in flight -- and, in the NS-1 iterations after the
            // B_in prefetch went out behind tile pf_at+NS, those loads too (loads return in issue order)
            if (PF && pf_on && kt > pf_at && kt < pf_at + NS) {
                wait_vmcnt<(NS - 2) * LPT + PFR>();
            } else if (CARRY_A && kt == carry_at) {  // tile kt goes on to the landing buffer (stores not awaited here)
                carry_tile(kt, cur);
                wait_vmcnt<(NS - 2) * LPT + A_LD>();
            } else {
                wait_vmcnt<(NS - 2) * LPT>();
            }
            __syncthreads();                 // tile kt is read by all, tile kt+1 is published
            issue_range(kt + NS, cur, cur, c0{}, cLPT{});
            if constexpr (PF) {
                if (pf_on && kt == pf_at) {
                    wait_delivery(false);
                    if (cFlag != nullptr)
                        prefetch_recv(std::integral_constant<int, COHERENT_LD>{});
                    else
                        prefetch_recv(std::integral_constant<int, 0>{});
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            phase_b(af1, wf1, true, nxt, 0, af0, wf0, rpm1{});
            cur = nxt;
        }
        if (nk > 0) {
            phase_b(af0, wf0, true, cur, 1, af1, wf1, rpm1{});
            phase_b(af1, wf1, true, cur, 2, af0, wf0, rpm1{});
            phase_b(af0, wf0, true, cur, 3, af1, wf1, rpm1{});
            if (CARRY_A && nk - 1 == carry_at)
                carry_tile(nk - 1, cur);
            phase_b(af1, wf1, false, 0, 0, af0, wf0, rpm1{});
        }
    }
    wait_vmcnt<0>();                                 // no direct load may outlive its LDS allocation

    // Row and first column (of four) of accumulator registers 4g .. 4g+3 of this lane's 32x32 sub-tile (i, j).
    auto e_row = [&](int i, int g) __attribute__((always_inline)) {
        return MF16 ? m0 + wm * WTM + i * 32 + 16 * (g >> 1) + (lane & 15) : m0 + wm * WTM + i * 32 + (lane & 31);
    };
    auto e_col = [&](int j, int g) __attribute__((always_inline)) {
        return MF16 ? n0 + wn * WTN + j * 32 + 16 * (g & 1) + 4 * (lane >> 4) : n0 + wn * WTN + j * 32 + g * 8 + (lane >> 5) * 4;
    };

    // Split-K: every split parks its fp32 partial tile in the workspace; the split that finishes
    // last sums all partials in split order (so the result does not depend on which one that is),
    // then runs the epilogue.  No split ever waits for another.
    // The chip's eight XCDs have separate L2 caches.  Instead of writing back and invalidating whole
    // L2s around the hand-over, the partial tiles and the arrival counter are accessed with the
    // device-coherent cache policy (sc0 sc1: stores write through to memory, loads and the atomic
    // are served there), which keeps every other line of every L2 in place.
    if (splits > 1) {
        constexpr int COHERENT = 1 | 16;         // buffer cache-policy bits sc0 | sc1
        const size_t plane = (size_t)M * N;
        __amdgpu_buffer_rsrc_t ws_rsrc =
            __builtin_amdgcn_make_buffer_rsrc(P.ws + (size_t)split * plane, 0, (int)(plane * 4), 0x00020000);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int m = e_row(i, g), n = e_col(j, g);
                    const int boff = (m < M && n < N) ? (int)(((unsigned)m * (unsigned)N + n) * 4u) : (int)OOB;
                    const f32x4_t o = acc_get(i, j, g);
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, o), ws_rsrc, boff, 0, COHERENT);
                }
        }
        __builtin_amdgcn_s_waitcnt(0);           // this wave's partial stores are acknowledged
        __syncthreads();                         // ... and every wave's
        unsigned *arrived = reinterpret_cast<unsigned *>(smem);   // the stages are no longer read by anyone
        if (tid == 0)
            *arrived = __hip_atomic_fetch_add(&P.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*arrived != (unsigned)(splits - 1))
            return;                              // not the last to finish: done
        if (tid == 0)                            // leave the counter ready for the next launch
            __hip_atomic_store(&P.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int m = e_row(i, g), n = e_col(j, g);
                    const int boff = (m < M && n < N) ? (int)(((unsigned)m * (unsigned)N + n) * 4u) : (int)OOB;
                    f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
                    for (int sp = 0; sp < splits; ++sp) {
                        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                            P.ws + (size_t)sp * plane, 0, (int)(plane * 4), 0x00020000);
                        const f32x4_t v =
                            __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs, boff, 0, COHERENT));
                        sum = sp == 0 ? v : sum + v;
                    }
                    acc_set(i, j, g, sum);
                }
        }
    }

    // Epilogue.  Accumulator register 4g+e of lane L holds row (L & 31), column 8g + 4(L >> 5) + e
    // of its 32x32 tile.  Bounds-checked buffer accesses: a lane outside the matrix reads zero
    // and its store is dropped.
    if (!(RLDS && streamed))
        __syncthreads();                             // the stores' scratch lies in a stage: all waves are done with them
    constexpr unsigned o_elem = OUT_BF16 ? 2 : 4;
    const unsigned o_bytes = (unsigned)(((int64_t)(M - 1) * P.ldo + N) * o_elem);
    __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(cOut, 0, (int)o_bytes, 0x00020000);
    const bool has_recv = cRecv != nullptr;
    if (!P.wait_at_start && !pf_on)
        wait_delivery(false);                        // B_in has travelled under the main loop
    if (wait_tiles) {
        // The workgroups that landed this tile's arrivals wrote them through to memory and counted up afterwards;
        // they hold earlier work items, so they are running or done.  One lane polls, at most spin_limit times.
        if (tid == 0) {
            unsigned n = 0;
            while (__hip_atomic_load(&P.tile_ready[tile], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) < (unsigned)P.ready_count) {
                if (++n >= P.spin_limit) {
                    __hip_atomic_fetch_or(P.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    break;
                }
                __builtin_amdgcn_s_sleep(32);
            }
            // (this item is the tile's only reader: the counter is left ready for the next launch)
            __hip_atomic_store(&P.tile_ready[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        // the arrivals were written through another XCD's L2: drop what this one may hold of those lines, once per
        // workgroup, so that the epilogue's loads can go through the caches (they read a line in several pieces)
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    const bool recv_coherent = cFlag != nullptr && !P.wait_at_start;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        unsigned eoff[TN][4];
        f32x4_t rv[TN][4];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = e_row(i, g), n = e_col(j, g);
                eoff[j][g] = (m < M && n < N) ? (unsigned)((int64_t)m * P.ldo + n) : OOB;
            }
        if (PF && pf_on) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    rv[j][g] = pre[PF ? i : 0][PF ? j : 0][g];
        } else if (has_recv && !streamed) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int boff = eoff[j][g] == OOB ? (int)OOB : (int)(eoff[j][g] * 4);
                    rv[j][g] = __builtin_bit_cast(f32x4_t, recv_coherent
                                   ? __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, boff, 0, COHERENT_LD)
                                   : __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, boff, 0, 0));
                    if constexpr (PERSIST && RLDS) {
                        if (cLand != nullptr) {      // (a work item that could not stream still delivers)
                            __amdgpu_buffer_rsrc_t le_rsrc =
                                __builtin_amdgcn_make_buffer_rsrc(static_cast<float *>(cLand), 0, (int)r_bytes, 0x00020000);
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, rv[j][g]), le_rsrc, boff, 0, 0);
                        }
                    }
                }
            // further received partials, summed in index order: one batch of independent loads per buffer
            for (int b = 0; b < n_more; ++b) {
                __amdgpu_buffer_rsrc_t m_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<float *>(P.recv_more[b]), 0, (int)r_bytes, 0x00020000);
                f32x4_t tv[TN][4];
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        tv[j][g] = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                            m_rsrc, eoff[j][g] == OOB ? (int)OOB : (int)(eoff[j][g] * 4), 0, 0));
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        rv[j][g] = rv[j][g] + tv[j][g];
            }
        }
        // The stores go through a wave-private LDS scratch so that they leave as whole 128-byte lines: the
        // accumulator layout would store 32-byte (bf16: 16-byte) pieces of thirty-two rows per instruction, which
        // the memory system handles markedly worse (measured: 70B down-projection rank step 438 -> 418 us).
        unsigned char *const scr = smem + land_stage * A_BYTES + wave * E_SCR_BYTES;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4_t o = acc_get(i, j, g);
                if (has_recv && !streamed)
                    o = rv[j][g] + o;                                    // "O <- B_in + O"
                if constexpr (OUT_BF16) {
                    // row (lane & 31) of the wave tile's row block i: 64-column rows of bf16 (128 bytes), their
                    // eight 16-byte chunks XOR-ed with the row so that the rows spread over the banks
                    bf16x4_t h;
                    h[0] = static_cast<__bf16>(o[0]);
                    h[1] = static_cast<__bf16>(o[1]);
                    h[2] = static_cast<__bf16>(o[2]);
                    h[3] = static_cast<__bf16>(o[3]);
                    if constexpr (MF16) {
                        // row 16 (g / 2) + (lane & 15), columns 32 j + 16 (g & 1) + 4 (lane >> 4) .. + 3 of the row block
                        const int r = 16 * (g >> 1) + (lane & 15);
                        const int ch = j * 4 + 2 * (g & 1) + (lane >> 5);
                        *reinterpret_cast<bf16x4_t *>(scr + r * 128 + ((ch ^ (r & 7)) << 4) + ((lane >> 4) & 1) * 8) = h;
                    } else
                    *reinterpret_cast<bf16x4_t *>(scr + (lane & 31) * 128 + (((j * 4 + g) ^ (lane & 7)) << 4) + (lane >> 5) * 8) = h;
                } else {
                    // plane g of the 32x32 sub-tile (i, j), the rows permuted within the plane (row ^ chunk number:
                    // the chunks of a row lie 512 bytes apart and would all fall into one bank otherwise)
                    if constexpr (MF16) {
                        // chunk c = 4 (g & 1) + (lane >> 4) of row r = 16 (g / 2) + (lane & 15): plane c / 2, slot (r ^ c) + 32 (c & 1)
                        const int r = 16 * (g >> 1) + (lane & 15), c = 4 * (g & 1) + (lane >> 4);
                        *reinterpret_cast<f32x4_t *>(scr + (c >> 1) * 1024 + ((32 * (c & 1) + (r ^ c)) << 4)) = o;
                    } else
                    *reinterpret_cast<f32x4_t *>(scr + g * 1024 + (((lane & 32) | ((lane & 31) ^ (2 * g + (lane >> 5)))) << 4)) = o;
                }
            }
            if constexpr (!OUT_BF16) {
                // read back eight lanes to a row: chunk c of row r lies in plane c / 2 at lane slot (r ^ c) + 32 (c & 1)
                const int c = lane & 7, r8 = lane >> 3;
                const unsigned char *base = scr + (c >> 1) * 1024 + (32 * (c & 1)) * 16;
                const int sn = n0 + wn * WTN + j * 32 + c * 4;
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    const int row = 8 * s4 + r8;
                    const f32x4_t t = *reinterpret_cast<const f32x4_t *>(base + ((row ^ c) << 4));
                    const int sm = m0 + wm * WTM + i * 32 + row;
                    const int so = (sm < M && sn < N) ? (int)(((int64_t)sm * P.ldo + sn) * 4) : (int)OOB;
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, t), o_rsrc, so, 0, 0);
                }
            }
        }
        if constexpr (OUT_BF16) {
            static_assert(!OUT_BF16 || TN == 2, "a wave tile row of 64 bf16 columns is one 128-byte line");
            const int c = lane & 7, r8 = lane >> 3;                  // eight 16-byte chunks (8 columns each) per row
            const int sn = n0 + wn * WTN + c * 8;
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const int row = 8 * s4 + r8;
                const u32x4_t t = *reinterpret_cast<const u32x4_t *>(scr + row * 128 + ((c ^ (row & 7)) << 4));
                const int sm = m0 + wm * WTM + i * 32 + row;
                const int so = (sm < M && sn < N) ? (int)(((int64_t)sm * P.ldo + sn) * 2) : (int)OOB;
                __builtin_amdgcn_raw_buffer_store_b128(t, o_rsrc, so, 0, 0);
            }
        }
    }
    if constexpr (PERSIST) {
        if (TAILS && !tail_early) {
            if (tl_on && tl_c > 0 && tl_c <= TL_N)   // the instruction in flight when the main loop ended
                __builtin_amdgcn_raw_buffer_store_b128(tl_v, tl_drsrc, tl_voff, (tl_c - 1) * tl_stride, COHERENT_LD);
            land_arrival(tl_on ? (tl_c < TL_N ? tl_c : TL_N) : 0);
        }
        __syncthreads();                             // every wave is done with the LDS stages
    }
    item += item_stride;
    } while (PERSIST && item < n_items);             // next work item
}

template <int BM, int BN, int WGM, int WGN, int NS, bool SPREAD>
hipError_t launch_cfg(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s)
{
    // reduce-scatter steps on the 256x256 tile: the variant that brings B_in in under the main loop
    bool any_recv = p.n_steps == 0 && p.recv != nullptr;     // (a persistent launch ignores recv and wait_flag)
    for (int j = 0; j < p.n_steps; ++j)
        any_recv = any_recv || p.recv_step[j] != nullptr;
    // (only where the kernel would stream: a long enough k range, one received partial per step, no delivery flag, no
    // k-split -- otherwise the variant with three left-operand stages is the faster one)
    bool any_flag = p.n_steps == 0 && p.wait_flag != nullptr;
    for (int j = 0; j < p.n_steps; ++j)
        any_flag = any_flag || p.flag_step[j] != nullptr;
    const int nk_all = (p.K + BK - 1) / BK;
    bool any_tail = false;                           // a step lands an arrival beside its GEMM (GemmParams::tail_src)
    for (int j = 0; j < p.n_steps; ++j)
        any_tail = any_tail || p.tail_src[j] != nullptr;
    [[maybe_unused]] const bool rlds = SPREAD && NS == 2 && any_recv && !out_bf16 && !p.a_t && p.stream_recv && !any_flag &&
                                       p.n_recv_more == 0 && p.splits == 1 && nk_all >= 18 + (p.K % BK != 0 ? 2 : 0) &&
                                       p.tile_ready == nullptr && !any_tail;
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    int wgs = tiles_m * tiles_n * p.splits + p.cp_wgs;
    if (p.n_steps > 0) {                             // persistent: a grid that fills the chip once
        constexpr int per_cu = (NS * (BM + BN) * 64 * 2 <= 80 * 1024) ? 2 : 1;
        const int items = tiles_m * tiles_n * p.n_steps;
        wgs = items < p.num_cu * per_cu ? items : p.num_cu * per_cu;
        if (p.xcd_steps)                             // whole octets of workgroups: the same number per XCD
            wgs = (tiles_m * tiles_n * p.n_steps / 8 < p.num_cu * per_cu / 8 ? tiles_m * tiles_n * p.n_steps / 8
                                                                            : p.num_cu * per_cu / 8) * 8;
        if (const int cap = tuning().persist_wgs; cap >= 8 && cap < wgs)   // override: leave compute units free
            wgs = p.xcd_steps ? cap / 8 * 8 : cap;
    }
    const dim3 grid(wgs), block(64 * WGM * WGN);
    if (p.n_steps > 0) {                             // persistent rank step: fp32 or bf16 output, either weight order
        if (p.a_t)
            return hipErrorInvalidValue;
        // (256x256 tile: the main loop on 16x16x32 MFMAs where the launcher asks for it, GemmParams::mfma16)
#define CF_LAUNCH_PERSIST(WKN, OBF, RL)                                                                                         \
    do {                                                                                                                        \
        if constexpr (SPREAD && NS == 2) {                                                                                      \
            if (p.mfma16 && !(RL))                                                                                              \
                hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, WKN, OBF, false, true, false, true>),    \
                                   grid, block, 0, s, p, tiles_m, tiles_n);                                                     \
            else                                                                                                                \
                hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, WKN, OBF, false, true, RL>), grid, block, \
                                   0, s, p, tiles_m, tiles_n);                                                                  \
        } else {                                                                                                                \
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, WKN, OBF, false, true, false>), grid, block,  \
                               0, s, p, tiles_m, tiles_n);                                                                      \
        }                                                                                                                       \
    } while (0)
        if (w_kn) {
            if (out_bf16)
                CF_LAUNCH_PERSIST(true, true, false);
            else if (SPREAD && NS == 2 && rlds)
                CF_LAUNCH_PERSIST(true, false, true);
            else
                CF_LAUNCH_PERSIST(true, false, false);
        } else {
            if (out_bf16)
                CF_LAUNCH_PERSIST(false, true, false);
            else if (SPREAD && NS == 2 && rlds)
                CF_LAUNCH_PERSIST(false, false, true);
            else
                CF_LAUNCH_PERSIST(false, false, false);
        }
#undef CF_LAUNCH_PERSIST
        return hipGetLastError();
    }
    if (p.a_t) {
        if (!w_kn || out_bf16)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, true, false, true>), grid, block, 0, s, p, tiles_m, tiles_n);
    } else if (w_kn) {
        if (out_bf16)
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, true, true>), grid, block, 0, s, p, tiles_m, tiles_n);
        else if constexpr (SPREAD && NS == 2) {
            if (rlds)
                hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, true, false, false, false, true>), grid, block, 0, s, p, tiles_m, tiles_n);
            else
                hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, true, false>), grid, block, 0, s, p, tiles_m, tiles_n);
        } else
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, true, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    } else {
        if (out_bf16)
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, false, true>), grid, block, 0, s, p, tiles_m, tiles_n);
        else if constexpr (SPREAD && NS == 2) {
            if (rlds)
                hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, false, false, false, false, true>), grid, block, 0, s, p, tiles_m, tiles_n);
            else
                hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, false, false>), grid, block, 0, s, p, tiles_m, tiles_n);
        } else
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, NS, SPREAD, false, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace

bool gemm_bf16_dl_supported(const GemmParams &p, bool w_kn)
{
    // byte extents of operands and outputs must stay below 2^31 (32-bit buffer offsets, OOB marker above them)
    const int64_t lim = (int64_t)1 << 31;
    const int64_t a_bytes = ((int64_t)(p.a_t ? p.K : p.M) * p.lda) * 2;
    const int64_t w_bytes = ((int64_t)(w_kn ? p.K : p.N) * p.ldw) * 2;
    const int64_t o_bytes = ((int64_t)p.M * p.ldo) * 4;
    return p.M > 0 && p.N > 0 && p.K > 0 && a_bytes < lim && w_bytes < lim && o_bytes < lim;
}

// Would launch_gemm_bf16_dl take the kernel variant that streams B_in through LDS (and so can carry the delivery)
// for this persistent launch with tile t?  Mirrors the choice in launch_cfg.
bool gemm_bf16_dl_streams_recv(const GemmParams &p, bool w_kn, bool out_bf16, TileChoice t)
{
    (void)w_kn;
    const int nk_all = (p.K + BK - 1) / BK;
    return p.n_steps > 0 && t.bm == 256 && t.bn == 256 && !out_bf16 && !p.a_t && tuning().stream_recv != 0 &&
           p.n_recv_more == 0 && nk_all >= 18 + (p.K % BK != 0 ? 2 : 0);
}

// Can a persistent all-gather launch carry its deliveries (GemmParams::land_step with steps that add nothing)?  Every
// tile shape can; the k-tiles must be whole (a ragged one would be stored beyond the end of its rows).
bool gemm_bf16_dl_carries_operand(const GemmParams &p)
{
    return p.n_steps > 0 && !p.a_t && p.K % BK == 0;
}

hipError_t launch_gemm_bf16_dl(const GemmParams &p_in, bool w_kn, bool out_bf16, hipStream_t s, TileChoice t)
{
    GemmParams p = p_in;
    const Tuning tn = tuning();
    if (tn.prefetch >= 0)                              // override: lead of the B_in prefetch in k-tiles, 0 = off
        p.pf_lead = tn.prefetch;
    p.stream_recv = tn.stream_recv != 0;               // override: 0 = B_in is loaded in the epilogue (256x256 tile)
    p.splits = t.splitk < 1 ? 1 : t.splitk;
    const int nk_all = (p.K + BK - 1) / BK;
    if (p.splits > nk_all)
        p.splits = nk_all;
    const int64_t tiles = (int64_t)((p.M + t.bm - 1) / t.bm) * ((p.N + t.bn - 1) / t.bn);
    if (p.n_steps > 0) {
        for (int j = 0; j < p.n_steps; ++j)
            if (p.land_step[j] != nullptr && p.recv_step[j] == nullptr && !gemm_bf16_dl_carries_operand(p))
                return hipErrorInvalidValue;          // callers ask gemm_bf16_carries_delivery first
        if (p.tile_ready != nullptr && (out_bf16 || tiles > p.max_tiles || p.status == nullptr || p.spin_limit == 0))
            return hipErrorInvalidValue;              // callers ask gemm_bf16_tiles_landing_arrivals first
        for (int j = 0; j < p.n_steps; ++j)
            if ((p.tail_src[j] != nullptr) != (p.tail_dst[j] != nullptr) || (p.tail_src[j] != nullptr && out_bf16))
                return hipErrorInvalidValue;
        p.splits = 1;
        p.cp_wgs = 0;
        p.cp_bytes = 0;
        // overrides: xcd_steps 0 = every XCD takes a band of every step; k_rotate 0 = every XCD walks k from 0
        // (whole steps per XCD not when one step carries the sum of several received partials: that step's
        // epilogue is heavy and would fall on one XCD)
        // (... or, with fewer steps than XCDs -- a group of steps launched on its own --, 8 / NB step groups x NB bands
        // of tile columns, which needs NB to divide the tile columns and 8 / NB the steps)
        const int tiles_n_ = (p.N + t.bn - 1) / t.bn;
        bool cut = false;
        for (int nb = 1; nb <= 8; nb *= 2)
            cut = cut || (tiles_n_ % nb == 0 && p.n_steps % (8 / nb) == 0);
        // (... nor when work items hand arrivals on to the last step's: step-major order keeps the producers in front)
        p.xcd_steps = cut && p.num_cu % 8 == 0 && p.n_recv_more == 0 && p.tile_ready == nullptr && tn.xcd_steps != 0;
        // Step groups x column bands: per k-tile the 32 (or fewer) workgroups of an XCD that run side by side fetch
        // `a` left-operand bands of bm rows and `b` weight bands of bn columns, a = (step, tile row) pairs of the XCD
        // (at most its workgroups), b = the columns they spread over; the number of bands NB that makes a bm + b bn
        // smallest (ties: the fewest bands).  7B down-projection (2 tile rows x 16 tile columns per step): NB = 2,
        // 12 instead of 18 bands; the 70B shapes stay at NB = 1 (4 x 8 is already the best cut of 32).
        p.xcd_bands = 1;
        if (p.xcd_steps) {
            const int tiles_m = (p.M + t.bm - 1) / t.bm, tiles_n = (p.N + t.bn - 1) / t.bn;
            const int per_cu = (t.bm == 128 && t.bn == 128 && !t.deep) ? 2 : 1;
            const int items_x = tiles_m * tiles_n * p.n_steps / 8;
            const int wgs_x = items_x < p.num_cu * per_cu / 8 ? items_x : p.num_cu * per_cu / 8;
            long best = -1;
            for (int nb = 1; nb <= 8; nb *= 2) {
                if (tiles_n % nb != 0 || p.n_steps % (8 / nb) != 0)
                    continue;
                if (tn.xcd_bands > 0 && nb != tn.xcd_bands && p.n_steps % 8 == 0)
                    continue;                          // override: this many bands where the shape allows it
                const int rows = p.n_steps / (8 / nb) * tiles_m;
                const int a = rows < wgs_x ? rows : wgs_x;
                const int cols = tiles_n / nb;
                int b = (wgs_x + a - 1) / a;
                b = b < cols ? b : cols;
                const long cost = (long)a * t.bm + (long)b * t.bn;
                if (best < 0 || cost < best) {
                    best = cost;
                    p.xcd_bands = nb;
                }
            }
            if (best < 0 && p.n_steps % 8 != 0)
                p.xcd_steps = false;                   // (no cut fits: every XCD takes a band of every step)
        }
        // (measured with whole steps per XCD only; a ragged k tail stays the last k-tile of every work item,
        // which keeps all earlier iterations of the 256x256 main loop branch-free)
        p.k_rotate = p.xcd_steps && tn.k_rotate != 0 && p.K % BK == 0;
        // the 256x256 tile's main loop on 16x16x32 MFMAs (override: COMMFUSE_MFMA16 = 0 | 1)
        p.mfma16 = t.bm == 256 && t.bn == 256 && p.M % 256 == 0 && p.N % 256 == 0 && tn.mfma16 != 0;
    }
    if (p.splits > 1 && (p.ws == nullptr || p.counters == nullptr ||
                         (size_t)p.splits * p.M * p.N * sizeof(float) > p.ws_bytes || tiles > p.max_tiles ||
                         (int64_t)p.M * p.N * 4 >= ((int64_t)1 << 31)))
        p.splits = 1;                          // no (or too small a) workspace: plain kernel
    if (p.cp_src == nullptr || p.cp_dst == nullptr || p.cp_bytes == 0)
        p.cp_wgs = 0;
    // LDS stages: as many as fit (160 KiB per CU); the 128x128 tile comes with two stages (two
    // workgroups share a CU) or four (one workgroup per CU, tiles requested three ahead).
    if (t.bm == 256 && t.bn == 256) return launch_cfg<256, 256, 2, 4, 2, true>(p, w_kn, out_bf16, s);
    if (t.bm == 256 && t.bn == 128) return launch_cfg<256, 128, 4, 2, 3, false>(p, w_kn, out_bf16, s);
    if (t.deep) return launch_cfg<128, 128, 2, 2, 4, false>(p, w_kn, out_bf16, s);
    return launch_cfg<128, 128, 2, 2, 2, false>(p, w_kn, out_bf16, s);
}

}  // namespace cf

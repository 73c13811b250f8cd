// bf16 x bf16 -> fp32 chunk GEMM for gfx950, direct-to-LDS variant.
//
//  * Operand tiles go from global memory straight into LDS (buffer_load ... lds,
//    16 bytes per lane) without passing through registers.
//  * A [k x n] weight tile stays in its natural order in LDS and is read back
//    with the transposing LDS read (ds_read_b64_tr_b16); a [n x k] weight tile
//    and the activations are read with plain 16-byte reads.
//  * k-tiles of 64 (full 128-byte lines of the k-contiguous operands) in two LDS
//    stages.  A k-tile is consumed in four 16-wide slices; fragments are
//    double-buffered in registers and the LDS reads of slice s+1 are interleaved
//    with the MFMAs of slice s.  The one barrier per k-tile sits before the last
//    slice: by then every wave has read all of the tile, so the other stage's
//    successor can be requested, and the next tile (requested one barrier
//    earlier) is published; its first fragments are fetched under the MFMAs of
//    the last slice, so the matrix pipe does not drain at tile boundaries.
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
constexpr int NS = 2;                     // LDS stages
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

template <int BM, int BN, int WGM, int WGN, bool W_KN, bool OUT_BF16>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_dl_kernel(GemmParams P, int tiles_m, int tiles_n)
{
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = (A_BYTES / 1024) / NW;     // 1 KiB wave-loads of the A tile per wave
    constexpr int B_LD = (B_BYTES / 1024) / NW;
    constexpr int LPT = A_LD + B_LD;                // direct loads per wave per k-tile
    static_assert(A_LD >= 1 && B_LD >= 1 && (A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "tile vs waves");
    static_assert(NS * STAGE <= 160 * 1024, "LDS budget");
    static_assert(KS == 4, "the slice schedule below is written for four slices per stage");
    constexpr int W_ROWB = BN * 2;                   // bytes of one k-row of a [k x n] weight tile

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NS * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;

    const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int m0 = (tile % tiles_m) * BM;
    const int n0 = (tile / tiles_m) * BN;
    const int M = P.M, N = P.N, K = P.K;

    // Buffer resources; all byte extents are below 2^31 (host-checked).
    const unsigned a_bytes = (unsigned)(((int64_t)(M - 1) * P.lda + K) * 2);
    const unsigned w_bytes = (unsigned)((W_KN ? ((int64_t)(K - 1) * P.ldw + N) : ((int64_t)(N - 1) * P.ldw + K)) * 2);
    const i32x4_t a_rsrc = make_rsrc(P.A, a_bytes);
    const i32x4_t w_rsrc = make_rsrc(P.W, w_bytes);
    const unsigned lds_base = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem);

    // Per-lane global byte offsets (k0 = 0) of every wave-load, and the k index of its chunk for the tail test.
    unsigned a_off[A_LD], b_off[B_LD];
    int a_k[A_LD], b_k[B_LD];
#pragma unroll
    for (int j = 0; j < A_LD; ++j) {
        const int pos = (j * NW + wave) * 1024 + lane * 16;
        int row, kc;
        unswz_row(pos, row, kc);
        const int gm = m0 + row;
        a_k[j] = kc * 8;
        a_off[j] = gm < M ? (unsigned)(((int64_t)gm * P.lda + kc * 8) * 2) : OOB;
    }
#pragma unroll
    for (int j = 0; j < B_LD; ++j) {
        const int pos = (j * NW + wave) * 1024 + lane * 16;
        if constexpr (W_KN) {
            const int k = pos / W_ROWB, inrow = pos % W_ROWB;
            const int q = (inrow >> 6) ^ (k & 3);
            const int gn = n0 + q * 32 + ((inrow >> 4) & 3) * 8;
            b_k[j] = k;
            b_off[j] = gn < N ? (unsigned)(((int64_t)k * P.ldw + gn) * 2) : OOB;
        } else {
            int row, kc;
            unswz_row(pos, row, kc);
            const int gn = n0 + row;
            b_k[j] = kc * 8;
            b_off[j] = gn < N ? (unsigned)(((int64_t)gn * P.ldw + kc * 8) * 2) : OOB;
        }
    }
    const int w_kstep = W_KN ? (int)(P.ldw * 2) : 2;   // bytes per unit of k along W

    auto issue_loads = [&](int kt) {
        const int k0 = kt * BK;
        const unsigned sa = lds_base + (kt & 1) * STAGE + wave * 1024;
        const bool tail = (k0 + BK) > K;
#pragma unroll
        for (int j = 0; j < A_LD; ++j) {
            unsigned off = a_off[j];
            if (tail && (k0 + a_k[j]) >= K)
                off = OOB;
            direct_load_16(a_rsrc, off, k0 * 2, sa + j * NW * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_LD; ++j) {
            unsigned off = b_off[j];
            if (tail && (k0 + b_k[j]) >= K)
                off = OOB;
            direct_load_16(w_rsrc, off, k0 * w_kstep, sa + A_BYTES + j * NW * 1024);
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[i][j][e] = 0.0f;

    // Fragment addressing (byte offsets inside a stage), fixed for the whole loop.  The swizzle
    // uses row bits 0..3 only, so the 32-row MFMA tiles of a wave differ by constants, and the
    // 16-wide k-slice ks is reached by XOR-ing (ks << 5) into the offset of slice 0.
    const int frow = lane & 31, fkc = lane >> 5;
    const int a_addr = swz_row(wm * WTM + frow, fkc);
    int w_addr[W_KN ? TN : 1];
    if constexpr (W_KN) {
        const int blk = lane >> 4, i16 = lane & 15;
        const int kl = (blk >> 1) * 8 + (i16 >> 2);                      // k of (ks = 0, h = 0)
        const int nl = wn * WTN + (blk & 1) * 16 + (i16 & 3) * 4;        // column of tile j = 0
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int q = ((nl >> 5) + j) ^ (kl & 3);
            w_addr[j] = A_BYTES + kl * W_ROWB + (q << 6) + (nl & 31) * 2;
        }
    } else {
        w_addr[0] = A_BYTES + swz_row(wn * WTN + frow, fkc);
    }

    auto read_frags = [&](int kt, int ks, bf16x8_t (&af)[TM], bf16x8_t (&wf)[TN]) {
        const unsigned char *st = smem + (kt & 1) * STAGE;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[i] = *reinterpret_cast<const bf16x8_t *>(st + (a_addr ^ (ks << 5)) + i * 32 * 128);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (W_KN) {
                const unsigned char *pw = st + w_addr[j] + ks * 16 * W_ROWB;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pw));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pw + 4 * W_ROWB));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                wf[j] = __builtin_bit_cast(bf16x8_t, both);
            } else {
                wf[j] = *reinterpret_cast<const bf16x8_t *>(st + (w_addr[0] ^ (ks << 5)) + j * 32 * 128);
            }
        }
    };
    auto mfma_block = [&](const bf16x8_t (&af)[TM], const bf16x8_t (&wf)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
    };

    // One slice phase: the MFMAs of the fragments in (afc, wfc) with the LDS reads of the next
    // slice's fragments (into afn, wfn) interleaved, RPM reads after each of the first MFMAs.
    constexpr int NREAD = TM + (W_KN ? 2 * TN : TN);
    constexpr int NMFMA = TM * TN;
    auto mfma_only = [&](const bf16x8_t (&afc)[TM], const bf16x8_t (&wfc)[TN]) {
        mfma_block(afc, wfc);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto phase = [&](const bf16x8_t (&afc)[TM], const bf16x8_t (&wfc)[TN], int kt_n, int ks_n, bf16x8_t (&afn)[TM],
                     bf16x8_t (&wfn)[TN], auto rpm_tag) {
        constexpr int RPM = decltype(rpm_tag)::value;
        read_frags(kt_n, ks_n, afn, wfn);
        mfma_block(afc, wfc);
        interleave_mfma_reads<NREAD, RPM>();
        __builtin_amdgcn_sched_barrier(0);
    };
    constexpr int RPM_N = (NREAD + NMFMA - 1) / NMFMA;      // reads spread over the whole phase
    using rpm1 = std::integral_constant<int, RPM_N>;
    using rpm2 = std::integral_constant<int, 2 * RPM_N>;    // reads packed into its first half

    const int nk = (K + BK - 1) / BK;
    bf16x8_t af0[TM], wf0[TN], af1[TM], wf1[TN];

    // Prologue: tile 0 in stage 0, its first fragments in registers, tile 1 requested.
    if (nk > 0)
        issue_loads(0);
    wait_vmcnt<0>();
    __syncthreads();
    if (nk > 0)
        read_frags(0, 0, af0, wf0);
    if (nk > 1)
        issue_loads(1);
    __builtin_amdgcn_sched_barrier(0);

    for (int kt = 0; kt + 1 < nk; ++kt) {
        phase(af0, wf0, kt, 1, af1, wf1, rpm1{});
        phase(af1, wf1, kt, 2, af0, wf0, rpm1{});
        phase(af0, wf0, kt, 3, af1, wf1, rpm2{});   // reads early: they must be complete at the barrier
        wait_vmcnt<0>();             // this wave's part of tile kt+1 has landed
        __syncthreads();             // every wave has read all of tile kt; tile kt+1 is published
        if (kt + 2 < nk)
            issue_loads(kt + 2);     // into the stage tile kt just vacated
        __builtin_amdgcn_sched_barrier(0);
        phase(af1, wf1, kt + 1, 0, af0, wf0, rpm1{});
    }
    if (nk > 0) {                    // last tile: nothing follows it
        phase(af0, wf0, nk - 1, 1, af1, wf1, rpm1{});
        phase(af1, wf1, nk - 1, 2, af0, wf0, rpm1{});
        phase(af0, wf0, nk - 1, 3, af1, wf1, rpm1{});
        mfma_only(af1, wf1);
    }

    // Epilogue.  Accumulator register 4g+e of lane L holds row (L & 31), column 8g + 4(L >> 5) + e
    // of its 32x32 tile.  Bounds-checked buffer accesses: a lane outside the matrix reads zero
    // and its store is dropped.
    constexpr unsigned o_elem = OUT_BF16 ? 2 : 4;
    const unsigned o_bytes = (unsigned)(((int64_t)(M - 1) * P.ldo + N) * o_elem);
    __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(P.out, 0, (int)o_bytes, 0x00020000);
    const unsigned r_bytes = (unsigned)(((int64_t)(M - 1) * P.ldo + N) * 4);
    const bool has_recv = P.recv != nullptr;
    __amdgpu_buffer_rsrc_t r_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.recv), 0, has_recv ? (int)r_bytes : 0, 0x00020000);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * WTM + i * 32 + (lane & 31);
        unsigned eoff[TN][4];
        u32x4_t rv[TN][4];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * WTN + j * 32 + g * 8 + (lane >> 5) * 4;
                eoff[j][g] = (m < M && n < N) ? (unsigned)((int64_t)m * P.ldo + n) : OOB;
            }
        if (has_recv) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    rv[j][g] = __builtin_amdgcn_raw_buffer_load_b128(
                        r_rsrc, eoff[j][g] == OOB ? (int)OOB : (int)(eoff[j][g] * 4), 0, 0);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4_t o;
                o[0] = acc[i][j][4 * g + 0];
                o[1] = acc[i][j][4 * g + 1];
                o[2] = acc[i][j][4 * g + 2];
                o[3] = acc[i][j][4 * g + 3];
                if (has_recv)
                    o = __builtin_bit_cast(f32x4_t, rv[j][g]) + o;       // "O <- B_in + O"
                const int boff = eoff[j][g] == OOB ? (int)OOB : (int)(eoff[j][g] * o_elem);
                if constexpr (OUT_BF16) {
                    bf16x4_t h;
                    h[0] = static_cast<__bf16>(o[0]);
                    h[1] = static_cast<__bf16>(o[1]);
                    h[2] = static_cast<__bf16>(o[2]);
                    h[3] = static_cast<__bf16>(o[3]);
                    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, h), o_rsrc, boff, 0, 0);
                } else {
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, o), o_rsrc, boff, 0, 0);
                }
            }
    }
}

template <int BM, int BN, int WGM, int WGN>
hipError_t launch_cfg(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s)
{
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const dim3 grid(tiles_m * tiles_n), block(64 * WGM * WGN);
    if (w_kn) {
        if (out_bf16)
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, true, true>), grid, block, 0, s, p, tiles_m, tiles_n);
        else
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, true, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    } else {
        if (out_bf16)
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, false, true>), grid, block, 0, s, p, tiles_m, tiles_n);
        else
            hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, false, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace

bool gemm_bf16_dl_supported(const GemmParams &p, bool w_kn)
{
    // byte extents of operands and outputs must stay below 2^31 (32-bit buffer offsets, OOB marker above them)
    const int64_t lim = (int64_t)1 << 31;
    const int64_t a_bytes = ((int64_t)p.M * p.lda) * 2;
    const int64_t w_bytes = ((int64_t)(w_kn ? p.K : p.N) * p.ldw) * 2;
    const int64_t o_bytes = ((int64_t)p.M * p.ldo) * 4;
    return p.M > 0 && p.N > 0 && p.K > 0 && a_bytes < lim && w_bytes < lim && o_bytes < lim;
}

hipError_t launch_gemm_bf16_dl(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s, TileChoice t)
{
    if (t.bm == 256 && t.bn == 256) return launch_cfg<256, 256, 2, 4>(p, w_kn, out_bf16, s);
    if (t.bm == 256 && t.bn == 128) return launch_cfg<256, 128, 4, 2>(p, w_kn, out_bf16, s);
    return launch_cfg<128, 128, 2, 2>(p, w_kn, out_bf16, s);
}

}  // namespace cf

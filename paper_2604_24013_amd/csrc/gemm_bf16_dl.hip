// bf16 x bf16 -> fp32 chunk GEMM for gfx950, direct-to-LDS variant: the operand
// tiles go from global memory straight into LDS (buffer_load ... lds, 16 bytes
// per lane) without passing through registers, and a [k x n] weight tile is
// read back with the transposing LDS read (ds_read_b64_tr_b16), so no register
// transposition is needed either.  Same fused epilogue as the register-staged
// kernel: Alg. 2 "O <- B_in + O", "B_out <- O", or Alg. 1's in-place slice store.
//
// Layout in LDS (per stage, two stages):
//   activations / [n x k] weights: 128-byte rows (64 k), eight 16-byte chunks per
//     row, XOR-swizzled so that 16-byte fragment reads are bank-conflict free.
//     A wave-wide direct load fills 1 KiB of contiguous LDS (8 rows); the
//     swizzle is applied by choosing which global chunk each lane fetches.
//   [k x n] weights: natural order, one k-row of BN bf16 after the other; the
//     64-byte groups of a row are XOR-ed with (k & 3) so that the four rows a
//     transposing read touches fall into different banks.
// Out-of-range rows, columns and the k tail are zero-filled by the buffer
// bounds check (a lane that must read zero gets an offset beyond num_records).
#include "cf_internal.h"

#include <cstdio>
#include <cstdlib>

namespace cf {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

constexpr int BK = 64;
constexpr unsigned OOB = 0x80000000u;     // byte offset beyond any buffer this kernel accepts

// Byte offset of 16-byte chunk kc (0..7) of tile row `row`.  Only row bits 0..3 enter
// the swizzle, so rows 32 apart differ by a constant 4096 bytes.
__device__ __forceinline__ int swz_row(int row, int kc)
{
    const int r0 = row & 1, r1 = (row >> 1) & 1, r2 = (row >> 2) & 1, r3 = (row >> 3) & 1;
    const int half = r0 ^ r3;
    const int kcp = kc ^ ((r1 << 2) | (r2 << 1) | r3);
    return ((row >> 1) << 8) + (half << 7) + (kcp << 4);
}

// Inverse of swz_row for the lane that fills bytes [pos, pos+16) of a tile.
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
// assembly so that the compiler does not order later LDS reads of the OTHER
// stage behind it; completion is awaited explicitly (vmcnt) before the barrier
// that publishes the stage.
__device__ __forceinline__ void direct_load_16(i32x4_t rsrc, unsigned voffset, int soffset, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "buffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory", "m0");
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
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = (A_BYTES / 1024) / NW;     // 1 KiB wave-loads of the A tile per wave
    constexpr int B_LD = (B_BYTES / 1024) / NW;
    static_assert(A_LD >= 1 && B_LD >= 1 && (A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "tile vs waves");
    constexpr int W_ROWB = BN * 2;                   // bytes of one k-row of a [k x n] weight tile

    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;

    const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int m0 = (tile % tiles_m) * BM;
    const int n0 = (tile / tiles_m) * BN;
    const int M = P.M, N = P.N, K = P.K;

    // Buffer resources: A slice [M x lda], W [K x ldw] or [N x ldw]; byte extents fit 31 bits (host-checked).
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

    auto issue_loads = [&](int k0, int stage) {
        const unsigned sa = lds_base + stage * STAGE + wave * 1024;
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
    // depends on row bits 0..3 only, so the 32-row MFMA tiles of a wave differ by constants.
    const int frow = lane & 31, fkc = lane >> 5;
    int a_addr[BK / 16];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks)
        a_addr[ks] = swz_row(wm * WTM + frow, ks * 2 + fkc);
    // [n x k] weights: as the activations.  [k x n] weights: two transposing 8-byte reads per
    // fragment; the swizzle term (k & 3) is a lane constant, (ks, h) add compile-time constants.
    int w_addr[W_KN ? TN : BK / 16];
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
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks)
            w_addr[ks] = A_BYTES + swz_row(wn * WTN + frow, ks * 2 + fkc);
    }

    auto read_frags = [&](const unsigned char *st, int ks, bf16x8_t (&af)[TM], bf16x8_t (&wf)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[i] = *reinterpret_cast<const bf16x8_t *>(st + a_addr[ks] + i * 32 * 128);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (W_KN) {
                const unsigned char *pw = st + w_addr[j] + ks * 16 * W_ROWB;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pw));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pw + 4 * W_ROWB));
                typedef short s16x8_t __attribute__((ext_vector_type(8)));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                wf[j] = __builtin_bit_cast(bf16x8_t, both);
            } else {
                wf[j] = *reinterpret_cast<const bf16x8_t *>(st + w_addr[ks] + j * 32 * 128);
            }
        }
    };

    const int nk = (K + BK - 1) / BK;
    if (nk > 0)
        issue_loads(0, 0);
    __builtin_amdgcn_s_waitcnt(0);    // all counters: the direct loads have landed
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk)
            issue_loads((kt + 1) * BK, (kt + 1) & 1);

        const unsigned char *st = smem + (kt & 1) * STAGE;
        bf16x8_t af[2][TM], wf[2][TN];
        read_frags(st, 0, af[0], wf[0]);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16)
                read_frags(st, ks + 1, af[(ks + 1) & 1], wf[(ks + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);   // keep the next fragments' reads ahead of this MFMA block
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_waitcnt(0);           // this wave's direct loads of the next stage have landed
        __syncthreads();
    }

    const float *recv = P.recv;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * WTM + i * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * WTN + j * 32 + g * 8 + (lane >> 5) * 4;
                if (m < M && n < N) {
                    f32x4_t o;
                    o[0] = acc[i][j][4 * g + 0];
                    o[1] = acc[i][j][4 * g + 1];
                    o[2] = acc[i][j][4 * g + 2];
                    o[3] = acc[i][j][4 * g + 3];
                    const int64_t off = (int64_t)m * P.ldo + n;
                    if (recv != nullptr) {
                        const f32x4_t r = *reinterpret_cast<const f32x4_t *>(recv + off);
                        o = r + o;                       // "O <- B_in + O"
                    }
                    if constexpr (OUT_BF16) {
                        bf16x4_t h;
                        h[0] = static_cast<__bf16>(o[0]);
                        h[1] = static_cast<__bf16>(o[1]);
                        h[2] = static_cast<__bf16>(o[2]);
                        h[3] = static_cast<__bf16>(o[3]);
                        *reinterpret_cast<bf16x4_t *>(static_cast<__bf16 *>(P.out) + off) = h;
                    } else {
                        *reinterpret_cast<f32x4_t *>(static_cast<float *>(P.out) + off) = o;
                    }
                }
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
    // byte extents of both operands must stay below 2^31 (32-bit buffer offsets, OOB marker above them)
    const int64_t lim = (int64_t)1 << 31;
    const int64_t a_bytes = ((int64_t)p.M * p.lda) * 2;
    const int64_t w_bytes = ((int64_t)(w_kn ? p.K : p.N) * p.ldw) * 2;
    return p.M > 0 && p.N > 0 && p.K > 0 && a_bytes < lim && w_bytes < lim;
}

hipError_t launch_gemm_bf16_dl(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s, TileChoice t)
{
    if (t.bm == 256 && t.bn == 256) return launch_cfg<256, 256, 2, 4>(p, w_kn, out_bf16, s);
    if (t.bm == 256 && t.bn == 128) return launch_cfg<256, 128, 4, 2>(p, w_kn, out_bf16, s);
    return launch_cfg<128, 128, 2, 2>(p, w_kn, out_bf16, s);
}

}  // namespace cf

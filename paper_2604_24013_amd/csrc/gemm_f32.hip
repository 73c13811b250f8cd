// fp32 x fp32 -> fp32 chunk GEMM for gfx950 (v_mfma_f32_32x32x2_f32, true fp32
// multiply-accumulate) with the same fused epilogue as the bf16 kernel:
// Alg. 2 "O <- B_in + O" / "B_out <- O", or Alg. 1's in-place slice store.
//
// Workgroup tile BM x BN x 16, four wavefronts in a 2 x 2 grid, each owning
// (BM/2) x (BN/2).  The MFMA "A" operand is fed from the weight tile and "B"
// from the activation tile, so a lane's four consecutive accumulator registers
// are four consecutive output columns (16-byte epilogue accesses).
// Within one k-tile the lanes of the lower / upper half-wave take k = 8q+e and
// k = 8q+4+e for MFMA e of group q; any pairing of k values is valid as long as
// both operands use the same one, and this one lets the activation fragment be
// a single 16-byte LDS read per four MFMAs.
#include "cf_internal.h"

#include <cstdio>
#include <cstdlib>

namespace cf {
namespace {

typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int FBK = 16;
constexpr int A_PITCH = FBK + 4;   // floats per activation row in LDS (80 B: 16-byte aligned, odd multiple of 16 B)

template <int BM, int BN, bool W_KN>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams P, int tiles_m, int tiles_n)
{
    constexpr int NT = 256;
    constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
    constexpr int W_PITCH = W_KN ? (BN + 8) : A_PITCH;   // [k][n] rows of BN+8 floats, or [n][k] rows like A
    constexpr int A_CH = (BM * 4) / NT;                  // 16-byte chunks of the A tile per thread
    constexpr int W_CH = (BN * 4) / NT;
    static_assert(A_CH >= 1 && W_CH >= 1, "tile too small for 256 threads");

    __shared__ __attribute__((aligned(16))) float As[BM * A_PITCH];
    __shared__ __attribute__((aligned(16))) float Ws[W_KN ? FBK * W_PITCH : BN * W_PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int tile = blockIdx.x;
    const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;
    const float *A = static_cast<const float *>(P.A);
    const float *W = static_cast<const float *>(P.W);
    const int M = P.M, N = P.N, K = P.K;

    f32x4_t ra[A_CH], rw[W_CH];
    const f32x4_t zero4 = {0.f, 0.f, 0.f, 0.f};

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int j = 0; j < A_CH; ++j) {
            const int c = tid + j * NT, row = c >> 2, kc = c & 3;
            const int gm = m0 + row, gk = k0 + kc * 4;
            ra[j] = (gm < M && gk < K) ? *reinterpret_cast<const f32x4_t *>(A + (int64_t)gm * P.lda + gk) : zero4;
        }
#pragma unroll
        for (int j = 0; j < W_CH; ++j) {
            const int c = tid + j * NT;
            if constexpr (W_KN) {
                const int kr = c / (BN / 4), nc = c % (BN / 4);
                const int gk = k0 + kr, gn = n0 + nc * 4;
                rw[j] = (gk < K && gn < N) ? *reinterpret_cast<const f32x4_t *>(W + (int64_t)gk * P.ldw + gn) : zero4;
            } else {
                const int row = c >> 2, kc = c & 3;
                const int gn = n0 + row, gk = k0 + kc * 4;
                rw[j] = (gn < N && gk < K) ? *reinterpret_cast<const f32x4_t *>(W + (int64_t)gn * P.ldw + gk) : zero4;
            }
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int j = 0; j < A_CH; ++j) {
            const int c = tid + j * NT, row = c >> 2, kc = c & 3;
            *reinterpret_cast<f32x4_t *>(&As[row * A_PITCH + kc * 4]) = ra[j];
        }
#pragma unroll
        for (int j = 0; j < W_CH; ++j) {
            const int c = tid + j * NT;
            if constexpr (W_KN) {
                const int kr = c / (BN / 4), nc = c % (BN / 4);
                *reinterpret_cast<f32x4_t *>(&Ws[kr * W_PITCH + nc * 4]) = rw[j];
            } else {
                const int row = c >> 2, kc = c & 3;
                *reinterpret_cast<f32x4_t *>(&Ws[row * W_PITCH + kc * 4]) = rw[j];
            }
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

    const int nk = (K + FBK - 1) / FBK;
    const int frow = lane & 31, fh = lane >> 5;
    if (nk > 0)
        load_tiles(0);
    for (int kt = 0; kt < nk; ++kt) {
        store_tiles();
        __syncthreads();
        if (kt + 1 < nk)
            load_tiles((kt + 1) * FBK);
#pragma unroll
        for (int q = 0; q < FBK / 8; ++q) {
            f32x4_t af[TM];
            float wf[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const f32x4_t *>(&As[(wm * WTM + i * 32 + frow) * A_PITCH + q * 8 + fh * 4]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nrow = wn * WTN + j * 32 + frow;
                if constexpr (W_KN) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        wf[j][e] = Ws[(q * 8 + fh * 4 + e) * W_PITCH + nrow];
                } else {
                    const f32x4_t t = *reinterpret_cast<const f32x4_t *>(&Ws[nrow * W_PITCH + q * 8 + fh * 4]);
                    wf[j][0] = t[0];
                    wf[j][1] = t[1];
                    wf[j][2] = t[2];
                    wf[j][3] = t[3];
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[j][e], af[i][e], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    const float *recv = P.recv;
    float *out = static_cast<float *>(P.out);
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
                    if (recv != nullptr)
                        o = *reinterpret_cast<const f32x4_t *>(recv + off) + o;   // "O <- B_in + O"
                    *reinterpret_cast<f32x4_t *>(out + off) = o;
                }
            }
        }
    }
}

template <int BM, int BN>
hipError_t launch_cfg(const GemmParams &p, bool w_kn, hipStream_t s)
{
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const dim3 grid(tiles_m * tiles_n), block(256);
    if (w_kn)
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, true>), grid, block, 0, s, p, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f32(const GemmParams &p, bool w_kn, hipStream_t s, int num_cu)
{
    if (p.M <= 0 || p.N <= 0)
        return hipSuccess;
    const int big = ((p.M + 127) / 128) * ((p.N + 127) / 128);
    bool use_big = big >= num_cu;
    if (const int bm = tuning().tile_f32_bm)             // override: "128x128" or "64x64"
        use_big = bm >= 128;
    if (use_big)
        return launch_cfg<128, 128>(p, w_kn, s);
    return launch_cfg<64, 64>(p, w_kn, s);
}

}  // namespace cf

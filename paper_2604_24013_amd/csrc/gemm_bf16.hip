// bf16 x bf16 -> fp32 chunk GEMM for gfx950 with the fused epilogue of the
// reduce-scatter step (Alg. 2: "O <- B_in + O", then "B_out <- O") or the plain
// in-place slice store of the all-gather step (Alg. 1: "O_s[l] <- ...").
//
// Design (CDNA4):
//  * v_mfma_f32_32x32x16_bf16, 64-wide wavefronts.  The MFMA "A" operand is fed
//    from the weight tile and the "B" operand from the activation tile, so a
//    lane's four consecutive accumulator registers are four consecutive output
//    columns of one output row: the epilogue moves 16-byte vectors.
//  * Workgroup tile BM x BN x 64, LDS double-buffered (two stages of
//    (BM+BN) x 64 bf16); the next k-tile is fetched from global memory into
//    registers while the current one is multiplied, then written to the other
//    stage: one barrier per k-tile.
//  * Both operand tiles sit in LDS with k contiguous (128-byte rows of eight
//    16-byte chunks) under an XOR swizzle that makes the 16-byte fragment reads,
//    the straight tile writes and the transposing writes of a [k x n] weight
//    tile all free of bank conflicts.
//  * A [k x n] weight tile (n contiguous in memory) is transposed in registers
//    (8x8 blocks of 16-bit values) on its way to LDS.
//  * Workgroup ids are remapped so that each XCD (own L2) works on a contiguous
//    band of tiles that share operand rows / columns.
#include "cf_internal.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace cf {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int BK = 64;          // k extent of one LDS stage
constexpr int ROW_BYTES = 128;  // BK * sizeof(bf16)

// Byte offset of 16-byte chunk kc (0..7) of tile row `row` inside an operand tile.
__device__ __forceinline__ int lds_swz(int row, int kc)
{
    const int r0 = row & 1, r1 = (row >> 1) & 1, r2 = (row >> 2) & 1;
    const int r3 = (row >> 3) & 1, r4 = (row >> 4) & 1, r5 = (row >> 5) & 1;
    const int half = r0 ^ r3;
    const int kcp = kc ^ (((r1 ^ r4) << 2) | ((r2 ^ r5) << 1) | r3);
    return ((row >> 1) << 8) + (half << 7) + (kcp << 4);
}

// Tile of R rows x 64 k, source rows are k-contiguous in memory.
template <int R, int NT>
struct StraightLoader {
    static constexpr int CH = (R * 8) / NT;
    static_assert(CH >= 1 && (R * 8) % NT == 0, "tile rows vs threads");
    uint4 v[CH];

    __device__ __forceinline__ void load(const __bf16 *base, int64_t ld, int row0, int rows_total,
                                         int k0, int K, int tid)
    {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + j * NT;
            const int row = c >> 3, kc = c & 7;
            const int grow = row0 + row, gk = k0 + kc * 8;
            uint4 x = make_uint4(0u, 0u, 0u, 0u);
            if (grow < rows_total && gk < K)
                x = *reinterpret_cast<const uint4 *>(base + (int64_t)grow * ld + gk);
            v[j] = x;
        }
    }
    __device__ __forceinline__ void store(unsigned char *lds, int tid) const
    {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int c = tid + j * NT;
            *reinterpret_cast<uint4 *>(lds + lds_swz(c >> 3, c & 7)) = v[j];
        }
    }
};

// Tile of 64 k x BN n from a [K x N] matrix (n contiguous): each of the first BN
// threads owns one 8(k) x 8(n) block, transposes it in registers and writes
// eight 16-byte k-runs.
template <int BN_, int NT>
struct TransposeLoader {
    static_assert(BN_ <= NT, "one 8x8 block per thread");
    uint4 v[8];

    __device__ __forceinline__ void load(const __bf16 *W, int64_t ldw, int n0, int N, int k0, int K, int tid)
    {
        if (tid < BN_) {
            const int kb = (tid >> 3) & 7;
            const int ncb = ((tid >> 6) << 3) + (tid & 7);
            const int gn = n0 + ncb * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int gk = k0 + kb * 8 + j;
                uint4 x = make_uint4(0u, 0u, 0u, 0u);
                if (gk < K && gn < N)
                    x = *reinterpret_cast<const uint4 *>(W + (int64_t)gk * ldw + gn);
                v[j] = x;
            }
        }
    }
    __device__ __forceinline__ void store(unsigned char *lds, int tid) const
    {
        if (tid < BN_) {
            const int kb = (tid >> 3) & 7;
            const int ncb = ((tid >> 6) << 3) + (tid & 7);
            const unsigned in[8][4] = {
                {v[0].x, v[0].y, v[0].z, v[0].w}, {v[1].x, v[1].y, v[1].z, v[1].w},
                {v[2].x, v[2].y, v[2].z, v[2].w}, {v[3].x, v[3].y, v[3].z, v[3].w},
                {v[4].x, v[4].y, v[4].z, v[4].w}, {v[5].x, v[5].y, v[5].z, v[5].w},
                {v[6].x, v[6].y, v[6].z, v[6].w}, {v[7].x, v[7].y, v[7].z, v[7].w}};
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                unsigned o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned lo = in[2 * e][n >> 1], hi = in[2 * e + 1][n >> 1];
                    o[e] = (n & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
                }
                *reinterpret_cast<uint4 *>(lds + lds_swz(ncb * 8 + n, kb)) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    }
};

// XCD-aware remap: hardware hands consecutive workgroup ids to the 8 XCDs in
// turn; give XCD x the contiguous tile range [start(x), start(x+1)).
__device__ __forceinline__ int xcd_remap(int pid, int total)
{
    constexpr int NXCD = 8;
    const int q = total / NXCD, rem = total % NXCD;
    const int xcd = pid % NXCD, idx = pid / NXCD;
    return xcd * q + (xcd < rem ? xcd : rem) + idx;
}

template <int BM, int BN, int WGM, int WGN, bool W_KN, bool OUT_BF16>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(GemmParams P, int tiles_m, int tiles_n)
{
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the MFMA tile");
    constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, STAGE = A_BYTES + B_BYTES;

    __shared__ __attribute__((aligned(256))) unsigned char smem[2 * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;

    const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int m0 = (tile % tiles_m) * BM;      // M fastest: a band shares weight columns
    const int n0 = (tile / tiles_m) * BN;

    const __bf16 *A = static_cast<const __bf16 *>(P.A);
    const __bf16 *W = static_cast<const __bf16 *>(P.W);
    const int M = P.M, N = P.N, K = P.K;

    StraightLoader<BM, NT> la;
    StraightLoader<BN, NT> lw_nk;
    TransposeLoader<BN, NT> lw_kn;

    auto load_tiles = [&](int k0) {
        la.load(A, P.lda, m0, M, k0, K, tid);
        if constexpr (W_KN)
            lw_kn.load(W, P.ldw, n0, N, k0, K, tid);
        else
            lw_nk.load(W, P.ldw, n0, N, k0, K, tid);
    };
    auto store_tiles = [&](int stage) {
        unsigned char *sa = smem + stage * STAGE;
        la.store(sa, tid);
        if constexpr (W_KN)
            lw_kn.store(sa + A_BYTES, tid);
        else
            lw_nk.store(sa + A_BYTES, tid);
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[i][j][e] = 0.0f;

    const int nk = (K + BK - 1) / BK;
    const int frow = lane & 31, fkc = lane >> 5;

    if (nk > 0) {
        load_tiles(0);
        store_tiles(0);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const bool more = (kt + 1) < nk;
        if (more)
            load_tiles((kt + 1) * BK);

        const unsigned char *sa = smem + (kt & 1) * STAGE;
        const unsigned char *sb = sa + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t af[TM], wf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t *>(sa + lds_swz(wm * WTM + i * 32 + frow, ks * 2 + fkc));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                wf[j] = *reinterpret_cast<const bf16x8_t *>(sb + lds_swz(wn * WTN + j * 32 + frow, ks * 2 + fkc));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
        }

        if (more)
            store_tiles((kt + 1) & 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register 4g+e of lane L holds
    //   row m = tile row (L & 31), column n = 8g + 4(L >> 5) + e   of the 32x32 tile.
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
            hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, true, true>), grid, block, 0, s, p, tiles_m, tiles_n);
        else
            hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, true, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    } else {
        if (out_bf16)
            hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, false, true>), grid, block, 0, s, p, tiles_m, tiles_n);
        else
            hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, false, false>), grid, block, 0, s, p, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace

TileChoice choose_tile_bf16(int M, int N, int K, int num_cu)
{
    // Measured on MI355X: the kernels are bound by the rate at which a CU can pull operand tiles
    // through its L1 (64 B/clk), so the largest tile that still fills the chip wins; a grid of at
    // most one 128x128 workgroup per CU runs best with four LDS stages, and when even that leaves
    // most CUs idle the k range is split (if the caller registered a workspace).
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    const int want = (num_cu * 7) / 8;
    TileChoice t{128, 128, 1};
    if (tiles(256, 256) >= want) return TileChoice{256, 256, 1};
    if (tiles(256, 128) >= want) return TileChoice{256, 128, 1};
    const int t128 = tiles(128, 128);
    if (t128 > num_cu) return t;                 // two workgroups per CU, two stages each
    t.deep = true;
    const int ktiles = (K + 63) / 64;
    if (t128 * 3 <= num_cu && ktiles / 3 >= 16)
        t.splitk = 3;
    else if (t128 * 2 <= num_cu && ktiles / 2 >= 16)
        t.splitk = 2;
    return t;
}

static bool staged_kernel_forced()                   // "staged": the register-staged kernel of this file
{
    return tuning().staged != 0;
}

bool gemm_bf16_takes_recv_list(const GemmParams &p, bool w_kn)
{
    return p.M > 0 && p.N > 0 && !staged_kernel_forced() && gemm_bf16_dl_supported(p, w_kn);
}

// Tile of a launch: the per-step choice, the persistent rank step's cost model, then the overrides.
static TileChoice tile_of_launch(const GemmParams &p, int num_cu)
{
    TileChoice t = choose_tile_bf16(p.M, p.N, p.K, num_cu);
    if (p.n_steps > 0) {
        // Persistent rank step: n_steps * tiles work items share one grid, so a step need not fill the chip
        // alone.  Cost of a tile shape = rounds over the chip x tile area x its measured cost per flop
        // (per-k-tile time of a full grid: 256x256 1.00, 256x128 1.15, 128x128 1.30, relative).
        const struct { int bm, bn; double cost; } cand[3] = {{256, 256, 1.00}, {256, 128, 1.15}, {128, 128, 1.30}};
        double best = 0.0;
        for (int c = 0; c < 3; ++c) {
            const int64_t items = (int64_t)((p.M + cand[c].bm - 1) / cand[c].bm) * ((p.N + cand[c].bn - 1) / cand[c].bn) * p.n_steps;
            const int64_t rounds = (items + num_cu - 1) / num_cu;
            const double cost = (double)rounds * cand[c].bm * cand[c].bn * cand[c].cost;
            if (c == 0 || cost < best) {
                best = cost;
                t.bm = cand[c].bm;
                t.bn = cand[c].bn;
            }
        }
        t.splitk = 1;
        t.deep = true;                               // 128x128: one workgroup per CU, four stages
    }
    const Tuning tn = tuning();                      // overrides: tile shape, stages, k-splits per output tile
    if (tn.tile_bm > 0) {
        t.bm = tn.tile_bm;
        t.bn = tn.tile_bn;
    }
    if (tn.deep >= 0)
        t.deep = tn.deep != 0;
    if (tn.splitk >= 1)
        t.splitk = tn.splitk;
    return t;
}

int gemm_bf16_tiles_landing_arrivals(const GemmParams &p, bool w_kn, int num_cu)
{
    const Tuning tn = tuning();                      // COMMFUSE_CARRY=0 keeps the copies in front
    if (p.n_steps < 2 || !gemm_bf16_takes_recv_list(p, w_kn) || (tn.carry >= 0 && tn.carry == 0))
        return 0;
    const TileChoice t = tile_of_launch(p, num_cu);
    const int64_t tiles = (int64_t)((p.M + t.bm - 1) / t.bm) * ((p.N + t.bn - 1) / t.bn);
    // every workgroup of the launch must be resident at once (a work item waits for others): one grid over the chip
    return tiles <= 1 << 20 ? (int)tiles : 0;
}

bool gemm_bf16_lands_beside(const GemmParams &p, bool w_kn, bool out_bf16, int num_cu)
{
    const Tuning tn = tuning();
    if (p.n_steps <= 0 || out_bf16 || p.a_t || !gemm_bf16_takes_recv_list(p, w_kn) || (tn.carry >= 0 && tn.carry == 0))
        return false;
    for (int j = 0; j < p.n_steps; ++j)
        if (p.flag_step[j] != nullptr)
            return false;
    return !gemm_bf16_dl_streams_recv(p, w_kn, out_bf16, tile_of_launch(p, num_cu));
}

bool gemm_bf16_carries_delivery(const GemmParams &p, bool w_kn, bool out_bf16, int num_cu, bool reduce_scatter)
{
    if (p.M <= 0 || p.N <= 0 || p.n_steps <= 0 || staged_kernel_forced() || !gemm_bf16_dl_supported(p, w_kn))
        return false;
    for (int j = 0; j < p.n_steps; ++j)
        if (p.flag_step[j] != nullptr)
            return false;                            // a step that waits for a flag keeps its B_in loads in the epilogue
    if (reduce_scatter) {
        const TileChoice t = tile_of_launch(p, num_cu);
        if (!gemm_bf16_dl_streams_recv(p, w_kn, out_bf16, t))
            return false;
    } else if (!gemm_bf16_dl_carries_operand(p)) {
        return false;
    }
    // Wherever the launch can, it does (measured, with the landed tiles stored as whole 128-byte lines: 7B
    // down-projection rank step 76 -> 57 us, 70B 482 -> 470 us against deliveries copied in front of the launch).
    // COMMFUSE_CARRY=0 keeps the copies in front.
    const Tuning tn = tuning();
    return tn.carry >= 0 ? tn.carry != 0 : true;
}

int gemm_bf16_steps_per_launch(const GemmParams &p, bool w_kn, int num_cu)
{
    if (p.M <= 0 || p.N <= 0 || p.n_steps <= 1 || staged_kernel_forced() || !gemm_bf16_dl_supported(p, w_kn))
        return p.n_steps > 0 ? p.n_steps : 1;
    const TileChoice t = tile_of_launch(p, num_cu);
    const int64_t tiles = (int64_t)((p.M + t.bm - 1) / t.bm) * ((p.N + t.bn - 1) / t.bn);
    const int64_t wgs = (int64_t)num_cu * ((t.bm == 128 && t.bn == 128 && !t.deep) ? 2 : 1);
    int64_t per_round = (wgs + tiles - 1) / tiles;       // steps that fill the chip once (rounded up)
    if (per_round < 1)
        per_round = 1;
    const int64_t launches = (p.n_steps + per_round - 1) / per_round;
    return (int)((p.n_steps + launches - 1) / launches);   // equal groups
}

hipError_t launch_gemm_bf16(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s, int num_cu)
{
    if (p.M <= 0 || p.N <= 0)
        return hipSuccess;
    const TileChoice t = tile_of_launch(p, num_cu);
    const bool staged = staged_kernel_forced();
    if (!staged && gemm_bf16_dl_supported(p, w_kn))
        return launch_gemm_bf16_dl(p, w_kn, out_bf16, s, t);
    if (p.n_recv_more != 0 || p.a_t || p.n_steps > 0)
        return hipErrorInvalidValue;                 // callers ask gemm_bf16_takes_recv_list first
    if (t.bm == 256 && t.bn == 256) return launch_cfg<256, 256, 2, 4>(p, w_kn, out_bf16, s);
    if (t.bm == 256 && t.bn == 128) return launch_cfg<256, 128, 4, 2>(p, w_kn, out_bf16, s);
    return launch_cfg<128, 128, 2, 2>(p, w_kn, out_bf16, s);
}

}  // namespace cf

// Attention of one query slice against the rank's full keys and values (Alg. 4: scores = Q_s[l] K^T,
// Softmax, times V), bf16 operands, fp32 accumulation and fp32 online softmax, for gfx950.
//
// One workgroup = 4 waves = 4 * 32 * QT queries of one (batch element, head); it walks over the keys in
// tiles of 64.  Per tile and wave:
//   S^T = K Q^T      v_mfma_f32_32x32x16_bf16 with the key tile as the MFMA "A" operand and the wave's
//                    queries (kept in registers for the whole walk) as "B": a lane then owns ONE query
//                    (lane & 31) and 16 of every 32 keys, so the softmax statistics of a query live in two
//                    lanes (lane, lane ^ 32) and need one cross-lane exchange per tile;
//   online softmax   m' = max(m, max S), P = exp2(S - m'), l = l * exp2(m - m') + sum P, O *= exp2(m - m');
//   O^T += V^T P^T   the probabilities, rounded to bf16, are already in the register layout of an MFMA "B"
//                    operand if the 16 contraction slots of a slice are taken to mean the keys the lane
//                    holds (a fixed permutation of the slice's keys); the V tile stays [key x d] in LDS and
//                    its transposed fragments are fetched with the transposing LDS read at the row offsets
//                    of that same permutation.  No data moves between lanes, no P tile goes through LDS.
// K and V tiles go global -> LDS directly (buffer_load ... lds), double-buffered; a key row of 256 bytes has
// its sixteen 16-byte chunks XOR-ed with (key & 15) so that the fragment reads of 16 consecutive keys hit 16
// different bank groups; the V tile uses the [k x n] weight-tile layout of the chunk GEMM.
// Keys beyond the sequence read as zero through the buffer bounds check and are masked to -inf; query rows
// beyond the slice are computed on zeros and not stored.
#include "cf_internal.h"

#include <cmath>
#include <cstdlib>
#include <type_traits>

namespace cf {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

constexpr unsigned OOB = 0x80000000u;
constexpr int DH = 128;                  // head dimension this kernel is written for
constexpr int BKV = 64;                  // keys per tile
constexpr int ROWB = DH * 2;             // bytes of one key / value row
constexpr int TILE_BYTES = BKV * ROWB;   // 16 KiB

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

// Wave-wide 16-byte-per-lane load from global memory straight into LDS (lane L lands at lds_addr + 16 L).
__device__ __forceinline__ void direct_load_16(i32x4_t rsrc, unsigned voffset, int soffset, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "buffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// QT: 32-query tiles per wave (1 or 2); NW: waves per workgroup (4, or 8 = two per SIMD, so that one wave's
// softmax arithmetic runs under the other's MFMAs).
template <int QT, int NW>
__global__ __launch_bounds__(64 * NW) void attn_slice_kernel(AttnParams P)
{
    constexpr int NT = 64 * NW;          // threads per workgroup
    constexpr int WQ = 32 * QT;          // queries per wave
    constexpr int BQ = NW * WQ;          // queries per workgroup
    constexpr int KT = BKV / 32;         // 32-key MFMA tiles per key tile
    constexpr int DS = DH / 16;          // 16-wide d slices (contraction of S^T)
    constexpr int DT = DH / 32;          // 32-wide d tiles (rows of O^T)
    constexpr int LOADS = 2 * TILE_BYTES / 1024 / NW;  // wave-loads per wave per key tile (K and V)

    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * 2 * TILE_BYTES];   // [buffer][K | V]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, lh = lane >> 5;

    const int qblocks = (P.c + BQ - 1) / BQ;
    const int KSP = P.ksplit;                                        // workgroups sharing a query block
    const int split = blockIdx.x % KSP;
    const int group = blockIdx.x / KSP;                              // (slice, batch element, head, query block)
    const int qb = group % qblocks;
    const int head = (group / qblocks) % P.heads;
    const int b = (group / (qblocks * P.heads)) % P.batch;
    const int slice = P.l + group / (qblocks * P.heads * P.batch);
    const int S = P.S;

    const size_t mat = (size_t)S * DH;                               // elements of one (b, head) matrix
    const __bf16 *Qm = static_cast<const __bf16 *>(P.Q) + ((size_t)b * P.heads + head) * mat;
    const __bf16 *Km = static_cast<const __bf16 *>(P.K) + ((size_t)b * P.heads + head) * mat;
    const __bf16 *Vm = static_cast<const __bf16 *>(P.V) + ((size_t)b * P.heads + head) * mat;
    const i32x4_t k_rsrc = make_rsrc(Km, (unsigned)(mat * 2));
    const i32x4_t v_rsrc = make_rsrc(Vm, (unsigned)(mat * 2));
    const unsigned lds_base = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem);

    // The wave's queries as MFMA "B" fragments: lane (lq, lh) holds d = 16 ks + 8 lh + 0..7 of query lq.
    const int q_in_slice = qb * BQ + wave * WQ;                      // first query of this wave in the slice
    bf16x8_t qf[QT][DS];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        const int qi = q_in_slice + t * 32 + lq;
        const bool ok = qi < P.c;
        const __bf16 *qrow = Qm + (size_t)(slice * P.c + (ok ? qi : 0)) * DH;
#pragma unroll
        for (int ks = 0; ks < DS; ++ks) {
            bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(qrow + ks * 16 + lh * 8);
            if (!ok)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (__bf16)0.0f;
            qf[t][ks] = v;
        }
    }

    // Direct loads of key tile `kt` into buffer `buf`: wave-load j covers 4 rows of 256 bytes.
    // K: the lane at LDS chunk position cp of row r fetches global chunk cp ^ (r & 15).
    // V: [k x n] weight-tile layout: the 64-byte groups of a row are XOR-ed with (row & 3).
    unsigned k_off[LOADS / 2], v_off[LOADS / 2];
#pragma unroll
    for (int j = 0; j < LOADS / 2; ++j) {
        const int row = (j * NW + wave) * 4 + (lane >> 4);           // key row inside the tile
        const int cp = lane & 15;
        k_off[j] = (unsigned)(row * ROWB + ((cp ^ (row & 15)) << 4));
        const int inrow = cp << 4;
        const int q = (inrow >> 6) ^ (row & 3);
        v_off[j] = (unsigned)(row * ROWB + (q << 6) + (inrow & 63));
    }
    auto issue_tile = [&](int kt, int buf) {
        const int key0 = kt * BKV;
        const unsigned sa = lds_base + buf * 2 * TILE_BYTES + wave * 1024;
#pragma unroll
        for (int j = 0; j < LOADS / 2; ++j) {
            const int row = (j * NW + wave) * 4 + (lane >> 4);
            const bool in = key0 + row < S;                          // rows beyond the sequence read as zero
            direct_load_16(k_rsrc, in ? k_off[j] : OOB, key0 * ROWB, sa + j * NW * 1024);
            direct_load_16(v_rsrc, in ? v_off[j] : OOB, key0 * ROWB, sa + TILE_BYTES + j * NW * 1024);
        }
    };

    // Fragment addresses inside a buffer.
    // K as "A" operand: lane (key = lq, lh) reads chunk (2 ks + lh) of its key row, swizzled.
    // V^T as "A" operand: transposing reads; lane (blk = lane >> 4, i16 = lane & 15); the two reads of a
    // slice start at key rows 4 lh + (i16 >> 2) and 8 more (the permutation the probabilities come in).
    const int blk = lane >> 4, i16 = lane & 15;
    const int v_kl = 4 * (blk >> 1) + (i16 >> 2);
    const int v_nl = (blk & 1) * 16 + (i16 & 3) * 4;
    int v_addr[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
        v_addr[t] = TILE_BYTES + v_kl * ROWB + (((t) ^ (v_kl & 3)) << 6) + v_nl * 2;

    f32x16_t oacc[QT][DT], lacc[QT];     // lacc: every element of a lane is the row sum l of the lane's query
    float m_run[QT], l_run[QT];
    bf16x8_t ones;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        ones[e] = (__bf16)1.0f;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        m_run[t] = -INFINITY;
        l_run[t] = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            lacc[t][e] = 0.0f;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                oacc[t][d][e] = 0.0f;
    }
    const float sl2 = P.scale * 1.4426950408889634f;                 // scores are kept in units of log2(e)

    const int nkt_all = (S + BKV - 1) / BKV;
    const int kt0 = (int)(((long long)nkt_all * split) / KSP);       // this workgroup's key tiles: [kt0, nkt)
    const int nkt = (int)(((long long)nkt_all * (split + 1)) / KSP);
    issue_tile(kt0, kt0 & 1);
    wait_vmcnt<0>();
    __syncthreads();

    for (int kt = kt0; kt < nkt; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nkt)
            issue_tile(kt + 1, buf ^ 1);                             // that buffer was released by the last barrier
        const unsigned char *st = smem + buf * 2 * TILE_BYTES;

        // S^T = K Q^T
        f32x16_t sacc[QT][KT];
#pragma unroll
        for (int t = 0; t < QT; ++t)
#pragma unroll
            for (int j = 0; j < KT; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    sacc[t][j][e] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < DS; ++ks) {
#pragma unroll
            for (int j = 0; j < KT; ++j) {
                const int row = j * 32 + lq;
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(st + row * ROWB + (((2 * ks + lh) ^ (row & 15)) << 4));
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    sacc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][ks], sacc[t][j], 0, 0, 0);
            }
        }

        // Online softmax; register 4g+e of key tile j is key 32 j + 8 g + 4 lh + e.  The vector ALU is the
        // busiest unit of this loop, so its work per score is kept to a max, one fused multiply-add, one exp2 and
        // half a packed conversion:
        //  * keys beyond the sequence are masked in the one tile that can hold them only;
        //  * the exponentials are taken against a running reference m that is raised only when the tile's
        //    maximum exceeds it by more than 2^RAISE (probabilities then stay below 2^RAISE: no overflow, the
        //    same relative precision in bf16), so the rescaling of the accumulators is rare and sits in a
        //    wave-uniform branch;
        //  * the row sums l come out of the matrix pipe: one more MFMA per 16-key slice with an all-ones "A"
        //    operand adds up exactly the rounded probabilities that multiply V (every row of its result is the
        //    sum over the slice's keys, both lanes of a query get the whole sum).
        constexpr float RAISE = 8.0f;
        bf16x8_t pf[QT][KT][2];                                      // "B" fragments of the two 16-key slices of a tile
        const bool partial = (kt + 1) * BKV > S;                     // uniform
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            if (partial) {
                float ninf = -INFINITY;
                asm volatile("" : "+v"(ninf));                       // (keeps this a branch: not 32 selects in every tile)
#pragma unroll
                for (int j = 0; j < KT; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kt * BKV + j * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                        if (key >= S)
                            sacc[t][j][r] = ninf;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < KT; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    mx = fmaxf(mx, sacc[t][j][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));                      // the query's other half lives in lane ^ 32
            const float mxs = mx * sl2;                              // scale > 0: the maximum of the scaled scores
            if (__builtin_amdgcn_ballot_w64(mxs > m_run[t] + RAISE) != 0) {   // finite: every tile holds a key
                const float m_new = fmaxf(m_run[t], mxs);
                float alpha = exp2f(m_run[t] - m_new);               // 0 on the first tile (m_run = -inf)
                asm volatile("" : "+v"(alpha));                      // (keeps this a branch, as above)
                m_run[t] = m_new;
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    lacc[t][e] *= alpha;
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        oacc[t][d][e] *= alpha;
            }
            const float nm = -m_run[t];
#pragma unroll
            for (int j = 0; j < KT; ++j)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    bf16x8_t f;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        f[e] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sacc[t][j][8 * s2 + e], sl2, nm));   // bare v_exp_f32: arguments below -126 give 0
                    pf[t][j][s2] = f;
                }
        }

        // O^T += V^T P^T, l += 1^T P^T
#pragma unroll
        for (int j = 0; j < KT; ++j)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int krow = (j * 32 + s2 * 16) * ROWB;
#pragma unroll
                for (int d = 0; d < DT; ++d) {
                    const unsigned char *pv = st + v_addr[d] + krow;
                    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4_t *)(pv));
                    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4_t *)(pv + 8 * ROWB));
                    const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                    for (int t = 0; t < QT; ++t)
                        oacc[t][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t][j][s2], oacc[t][d], 0, 0, 0);
                }
#pragma unroll
                for (int t = 0; t < QT; ++t)
                    lacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf[t][j][s2], lacc[t], 0, 0, 0);
            }

        wait_vmcnt<0>();                                             // the next tile has landed
        __syncthreads();                                             // ... for every wave, and this one is read by all
    }

#pragma unroll
    for (int t = 0; t < QT; ++t)
        l_run[t] = lacc[t][0];                                       // the whole row sum, in both lanes of the query

    // Key split across workgroups: park (m, l, O) in the workspace, thread-major so that every access is a
    // coalesced 4 bytes per lane; the workgroup that arrives last merges all splits (its own included) in
    // split order.  Cross-XCD visibility as in the chunk GEMM's k-split: device-coherent cache policy on
    // exactly these accesses, relaxed agent-scope atomics on the counter.
    if (KSP > 1) {
        constexpr int COHERENT = 1 | 16;
        constexpr int NV = QT * DT * 16 + 2 * QT;                    // floats per thread
        const size_t part = (size_t)NV * NT;
        auto part_rsrc = [&](int sp) {
            return __builtin_amdgcn_make_buffer_rsrc(P.ws + ((size_t)group * KSP + sp) * part, 0, (int)(part * 4), 0x00020000);
        };
        {
            __amdgpu_buffer_rsrc_t rs = part_rsrc(split);
#pragma unroll
            for (int t = 0; t < QT; ++t) {
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        // (through a plain VGPR: storing the accumulator elements straight from their AGPRs
                        // came out of this compiler as sixteen stores of element 0)
                        float v = oacc[t][d][e];
                        asm volatile("" : "+v"(v));
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rs,
                                                              (((t * DT + d) * 16 + e) * NT + tid) * 4, 0, COHERENT);
                    }
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, m_run[t]), rs,
                                                      ((QT * DT * 16 + 2 * t) * NT + tid) * 4, 0, COHERENT);
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, l_run[t]), rs,
                                                      ((QT * DT * 16 + 2 * t + 1) * NT + tid) * 4, 0, COHERENT);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        unsigned *arrived = reinterpret_cast<unsigned *>(smem);       // the key tiles are no longer read
        if (tid == 0)
            *arrived = __hip_atomic_fetch_add(&P.counters[group], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*arrived != (unsigned)(KSP - 1))
            return;
        if (tid == 0)
            __hip_atomic_store(&P.counters[group], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int t = 0; t < QT; ++t) {
            float m_all = -INFINITY;
            for (int sp = 0; sp < KSP; ++sp) {
                __amdgpu_buffer_rsrc_t rs = part_rsrc(sp);
                m_all = fmaxf(m_all, __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                         rs, ((QT * DT * 16 + 2 * t) * NT + tid) * 4, 0, COHERENT)));
            }
            float l_all = 0.0f;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    oacc[t][d][e] = 0.0f;
            // two splits per round: their loads (2 x 66 per lane) are in flight together, the sums stay in split order
            for (int sp = 0; sp < KSP; sp += 2) {
                const bool two = sp + 1 < KSP;
                __amdgpu_buffer_rsrc_t rs0 = part_rsrc(sp), rs1 = part_rsrc(two ? sp + 1 : sp);
                auto ld = [&](__amdgpu_buffer_rsrc_t rs, int idx) {
                    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (idx * NT + tid) * 4, 0, COHERENT));
                };
                const float m0 = ld(rs0, QT * DT * 16 + 2 * t), l0 = ld(rs0, QT * DT * 16 + 2 * t + 1);
                const float m1 = ld(rs1, QT * DT * 16 + 2 * t), l1 = ld(rs1, QT * DT * 16 + 2 * t + 1);
                float v0[DT][16], v1[DT][16];
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        v0[d][e] = ld(rs0, (t * DT + d) * 16 + e);
                        v1[d][e] = ld(rs1, (t * DT + d) * 16 + e);
                    }
                const float f0 = exp2f(m0 - m_all);                  // every split holds at least one key tile
                const float f1 = two ? exp2f(m1 - m_all) : 0.0f;
                l_all += l0 * f0;
                l_all += l1 * f1;
#pragma unroll
                for (int d = 0; d < DT; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        oacc[t][d][e] += f0 * v0[d][e];
                        oacc[t][d][e] += f1 * v1[d][e];
                    }
            }
            l_run[t] = l_all;
        }
    }

    // O = O^T / l, rounded to bf16, written as [token x (head, d)]: the left operand of the output projection.
    __bf16 *out = static_cast<__bf16 *>(P.out) + (size_t)(slice - P.l) * P.out_slice_stride;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
        const float inv = 1.0f / l_run[t];
        const int qi = q_in_slice + t * 32 + lq;
        if (qi < P.c) {
            __bf16 *orow = out + ((size_t)b * P.c + qi) * P.ldo + (size_t)head * DH;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4_t h;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        h[e] = (__bf16)(oacc[t][d][4 * g + e] * inv);
                    *reinterpret_cast<u32x2_t *>(orow + d * 32 + 8 * g + 4 * lh) = __builtin_bit_cast(u32x2_t, h);
                }
        }
    }
}

// Variant for slices with few queries (the per-step grids of Alg. 4 are small: seq/p queries per head): one
// workgroup = 32 queries of one (batch element, head); its four waves split the KEYS -- wave w takes the
// 32-key tiles w, w+4, w+8, ... -- each with its own double-buffered K/V landing zone in LDS (no barrier in
// the walk), and the four partial results (m, l, unnormalised O) are merged through LDS at the end.
__global__ __launch_bounds__(256) void attn_slice_ksplit_kernel(AttnParams P)
{
    constexpr int BK = 32;                   // keys per tile
    constexpr int TB = BK * ROWB;            // 8 KiB: one K (or V) tile
    constexpr int DS = DH / 16, DT = DH / 32;
    constexpr int WAVE_LDS = 4 * TB;         // [buffer][K | V]

    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * WAVE_LDS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, lh = lane >> 5;

    const int qtiles = (P.c + 31) / 32;
    const int head = blockIdx.x % P.heads;   // neighbouring workgroups (one per XCD in turn) take different heads:
    const int qt = (blockIdx.x / P.heads) % qtiles;   // with 8 heads, each XCD's L2 serves one head's K and V
    const int b = blockIdx.x / (P.heads * qtiles);
    const int S = P.S;

    const size_t mat = (size_t)S * DH;
    const __bf16 *Qm = static_cast<const __bf16 *>(P.Q) + ((size_t)b * P.heads + head) * mat;
    const __bf16 *Km = static_cast<const __bf16 *>(P.K) + ((size_t)b * P.heads + head) * mat;
    const __bf16 *Vm = static_cast<const __bf16 *>(P.V) + ((size_t)b * P.heads + head) * mat;
    const i32x4_t k_rsrc = make_rsrc(Km, (unsigned)(mat * 2));
    const i32x4_t v_rsrc = make_rsrc(Vm, (unsigned)(mat * 2));
    const unsigned lds_base = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem) + wave * WAVE_LDS;
    unsigned char *my = smem + wave * WAVE_LDS;

    const int qi = qt * 32 + lq;
    const bool q_ok = qi < P.c;
    bf16x8_t qf[DS];
    {
        const __bf16 *qrow = Qm + (size_t)(P.l * P.c + (q_ok ? qi : 0)) * DH;
#pragma unroll
        for (int ks = 0; ks < DS; ++ks) {
            bf16x8_t v = *reinterpret_cast<const bf16x8_t *>(qrow + ks * 16 + lh * 8);
            if (!q_ok)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (__bf16)0.0f;
            qf[ks] = v;
        }
    }

    // wave-load j (1 KiB) covers rows 4j .. 4j+3 of the tile; layouts as in the kernel above
    unsigned k_off[8], v_off[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int row = j * 4 + (lane >> 4);
        const int cp = lane & 15;
        k_off[j] = (unsigned)(row * ROWB + ((cp ^ (row & 15)) << 4));
        const int inrow = cp << 4;
        v_off[j] = (unsigned)(row * ROWB + (((inrow >> 6) ^ (row & 3)) << 6) + (inrow & 63));
    }
    auto issue_tile = [&](int kt, int buf) {
        const int key0 = kt * BK;
        const unsigned sa = lds_base + buf * 2 * TB;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool in = key0 + j * 4 + (lane >> 4) < S;
            direct_load_16(k_rsrc, in ? k_off[j] : OOB, key0 * ROWB, sa + j * 1024);
            direct_load_16(v_rsrc, in ? v_off[j] : OOB, key0 * ROWB, sa + TB + j * 1024);
        }
    };

    const int blk = lane >> 4, i16 = lane & 15;
    const int v_kl = 4 * (blk >> 1) + (i16 >> 2);
    const int v_nl = (blk & 1) * 16 + (i16 & 3) * 4;
    int v_addr[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
        v_addr[t] = TB + v_kl * ROWB + ((t ^ (v_kl & 3)) << 6) + v_nl * 2;

    f32x16_t oacc[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            oacc[d][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float sl2 = P.scale * 1.4426950408889634f;

    const int nkt = (S + BK - 1) / BK;
    int buf = 0;
    if (wave < nkt)
        issue_tile(wave, 0);
    for (int kt = wave; kt < nkt; kt += 4) {
        wait_vmcnt<0>();                                             // tile kt has landed (this wave's own loads)
        if (kt + 4 < nkt)
            issue_tile(kt + 4, buf ^ 1);                             // its last readers' MFMAs were issued long ago
        const unsigned char *st = my + buf * 2 * TB;

        f32x16_t sacc;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sacc[e] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < DS; ++ks) {
            const bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(st + lq * ROWB + (((2 * ks + lh) ^ (lq & 15)) << 4));
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc, 0, 0, 0);
        }
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kt * BK + 8 * (r >> 2) + 4 * lh + (r & 3);
            const float sv = key < S ? sacc[r] * sl2 : -INFINITY;
            sacc[r] = sv;
            mx = fmaxf(mx, sv);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f(m_run - m_new);
        float sum = 0.0f;
        bf16x8_t pf[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const __bf16 pb = (__bf16)exp2f(sacc[8 * s2 + e] - m_new);
                pf[s2][e] = pb;
                sum += (float)pb;
            }
        l_run = l_run * alpha + sum;
        m_run = m_new;
        if (__any(alpha != 1.0f)) {                                  // the running maximum settles after a few tiles
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    oacc[d][e] *= alpha;
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int d = 0; d < DT; ++d) {
                const unsigned char *pv = st + v_addr[d] + s2 * 16 * ROWB;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pv));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4_t *)(pv + 8 * ROWB));
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s2], oacc[d], 0, 0, 0);
            }
        buf ^= 1;
    }
    wait_vmcnt<0>();
    __syncthreads();                                                 // every wave is done with its tiles

    // Merge the four partial results: lane L of every wave owns the same (query, d) positions.
    float *mo = reinterpret_cast<float *>(smem);                     // [wave][lane][64] unnormalised O
    float *ms = reinterpret_cast<float *>(smem + 4 * 64 * 64 * 4);   // [wave][lane][2]   m, l (both half-lanes summed)
    const float l_pair = l_run + __shfl_xor(l_run, 32);
    if (wave > 0) {
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                mo[(wave * 64 + lane) * 64 + d * 16 + e] = oacc[d][e];
        ms[(wave * 64 + lane) * 2 + 0] = m_run;
        ms[(wave * 64 + lane) * 2 + 1] = l_pair;
    }
    __syncthreads();
    if (wave == 0) {
        float m_all = m_run;
#pragma unroll
        for (int w = 1; w < 4; ++w)
            m_all = fmaxf(m_all, ms[(w * 64 + lane) * 2 + 0]);
        const float f0 = exp2f(m_run - m_all);                       // wave 0 always has a tile: m_all is finite
        float l_all = l_pair * f0;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                oacc[d][e] *= f0;
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float fw = exp2f(ms[(w * 64 + lane) * 2 + 0] - m_all);   // 0 for a wave that saw no key
            l_all += ms[(w * 64 + lane) * 2 + 1] * fw;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    oacc[d][e] += mo[(w * 64 + lane) * 64 + d * 16 + e] * fw;
        }
        if (q_ok) {
            const float inv = 1.0f / l_all;
            __bf16 *orow = static_cast<__bf16 *>(P.out) + ((size_t)b * P.c + qi) * P.ldo + (size_t)head * DH;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4_t h;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        h[e] = (__bf16)(oacc[d][4 * g + e] * inv);
                    *reinterpret_cast<u32x2_t *>(orow + d * 32 + 8 * g + 4 * lh) = __builtin_bit_cast(u32x2_t, h);
                }
        }
    }
}

}  // namespace

bool attn_slice_supported(const AttnParams &p)
{
    return p.head_dim == DH && p.S > 0 && p.c > 0 && p.heads > 0 && p.batch > 0 &&
           (int64_t)p.S * DH * 2 < ((int64_t)1 << 31);
}

hipError_t launch_attn_slice(const AttnParams &p_in, hipStream_t s, int num_cu)
{
    // One workgroup = NW waves of 32 queries sharing the key tiles.  Slices with few queries (the per-step grids
    // of Alg. 4 are small) leave most of the chip idle that way: then the keys are split as well -- over
    // several workgroups per query block if a workspace is registered, else over the waves of 32-query
    // workgroups.
    AttnParams p = p_in;
    int qt = 1, nw = 8, ksp = 0;
    bool wave_split = false;
    const Tuning tn = tuning();                          // overrides
    if (tn.attn_waves)                                   // waves per workgroup, 4 or 8
        nw = tn.attn_waves;
    if (tn.attn_ksplit)                                  // workgroups per query block
        ksp = tn.attn_ksplit;
    if (tn.attn_qt >= 0) {                               // 32-query tiles per wave; 0 = keys over waves
        wave_split = tn.attn_qt == 0;
        qt = tn.attn_qt == 2 ? 2 : 1;
        if (qt == 2)
            nw = 4;
    }
    if (p.n_slices < 1)
        p.n_slices = 1;
    if (p.n_slices > 1)
        wave_split = false;                            // several slices per launch: the query-block kernel only
    const int bq = nw * 32 * qt;
    const int64_t groups = (int64_t)((p.c + bq - 1) / bq) * p.heads * p.batch * p.n_slices;
    const bool small_grid = groups * 4 < (int64_t)num_cu * 3;
    p.ksplit = 1;
    if (!wave_split && qt == 1 && (small_grid || ksp > 1) && p.ws != nullptr && p.counters != nullptr) {
        const int nkt = (p.S + BKV - 1) / BKV;
        int k = ksp > 0 ? ksp : (int)((num_cu + groups - 1) / groups);   // one workgroup per compute unit
        k = k > 16 ? 16 : k;
        k = k > nkt ? nkt : k;
        const size_t need = (size_t)groups * k * (64 + 2) * (64 * nw) * sizeof(float);
        if (k > 1 && need <= p.ws_bytes && groups <= p.max_groups)
            p.ksplit = k;
    }
    if (wave_split || (small_grid && p.ksplit == 1 && qt == 1 && p.n_slices == 1 && tn.attn_qt < 0)) {
        const dim3 grid(((p.c + 31) / 32) * p.heads * p.batch), block(256);
        hipLaunchKernelGGL(attn_slice_ksplit_kernel, grid, block, 0, s, p);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(groups * p.ksplit)), block(64 * nw);
    if (qt == 2)
        hipLaunchKernelGGL((attn_slice_kernel<2, 4>), grid, block, 0, s, p);
    else if (nw == 8)
        hipLaunchKernelGGL((attn_slice_kernel<1, 8>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((attn_slice_kernel<1, 4>), grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace cf

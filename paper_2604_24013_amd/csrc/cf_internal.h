// Internal declarations shared by the translation units of libcommfuse.so.
// Nothing here is part of the C ABI (that is include/commfuse.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {

// One chunk GEMM: out[M x N] = A[M x K] * W (+ recv), fp32 accumulation.
// A points at the first row of the slice; W is [K x N] (w_kn) or [N x K].
// With a_t the left operand is given transposed, as [K x M] with row stride lda (the weight-gradient
// contraction over tokens: both operands then have the contraction index as their row index).
struct GemmParams {
    bool a_t = false;    // direct-to-LDS bf16 kernel, w_kn, fp32 output only
    const void *A = nullptr;
    const void *W = nullptr;
    const float *recv = nullptr;   // nullable: B_in of Alg. 2
    // further received partials, added after `recv` in index order before the product is added
    // (pairwise schedule with the aggregation deferred to the last step; direct-to-LDS bf16 kernel only)
    static constexpr int MAX_RECV_MORE = 15;
    const float *recv_more[MAX_RECV_MORE] = {};
    int n_recv_more = 0;
    int pf_lead = 16;    // B_in prefetch: k-tiles before the end of the k loop at which it is issued (0 = off)
    bool stream_recv = true;   // 256x256 tile: B_in lands in LDS under the main loop and is added in mid-sum (set by the launcher)
    void *out = nullptr;
    int64_t lda = 0, ldw = 0, ldo = 0;
    int M = 0, N = 0, K = 0;
    // split-K workspace (direct-to-LDS bf16 kernel only): partial tiles and per-tile arrival counters
    float *ws = nullptr;
    unsigned *counters = nullptr;
    size_t ws_bytes = 0;
    int max_tiles = 0;
    int splits = 1;
    // optional delivery carried by extra workgroups of the same launch (direct-to-LDS bf16 kernel only):
    // cp_bytes (a multiple of 16) from cp_src to cp_dst, both 16-byte aligned, by cp_wgs workgroups
    // optional device-side wait (direct-to-LDS bf16 kernel only): the kernel waits, with a bounded spin,
    // until *wait_flag != 0 before it first touches the delivered buffer (the slice for an all-gather
    // step, B_in for a reduce-scatter step); on time-out it sets bit 0 of *status and carries on
    const unsigned *wait_flag = nullptr;
    unsigned *status = nullptr;
    unsigned spin_limit = 0;
    bool wait_at_start = false;   // true: before the first operand load; false: before the B_in loads
    // persistent mode (direct-to-LDS bf16 kernel only): n_steps > 0 makes one launch run that many chunk GEMMs
    // of the same shape, step s with its own left operand, B_in, output and delivery flag (each nullable as
    // above); A, recv, out and wait_flag are then ignored
    static constexpr int MAX_STEPS = 16;
    int n_steps = 0;
    int num_cu = 256;
    bool k_rotate = false;   // persistent mode: XCD x starts its k loops x/8 of the way into the k range (set by the launcher)
    bool xcd_steps = false;  // persistent mode: XCD x runs steps x, x+8, ... whole (set by the launcher)
    int xcd_bands = 1;       // ... or, > 1: 8 / xcd_bands step groups x xcd_bands bands of tile columns (set by the launcher)
    bool mfma16 = false;     // persistent mode, 256x256 tile: main loop on v_mfma_f32_16x16x32_bf16 (set by the launcher)
    const void *A_step[MAX_STEPS] = {};
    const float *recv_step[MAX_STEPS] = {};
    void *out_step[MAX_STEPS] = {};
    const unsigned *flag_step[MAX_STEPS] = {};
    // the delivery carried by the consumer (persistent launch).  Reduce-scatter (256x256 tile with B_in through LDS):
    // recv_step[s] points at what the neighbour sends (its buffer, not this rank's landing buffer), and the
    // waves that add B_in also store it to land_step[s], the landing buffer.  All-gather: A_step[s] points at the
    // neighbour's buffer, and every k-tile of the slice that comes in through LDS is stored on to land_step[s]
    // (same layout as A_step[s]) by one of the workgroups that load it.  Either way the emulated transfer happens
    // inside the kernel, under its main loop.  Null = the operand is already where recv_step[s] / A_step[s] points.
    void *land_step[MAX_STEPS] = {};
    // Pairwise schedule, the deliveries carried by the launch: every work item of step s, once its own output tile is
    // stored, copies that tile's part of tail_src[s] (the arrival that travels while step s computes, in the sender's
    // buffer) to tail_dst[s] (its landing buffer; both laid out like the output), written through to memory, and then
    // counts tile_ready[tile] up.  The last step's work item waits (bounded by spin_limit; a time-out sets bit 0 of
    // *status) until its tile's count reaches ready_count, then reads recv_step / recv_more -- the landing buffers --
    // past the caches.  tile_ready holds max_tiles words, all zero at launch.  With tile_ready == nullptr nothing is
    // counted and nobody waits: a reduce-scatter step whose B_in is loaded in its epilogue (recv_step[s] = the sender's
    // buffer) lands that same B_in beside its GEMM this way (tail_src[s] = recv_step[s]).
    const float *tail_src[MAX_STEPS] = {};
    float *tail_dst[MAX_STEPS] = {};
    unsigned *tile_ready = nullptr;
    int ready_count = 0;
    const void *cp_src = nullptr;
    void *cp_dst = nullptr;
    size_t cp_bytes = 0;
    int cp_wgs = 0;
};

// Attention of one query slice (Alg. 4): out[(b, s) x (head, d)] = softmax(scale * Q_l K^T) V per (b, head).
// Q, K, V are [batch, heads, S, head_dim] bf16, contiguous; out is bf16 with row stride ldo elements.
struct AttnParams {
    const void *Q, *K, *V;
    void *out;
    int batch, heads, S, head_dim;
    int c;               // queries of the slice per batch element (S / N)
    int l;               // slice index: queries [l*c, (l+1)*c)
    int64_t ldo;
    float scale;
    // several slices in one launch (the 128/256-query kernel only): slices l, l+1, ..., l+n_slices-1, the output
    // of slice l+i starting out_slice_stride elements after that of slice l+i-1
    int n_slices = 1;
    int64_t out_slice_stride = 0;
    // key split across workgroups (the 128-query kernel): the key tiles are divided over `ksplit` workgroups per
    // query block, which park (m, l, unnormalised O) in the workspace; the last one to finish merges them
    int ksplit = 1;
    float *ws = nullptr;
    unsigned *counters = nullptr;
    size_t ws_bytes = 0;
    int max_groups = 0;
};

// Tuning overrides (environment variables COMMFUSE_*; tests use them to force every code path).  They are read
// ONCE, at the first call into the library -- unless COMMFUSE_TUNING_LIVE is set to a non-zero value at that
// moment, in which case every call of tuning() reads the environment again (test mode).  A field keeps its
// "unset" value when its variable is absent.  The struct is plain data: it is part of the key under which a
// captured graph is cached, because the choices are baked into the captured launches.
struct Tuning {
    int tile_bm = 0, tile_bn = 0;   // COMMFUSE_TILE = "256x256" | "256x128" | "128x128"   (0 = unset)
    int deep = -1;                  // COMMFUSE_DEEP = 0 | 1                               (-1 = unset)
    int splitk = 0;                 // COMMFUSE_SPLITK = 1..8                              (0 = unset)
    int staged = 0;                 // COMMFUSE_KERNEL = "staged"
    int prefetch = -1;              // COMMFUSE_PREFETCH = lead of the B_in prefetch in k-tiles (-1 = unset)
    int xcd_steps = -1;             // COMMFUSE_XCD_STEPS = 0 | 1                          (-1 = unset)
    int k_rotate = -1;              // COMMFUSE_K_ROTATE = 0 | 1                           (-1 = unset)
    int xcd_bands = 0;              // COMMFUSE_XCD_BANDS = 1 | 2 | 4: column bands per step group (0 = unset: by shape)
    int stream_recv = -1;           // COMMFUSE_STREAM_RECV = 0 | 1                        (-1 = unset)
    int mfma16 = -1;                // COMMFUSE_MFMA16 = 0 | 1: 16x16x32 MFMAs in the 256x256 persistent kernel (-1 = unset)
    int persist_wgs = 0;            // COMMFUSE_PERSIST_WGS = cap on the persistent kernel's grid (0 = unset)
    int carry = -1;                 // COMMFUSE_CARRY = 0: the one-launch reduce-scatter never carries its deliveries
                                    // under CF_FUSED_COPY (-1 = unset, 1: wherever the launch streams B_in)
    int tile_f32_bm = 0;            // COMMFUSE_TILE_F32 = "128x128" | "64x64"             (0 = unset)
    unsigned spin_limit = 0;        // COMMFUSE_SPIN_LIMIT                                 (0 = unset)
    int attn_qt = -1;               // COMMFUSE_ATTN_QT = 0 | 1 | 2                        (-1 = unset)
    int attn_waves = 0;             // COMMFUSE_ATTN_WAVES = 4 | 8                         (0 = unset)
    int attn_ksplit = 0;            // COMMFUSE_ATTN_KSPLIT                                (0 = unset)
};
Tuning tuning();

struct TileChoice {
    int bm, bn;          // workgroup tile
    int splitk;          // k-splits per output tile (1 = none)
    bool deep = false;   // 128x128 only: four LDS stages, one workgroup per CU
};

// Chooses the workgroup tile for a chunk GEMM from its shape and the number of
// compute units (the per-step grids are small against 256 CUs).
TileChoice choose_tile_bf16(int M, int N, int K, int num_cu);

hipError_t launch_gemm_bf16(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s, int num_cu);
// True if launch_gemm_bf16 would run the kernel that honours GemmParams::recv_more for these operands.
bool gemm_bf16_takes_recv_list(const GemmParams &p, bool w_kn);
// Output tiles per step if launch_gemm_bf16 can run this persistent launch with GemmParams::tail_src / tile_ready (the
// arrivals of the pairwise schedule landed by the work items of the steps before the one that sums them), else 0.
// The caller provides that many zeroed counters.
int gemm_bf16_tiles_landing_arrivals(const GemmParams &p, bool w_kn, int num_cu);
// True if a persistent reduce-scatter launch that does NOT stream B_in (gemm_bf16_carries_delivery says no) can still
// carry its deliveries: B_in read from the sender's buffer in the epilogue and landed by the same work item beside
// its GEMM (GemmParams::tail_src without counters).  fp32 partial sums, direct-to-LDS kernel.
bool gemm_bf16_lands_beside(const GemmParams &p, bool w_kn, bool out_bf16, int num_cu);
// True if launch_gemm_bf16 would run this persistent launch (reduce_scatter: its steps add a received partial;
// else an all-gather's) on a kernel that honours GemmParams::land_step (the delivery carried by the consumer)
// for every step that receives.
bool gemm_bf16_carries_delivery(const GemmParams &p, bool w_kn, bool out_bf16, int num_cu, bool reduce_scatter);
// Steps per launch when a persistent rank step of p.n_steps steps is cut into launches that fill the chip about once
// each (equal groups; p.n_steps when the whole rank step is one round or less).
int gemm_bf16_steps_per_launch(const GemmParams &p, bool w_kn, int num_cu);
// Direct-to-LDS variant of the bf16 kernel (operand extents below 2^31 bytes).
bool gemm_bf16_dl_supported(const GemmParams &p, bool w_kn);
hipError_t launch_gemm_bf16_dl(const GemmParams &p, bool w_kn, bool out_bf16, hipStream_t s, TileChoice t);
bool gemm_bf16_dl_streams_recv(const GemmParams &p, bool w_kn, bool out_bf16, TileChoice t);
bool gemm_bf16_dl_carries_operand(const GemmParams &p);
hipError_t launch_gemm_f32(const GemmParams &p, bool w_kn, hipStream_t s, int num_cu);

bool attn_slice_supported(const AttnParams &p);
hipError_t launch_attn_slice(const AttnParams &p, hipStream_t s, int num_cu);

// dst[e] += src[e], e in [0, n)
// (land: nullable -- what is read from src is also stored there, the delivery carried by the consumer)
hipError_t launch_dp_reduce(float *dst, const float *src, int64_t n, hipStream_t s, int num_cu, float *land = nullptr);
// dst <- (((dst + src[0]) + src[1]) + ...) over n elements, one pass when all pointers are 16-byte aligned and
// n_src <= 15 (else one pass per source: same additions, same order, same bits)
hipError_t launch_dp_reduce_multi(float *dst, const float *const *src, int n_src, int64_t n, hipStream_t s, int num_cu,
                                  float *const *land = nullptr);
// n (<= 16) copies of `bytes` bytes each in one launch; copy_batch_takes says whether the arguments qualify
// (16-byte aligned pointers, bytes a multiple of 16), else the caller copies one by one
bool copy_batch_takes(const void *const *src, void *const *dst, int n, size_t bytes);
hipError_t launch_copy_batch(const void *const *src, void *const *dst, int n, size_t bytes, hipStream_t s);

// Writes `value` to each of dst[0..count) with device-coherent stores (flags polled by other kernels).
hipError_t launch_set_words(unsigned *dst, int count, unsigned value, hipStream_t s);

// Fills a buffer with 0xFF bytes (a NaN pattern for fp32 and bf16) -- debug poison.
hipError_t launch_fill_ff(void *dst, size_t bytes, hipStream_t s);

}  // namespace cf

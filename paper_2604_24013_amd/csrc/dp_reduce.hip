// Data-parallel gradient path: one ring step of Alg. 2 with the identity as
// compute_partial_output, i.e. "O <- B_in + O" on one slice of the local fp32
// gradient bucket, in place.  HBM-bound: 12 bytes per element (read slice, read
// B_in, write slice).  16-byte accesses, several independent loads in flight
// per lane, one pass over the slice.  A variant also carries the emulated delivery:
// B_in is read from the neighbour's buffer and stored on to the landing buffer in the
// same pass (16 bytes per element instead of a copy's 8 plus the add's 12).
#include "cf_internal.h"

namespace cf {
namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int DP_THREADS = 256;
constexpr int DP_UNROLL = 4;

// LAND: the delivery carried by the consumer -- src is the neighbour's buffer, and what is read from it is also stored
// to `land`, this rank's landing buffer: 16 bytes per element (two reads, two writes) where a copy followed by the add
// moves 20.
template <bool LAND>
__global__ __launch_bounds__(DP_THREADS) void dp_reduce_vec_kernel(f32x4_t *__restrict__ dst,
                                                                  const f32x4_t *__restrict__ src, int64_t n4,
                                                                  f32x4_t *__restrict__ land)
{
    // Every element is touched exactly once: all streams bypass the caches' retention
    // (non-temporal), which measured ~25% faster than cached accesses on MI355X.
    const int64_t stride = (int64_t)gridDim.x * DP_THREADS;
    int64_t i = (int64_t)blockIdx.x * DP_THREADS + threadIdx.x;
    for (; i + (DP_UNROLL - 1) * stride < n4; i += DP_UNROLL * stride) {
        f32x4_t a[DP_UNROLL], b[DP_UNROLL];
#pragma unroll
        for (int u = 0; u < DP_UNROLL; ++u) {
            a[u] = __builtin_nontemporal_load(&dst[i + u * stride]);
            b[u] = __builtin_nontemporal_load(&src[i + u * stride]);
        }
#pragma unroll
        for (int u = 0; u < DP_UNROLL; ++u) {
            __builtin_nontemporal_store(b[u] + a[u], &dst[i + u * stride]);   // "O <- B_in + O"
            if constexpr (LAND)
                __builtin_nontemporal_store(b[u], &land[i + u * stride]);
        }
    }
    for (; i < n4; i += stride) {
        const f32x4_t b = __builtin_nontemporal_load(&src[i]);
        __builtin_nontemporal_store(b + __builtin_nontemporal_load(&dst[i]), &dst[i]);
        if constexpr (LAND)
            __builtin_nontemporal_store(b, &land[i]);
    }
}

__global__ __launch_bounds__(DP_THREADS) void dp_reduce_scalar_kernel(float *__restrict__ dst,
                                                                     const float *__restrict__ src, int64_t n,
                                                                     float *__restrict__ land)
{
    const int64_t stride = (int64_t)gridDim.x * DP_THREADS;
    for (int64_t i = (int64_t)blockIdx.x * DP_THREADS + threadIdx.x; i < n; i += stride) {
        const float b = src[i];
        dst[i] = b + dst[i];
        if (land != nullptr)
            land[i] = b;
    }
}

// dst <- (((dst + src[0]) + src[1]) + ...) in ONE pass: the pairwise gradient reduce, where every round's arrival
// is added to the same slice.  4 (n + 2) bytes per element instead of 12 n for n separate passes; the additions
// are taken in the order of the separate passes, so the result is the same bit for bit.
struct AddBatch {
    static constexpr int MAX = 15;
    const float *src[MAX];
};

// LAND: as above -- source s is also stored to land[s].
template <bool LAND>
__global__ __launch_bounds__(DP_THREADS) void dp_reduce_multi_kernel(f32x4_t *__restrict__ dst, AddBatch ab, int n_src,
                                                                    int64_t n4, AddBatch lb)
{
    constexpr int U = 2;                             // vectors per lane: (n_src + 1) * U loads in flight
    const int64_t base = (int64_t)blockIdx.x * DP_THREADS * U + threadIdx.x;
    f32x4_t a[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (base + u * DP_THREADS < n4)
            a[u] = __builtin_nontemporal_load(&dst[base + u * DP_THREADS]);
    for (int s = 0; s < n_src; ++s) {
        const f32x4_t *__restrict__ src = reinterpret_cast<const f32x4_t *>(ab.src[s]);
        f32x4_t *__restrict__ land = reinterpret_cast<f32x4_t *>(const_cast<float *>(lb.src[s]));
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u * DP_THREADS < n4) {
                const f32x4_t b = __builtin_nontemporal_load(&src[base + u * DP_THREADS]);
                a[u] = b + a[u];
                if constexpr (LAND)
                    __builtin_nontemporal_store(b, &land[base + u * DP_THREADS]);
            }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (base + u * DP_THREADS < n4)
            __builtin_nontemporal_store(a[u], &dst[base + u * DP_THREADS]);
}

__global__ __launch_bounds__(DP_THREADS) void dp_reduce_multi_scalar_kernel(float *__restrict__ dst, AddBatch ab, int n_src,
                                                                           int64_t first, int64_t n, AddBatch lb, bool land)
{
    const int64_t stride = (int64_t)gridDim.x * DP_THREADS;
    for (int64_t i = first + (int64_t)blockIdx.x * DP_THREADS + threadIdx.x; i < n; i += stride) {
        float a = dst[i];
        for (int s = 0; s < n_src; ++s) {
            const float b = ab.src[s][i];
            a = b + a;
            if (land)
                const_cast<float *>(lb.src[s])[i] = b;
        }
        dst[i] = a;
    }
}

// Several equally long device-to-device copies in ONE launch (the deliveries of a whole rank step when they are
// all enqueued in front of the persistent kernel): workgroup b moves chunk b % per_buf of buffer b / per_buf,
// 16 bytes per lane and access, four independent vectors in flight, non-temporal both ways like the reduce above.
struct CopyBatch {
    static constexpr int MAX = 16;
    const void *src[MAX];
    void *dst[MAX];
};

__global__ __launch_bounds__(DP_THREADS) void copy_batch_kernel(CopyBatch cb, int64_t n16, int per_buf)
{
    const int buf = blockIdx.x / per_buf, chunk = blockIdx.x % per_buf;
    const f32x4_t *__restrict__ src = static_cast<const f32x4_t *>(cb.src[buf]);
    f32x4_t *__restrict__ dst = static_cast<f32x4_t *>(cb.dst[buf]);
    const int64_t base = (int64_t)chunk * DP_THREADS * DP_UNROLL + threadIdx.x;
    f32x4_t v[DP_UNROLL];
#pragma unroll
    for (int u = 0; u < DP_UNROLL; ++u)
        if (base + u * DP_THREADS < n16)
            v[u] = __builtin_nontemporal_load(&src[base + u * DP_THREADS]);
#pragma unroll
    for (int u = 0; u < DP_UNROLL; ++u)
        if (base + u * DP_THREADS < n16)
            __builtin_nontemporal_store(v[u], &dst[base + u * DP_THREADS]);
}

__global__ __launch_bounds__(64) void set_words_kernel(unsigned *dst, int count, unsigned value)
{
    for (int i = threadIdx.x; i < count; i += 64)
        __hip_atomic_store(&dst[i], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(256) void fill_ff_kernel(unsigned *dst, size_t nwords)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nwords; i += stride)
        dst[i] = 0xFFFFFFFFu;
}

}  // namespace

hipError_t launch_dp_reduce(float *dst, const float *src, int64_t n, hipStream_t s, int num_cu, float *land)
{
    if (n <= 0)
        return hipSuccess;
    const bool aligned = ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) |
                           reinterpret_cast<uintptr_t>(land)) & 15u) == 0;
    const int64_t n4 = aligned ? n / 4 : 0;
    if (n4 > 0) {
        // one workgroup per DP_THREADS * DP_UNROLL vectors: a grid that covers the slice once measured
        // faster than a grid-stride loop over a chip-sized grid (5.9 vs 4.4 TB/s at 125M elements)
        int64_t want = (n4 + (int64_t)DP_THREADS * DP_UNROLL - 1) / ((int64_t)DP_THREADS * DP_UNROLL);
        const int64_t cap = (int64_t)1 << 30;
        (void)num_cu;
        const int blocks = (int)(want < cap ? want : cap);
        if (land != nullptr)
            hipLaunchKernelGGL(dp_reduce_vec_kernel<true>, dim3(blocks), dim3(DP_THREADS), 0, s, reinterpret_cast<f32x4_t *>(dst),
                               reinterpret_cast<const f32x4_t *>(src), n4, reinterpret_cast<f32x4_t *>(land));
        else
            hipLaunchKernelGGL(dp_reduce_vec_kernel<false>, dim3(blocks), dim3(DP_THREADS), 0, s, reinterpret_cast<f32x4_t *>(dst),
                               reinterpret_cast<const f32x4_t *>(src), n4, static_cast<f32x4_t *>(nullptr));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
    }
    const int64_t done = n4 * 4;
    if (done < n) {
        const int64_t rest = n - done;
        int64_t want = (rest + DP_THREADS - 1) / DP_THREADS;
        const int64_t cap = (int64_t)num_cu * 8;
        const int blocks = (int)(want < cap ? want : cap);
        hipLaunchKernelGGL(dp_reduce_scalar_kernel, dim3(blocks), dim3(DP_THREADS), 0, s, dst + done, src + done, rest,
                           land != nullptr ? land + done : nullptr);
        return hipGetLastError();
    }
    return hipSuccess;
}

hipError_t launch_dp_reduce_multi(float *dst, const float *const *src, int n_src, int64_t n, hipStream_t s, int num_cu,
                                  float *const *land)
{
    if (n <= 0 || n_src <= 0)
        return hipSuccess;
    uintptr_t bits = reinterpret_cast<uintptr_t>(dst);
    for (int i = 0; i < n_src; ++i)
        bits |= reinterpret_cast<uintptr_t>(src[i]) | (land != nullptr ? reinterpret_cast<uintptr_t>(land[i]) : 0);
    if (n_src > AddBatch::MAX || (bits & 15u) != 0) {        // one pass per source: the same additions in the same order
        for (int i = 0; i < n_src; ++i) {
            hipError_t e = launch_dp_reduce(dst, src[i], n, s, num_cu, land != nullptr ? land[i] : nullptr);
            if (e != hipSuccess)
                return e;
        }
        return hipSuccess;
    }
    AddBatch ab = {}, lb = {};
    for (int i = 0; i < n_src; ++i) {
        ab.src[i] = src[i];
        lb.src[i] = land != nullptr ? land[i] : nullptr;
    }
    const int64_t n4 = n / 4;
    if (n4 > 0) {
        const int64_t per_wg = (int64_t)DP_THREADS * 2;
        const int64_t want = (n4 + per_wg - 1) / per_wg;
        if (want >= ((int64_t)1 << 31))
            return hipErrorInvalidValue;
        if (land != nullptr)
            hipLaunchKernelGGL(dp_reduce_multi_kernel<true>, dim3((unsigned)want), dim3(DP_THREADS), 0, s,
                               reinterpret_cast<f32x4_t *>(dst), ab, n_src, n4, lb);
        else
            hipLaunchKernelGGL(dp_reduce_multi_kernel<false>, dim3((unsigned)want), dim3(DP_THREADS), 0, s,
                               reinterpret_cast<f32x4_t *>(dst), ab, n_src, n4, lb);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
    }
    if (n4 * 4 < n) {
        hipLaunchKernelGGL(dp_reduce_multi_scalar_kernel, dim3(1), dim3(DP_THREADS), 0, s, dst, ab, n_src, n4 * 4, n, lb,
                           land != nullptr);
        return hipGetLastError();
    }
    return hipSuccess;
}

bool copy_batch_takes(const void *const *src, void *const *dst, int n, size_t bytes)
{
    if (n < 1 || n > CopyBatch::MAX || bytes == 0 || bytes % 16 != 0)
        return false;
    const int64_t per_buf = (int64_t)((bytes / 16 + (size_t)DP_THREADS * DP_UNROLL - 1) / ((size_t)DP_THREADS * DP_UNROLL));
    if (per_buf * n >= ((int64_t)1 << 31))
        return false;
    for (int i = 0; i < n; ++i)
        if (((reinterpret_cast<uintptr_t>(src[i]) | reinterpret_cast<uintptr_t>(dst[i])) & 15u) != 0)
            return false;
    return true;
}

hipError_t launch_copy_batch(const void *const *src, void *const *dst, int n, size_t bytes, hipStream_t s)
{
    CopyBatch cb = {};
    for (int i = 0; i < n; ++i) {
        cb.src[i] = src[i];
        cb.dst[i] = dst[i];
    }
    const int64_t n16 = (int64_t)(bytes / 16);
    const int per_buf = (int)((n16 + (int64_t)DP_THREADS * DP_UNROLL - 1) / ((int64_t)DP_THREADS * DP_UNROLL));
    hipLaunchKernelGGL(copy_batch_kernel, dim3((unsigned)(per_buf * n)), dim3(DP_THREADS), 0, s, cb, n16, per_buf);
    return hipGetLastError();
}

hipError_t launch_set_words(unsigned *dst, int count, unsigned value, hipStream_t s)
{
    if (count <= 0)
        return hipSuccess;
    hipLaunchKernelGGL(set_words_kernel, dim3(1), dim3(64), 0, s, dst, count, value);
    return hipGetLastError();
}

hipError_t launch_fill_ff(void *dst, size_t bytes, hipStream_t s)
{
    const size_t nwords = bytes / 4;
    if (nwords == 0)
        return hipSuccess;
    size_t want = (nwords + 255) / 256;
    const int blocks = (int)(want < 2048 ? want : 2048);
    hipLaunchKernelGGL(fill_ff_kernel, dim3(blocks), dim3(256), 0, s, static_cast<unsigned *>(dst), nwords);
    return hipGetLastError();
}

}  // namespace cf

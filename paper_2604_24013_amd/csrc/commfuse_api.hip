// C ABI of libcommfuse.so: argument checking, slice selection (the index lines
// of Alg. 1 and Alg. 2), kernel dispatch, and the two-stream emulated rank step.
// The contract of every entry point is stated in include/commfuse.h.
#include "../../include/commfuse.h"
#include "cf_internal.h"

#include <climits>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <unordered_map>
#include <vector>

namespace {

thread_local char g_err[512] = "";

cf_status fail(cf_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

cf_status fail_hip(hipError_t e, const char *what)
{
    return fail(CF_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define CF_HIP(call)                         \
    do {                                     \
        hipError_t e_ = (call);              \
        if (e_ != hipSuccess)                \
            return fail_hip(e_, #call);      \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int num_cu_of_current_device()
{
    static std::mutex mu;
    static int cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return 256;
    std::lock_guard<std::mutex> lk(mu);
    if (cache[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cache[dev] = n;
    }
    return cache[dev];
}

// Caller-owned split-K workspace (commfuse_set_workspace): [0, WS_COUNTER_BYTES) arrival counters,
// the rest fp32 partial tiles.
constexpr size_t WS_COUNTER_BYTES = 64 * 1024;
constexpr size_t WS_TILE_COUNTER_BYTES = 60 * 1024;   // split-K arrival counters
constexpr size_t WS_FLAG_OFFSET = 60 * 1024;          // delivery flags (CF_DEVICE_WAIT): one word per step
constexpr int WS_MAX_FLAGS = 512;
constexpr size_t WS_STATUS_OFFSET = 63 * 1024;        // one status word (bit 0: a device-side wait timed out)
constexpr int WS_MAX_SPLITS = 8;
struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
};
std::mutex g_ws_mu;
Workspace g_ws;                                              // registered without a stream: serves every stream ...
std::unordered_map<hipStream_t, Workspace> g_ws_of_stream;   // ... that has no registration of its own

// The workspace the work enqueued on stream `s` uses.
Workspace workspace_for(hipStream_t s)
{
    std::lock_guard<std::mutex> lk(g_ws_mu);
    if (s != nullptr) {
        auto it = g_ws_of_stream.find(s);
        if (it != g_ws_of_stream.end())
            return it->second;
    }
    return g_ws;
}

// Scratch of commfuse_rs_step_noalloc: the same layout as a registered workspace (arrival counters, then fp32
// partial tiles), but owned by the library, in device memory that exists from the moment the code object is
// loaded.  Every GPU the library runs on holds its own copy of the array until the process ends.  In host
// code the array's name only stands for the symbol; the device address is looked up once per device
// (static_scratch_of_current_device) and everything below uses that pointer.
constexpr size_t STATIC_PARTIAL_BYTES = (size_t)64 << 20;                       // 8 k-splits of 2^21 fp32 elements
constexpr size_t STATIC_SCRATCH_BYTES = WS_COUNTER_BYTES + STATIC_PARTIAL_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

struct Resolved {      // descriptor with defaults filled in
    int p, rank;
    int m;             // slicing granularity: sub-steps per ring hop
    int64_t mc;        // rows one (sub-)step works on: m_chunk / m
    int64_t n, k, lda, ldw, ldo;
    bool bf16_in, bf16_out, w_kn;
};

bool is_pair_kind(int kind) { return kind == CF_KIND_RS_PAIR || kind == CF_KIND_DP_PAIR; }
bool is_dp_kind(int kind) { return kind == CF_KIND_DP || kind == CF_KIND_DP_PAIR; }
bool is_rs_kind(int kind) { return kind == CF_KIND_RS || kind == CF_KIND_RS_PAIR; }
bool known_kind(int kind) { return kind >= CF_KIND_RS && kind <= CF_KIND_WGRAD_G; }
bool is_wgrad_kind(int kind) { return kind == CF_KIND_WGRAD_X || kind == CF_KIND_WGRAD_G; }

size_t in_elem(const Resolved &r) { return r.bf16_in ? 2 : 4; }

cf_status resolve(const cf_layer_desc *d, int kind, Resolved *out)
{
    if (d == nullptr)
        return fail(CF_ERR_NULL_PTR, "descriptor is NULL");
    if (d->p < 1)
        return fail(CF_ERR_INVALID_ARG, "p = %d must be >= 1", d->p);
    if (d->rank < 0 || d->rank >= d->p)
        return fail(CF_ERR_INVALID_ARG, "rank = %d not in [0, %d)", d->rank, d->p);
    if (d->m_chunk < 0 || d->n < 0 || d->k < 0)
        return fail(CF_ERR_INVALID_ARG, "negative size (m_chunk=%lld n=%lld k=%lld)", (long long)d->m_chunk,
                    (long long)d->n, (long long)d->k);
    if (d->m < 0 || d->m > 4096)
        return fail(CF_ERR_INVALID_ARG, "slicing granularity m = %d not in [0, 4096]", d->m);
    Resolved r;
    r.p = d->p;
    r.rank = d->rank;
    r.m = d->m > 1 ? d->m : 1;
    if (r.m > 1 && is_pair_kind(kind))
        return fail(CF_ERR_UNSUPPORTED, "the pairwise kinds need slicing granularity m = 1");
    if (d->m_chunk % r.m != 0)
        return fail(CF_ERR_INVALID_ARG, "m = %d must divide m_chunk = %lld", r.m, (long long)d->m_chunk);
    r.mc = d->m_chunk / r.m;
    r.n = d->n;
    r.k = d->k;
    if (is_dp_kind(kind)) {
        r.lda = r.ldw = r.ldo = 0;
        r.bf16_in = r.bf16_out = false;
        r.w_kn = true;
        *out = r;
        return CF_OK;
    }
    if (d->in_dtype != CF_BF16 && d->in_dtype != CF_F32)
        return fail(CF_ERR_UNSUPPORTED, "in_dtype %d", d->in_dtype);
    if (d->out_dtype != CF_BF16 && d->out_dtype != CF_F32)
        return fail(CF_ERR_UNSUPPORTED, "out_dtype %d", d->out_dtype);
    if (d->w_layout != CF_W_KN && d->w_layout != CF_W_NK && !is_wgrad_kind(kind))
        return fail(CF_ERR_UNSUPPORTED, "w_layout %d", d->w_layout);
    r.bf16_in = d->in_dtype == CF_BF16;
    r.bf16_out = (kind == CF_KIND_AG) && d->out_dtype == CF_BF16;
    if (r.bf16_out && !r.bf16_in)
        return fail(CF_ERR_UNSUPPORTED, "bf16 output needs bf16 operands");
    r.w_kn = is_wgrad_kind(kind) || d->w_layout == CF_W_KN;   // both weight-gradient operands are [rows x .]
    if (d->lda < 0 || d->ldw < 0 || d->ldo < 0)
        return fail(CF_ERR_INVALID_ARG, "negative row stride");
    r.lda = d->lda ? d->lda : r.k;
    r.ldw = d->ldw ? d->ldw : (r.w_kn ? r.n : r.k);
    r.ldo = d->ldo ? d->ldo : r.n;
    if (r.lda < r.k || r.ldw < (r.w_kn ? r.n : r.k) || r.ldo < r.n)
        return fail(CF_ERR_INVALID_ARG, "row stride smaller than the row (lda=%lld ldw=%lld ldo=%lld)",
                    (long long)r.lda, (long long)r.ldw, (long long)r.ldo);
    const int64_t mult = r.bf16_in ? 8 : 4;
    if (r.k % mult || r.n % mult || r.lda % mult || r.ldw % mult || r.ldo % mult)
        return fail(CF_ERR_MISALIGNED, "k, n and row strides must be multiples of %lld elements", (long long)mult);
    const int64_t lim = INT_MAX / 2;
    if (d->m_chunk * r.p > lim || r.n > lim || r.k > lim)
        return fail(CF_ERR_INVALID_ARG, "size exceeds the 32-bit index range of the kernels");
    *out = r;
    return CF_OK;
}

int chunk_index(int kind, int p, int rank, int step)
{
    // Alg. 1: l = (r - i + N) mod N.   Alg. 2: l = (r - i - 1 + N) mod N.
    if (kind == CF_KIND_AG)
        return ((rank - step) % p + p) % p;
    return ((rank - step - 1) % p + p) % p;
}

// Granularity m: sub-step j = hop*m + s handles sub-slice l(hop)*m + s.
int subslice_index(int kind, int p, int m, int rank, int j) { return chunk_index(kind, p, rank, j / m) * m + j % m; }

// Appendix A(a): partner of `rank` in round t of the pairwise schedule (p even, t in [1, p-1]).
int pair_partner(int p, int rank, int t)
{
    if ((p & (p - 1)) == 0)
        return rank ^ t;                           // reproduces the appendix's four-device table
    const int a = t - 1;                           // circle method: rank p-1 fixed, the others rotate
    if (rank == p - 1)
        return a;
    if (rank == a)
        return p - 1;
    return ((2 * a - rank) % (p - 1) + (p - 1)) % (p - 1);
}

// Slice computed at step i of the pairwise schedule: what travels in round i+1 first, the own slice last.
int pair_slice(int p, int rank, int step) { return (step == p - 1) ? rank : pair_partner(p, rank, step + 1); }

cf_status check_pair_p(int p)
{
    if (p != 1 && (p & 1))
        return fail(CF_ERR_INVALID_ARG, "the pairwise schedule is defined for even p (or p = 1), not p = %d", p);
    return CF_OK;
}

cf_status check_step(const Resolved &r, int step)
{
    if (step < 0 || step >= r.p * r.m)
        return fail(CF_ERR_INVALID_ARG, "step = %d not in [0, %d)", step, r.p * r.m);
    return CF_OK;
}

// A delivery to be carried by extra workgroups of a step's launch (CF_FUSED_COPY).
struct CopyJob {
    const void *src = nullptr;
    void *dst = nullptr;
    size_t bytes = 0;
    const unsigned *wait_flag = nullptr;   // CF_DEVICE_WAIT: flag the step kernel waits on
    unsigned *status = nullptr;
    bool wait_at_start = false;
};

unsigned spin_limit()
{
    const unsigned v = cf::tuning().spin_limit;            // tests force a time-out with a tiny limit
    return v > 0 ? v : 400000u;                            // default: about a second of polling
}

// True if a step of this layer runs the kernel that can carry a delivery (direct-to-LDS bf16 kernel).
bool step_can_carry_copy(const Resolved &r)
{
    if (!r.bf16_in || r.mc <= 0 || r.n <= 0 || r.k <= 0)
        return false;
    const int64_t lim = (int64_t)1 << 31;
    return r.mc * r.lda * 2 < lim && (r.w_kn ? r.k : r.n) * r.ldw * 2 < lim && r.mc * r.ldo * 4 < lim;
}

void fill_shape(cf::GemmParams &gp, const Resolved &r)
{
    gp.lda = r.lda;
    gp.ldw = r.ldw;
    gp.ldo = r.ldo;
    gp.M = (int)r.mc;
    gp.N = (int)r.n;
    gp.K = (int)r.k;
}

bool wgrad_can_carry_copy(const Resolved &r)
{
    if (!r.bf16_in || r.mc <= 0 || r.n <= 0 || r.k <= 0)
        return false;
    const int64_t lim = (int64_t)1 << 31;
    return r.mc * r.lda * 2 < lim && r.mc * r.ldw * 2 < lim && r.k * r.ldo * 4 < lim;
}

cf_status launch_gemm(const Resolved &r, const void *A_rows, const void *W, const float *recv, void *out,
                      hipStream_t s, const CopyJob *job = nullptr, const float *const *recv_more = nullptr,
                      int n_recv_more = 0, const Workspace *ws_instead = nullptr)
{
    cf::GemmParams gp;
    for (int b = 0; b < n_recv_more; ++b)
        gp.recv_more[b] = recv_more[b];
    gp.n_recv_more = n_recv_more;
    gp.A = A_rows;
    gp.W = W;
    gp.recv = recv;
    gp.out = out;
    fill_shape(gp, r);
    {
        const Workspace ws = ws_instead != nullptr ? *ws_instead : workspace_for(s);   // (the library's own scratch, or the registered one)
        if (ws.ptr != nullptr && ws.bytes > WS_COUNTER_BYTES) {
            gp.counters = static_cast<unsigned *>(ws.ptr);
            gp.ws = reinterpret_cast<float *>(static_cast<char *>(ws.ptr) + WS_COUNTER_BYTES);
            gp.ws_bytes = ws.bytes - WS_COUNTER_BYTES;
            gp.max_tiles = (int)(WS_TILE_COUNTER_BYTES / sizeof(unsigned));
        }
    }
    const int ncu = num_cu_of_current_device();
    if (job != nullptr && job->wait_flag != nullptr) {
        gp.wait_flag = job->wait_flag;
        gp.status = job->status;
        gp.spin_limit = spin_limit();
        gp.wait_at_start = job->wait_at_start;
    }
    if (job != nullptr && job->bytes > 0) {
        gp.cp_src = job->src;
        gp.cp_dst = job->dst;
        gp.cp_bytes = job->bytes;
        gp.cp_wgs = ncu / 4;                       // 64 copy workgroups on a 256-CU part
    }
    hipError_t e = r.bf16_in ? cf::launch_gemm_bf16(gp, r.w_kn, r.bf16_out, s, ncu)
                             : cf::launch_gemm_f32(gp, r.w_kn, s, ncu);
    if (e != hipSuccess)
        return fail_hip(e, "chunk GEMM launch");
    return CF_OK;
}

cf_status rs_step_impl(const Resolved &r, int step, const void *A, const void *W, const float *recv, float *out,
                       hipStream_t s, const CopyJob *job = nullptr, const Workspace *ws_instead = nullptr)
{
    if (cf_status st = check_step(r, step))
        return st;
    if (A == nullptr || W == nullptr || out == nullptr)
        return fail(CF_ERR_NULL_PTR, "A, W and out must not be NULL");
    if (step < r.m && recv != nullptr)
        return fail(CF_ERR_NULL_PTR, "recv must be NULL in the first hop (nothing has been received yet)");
    if (step >= r.m && recv == nullptr)
        return fail(CF_ERR_NULL_PTR, "recv must not be NULL at step %d", step);
    if (recv == out)
        return fail(CF_ERR_INVALID_ARG, "out may not alias recv");
    if (!aligned16(A) || !aligned16(W) || !aligned16(out) || !aligned16(recv))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    const int l = subslice_index(CF_KIND_RS, r.p, r.m, r.rank, step);
    const char *a_rows = static_cast<const char *>(A) + (size_t)l * r.mc * r.lda * in_elem(r);
    return launch_gemm(r, a_rows, W, recv, out, s, job, nullptr, 0, ws_instead);
}

cf_status ag_step_impl(const Resolved &r, int step, const void *shard, const void *W, void *O, hipStream_t s,
                       const CopyJob *job = nullptr)
{
    if (cf_status st = check_step(r, step))
        return st;
    if (shard == nullptr || W == nullptr || O == nullptr)
        return fail(CF_ERR_NULL_PTR, "shard, W and O must not be NULL");
    if (!aligned16(shard) || !aligned16(W) || !aligned16(O))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    const int l = subslice_index(CF_KIND_AG, r.p, r.m, r.rank, step);
    char *o_rows = static_cast<char *>(O) + (size_t)l * r.mc * r.ldo * (r.bf16_out ? 2 : 4);
    return launch_gemm(r, shard, W, nullptr, o_rows, s, job);
}

// chunk_elems: elements per (sub-)step; m: sub-steps per hop
cf_status dp_step_impl(int p, int rank, int step, float *bucket, int64_t chunk_elems, const float *recv,
                       hipStream_t s, int m = 1, float *land = nullptr)
{
    if (p < 1)
        return fail(CF_ERR_INVALID_ARG, "p = %d must be >= 1", p);
    if (rank < 0 || rank >= p)
        return fail(CF_ERR_INVALID_ARG, "rank = %d not in [0, %d)", rank, p);
    if (step < 0 || step >= p * m)
        return fail(CF_ERR_INVALID_ARG, "step = %d not in [0, %d)", step, p * m);
    if (chunk_elems < 0)
        return fail(CF_ERR_INVALID_ARG, "chunk_elems < 0");
    if (step < m || chunk_elems == 0)
        return CF_OK;   // the slices of the first hop are only sent: nothing to add
    if (bucket == nullptr || recv == nullptr)
        return fail(CF_ERR_NULL_PTR, "bucket and recv must not be NULL at step %d", step);
    if ((reinterpret_cast<uintptr_t>(bucket) | reinterpret_cast<uintptr_t>(recv)) & 3u)
        return fail(CF_ERR_MISALIGNED, "fp32 pointers must be 4-byte aligned");
    const int l = subslice_index(CF_KIND_DP, p, m, rank, step);
    hipError_t e = cf::launch_dp_reduce(bucket + (int64_t)l * chunk_elems, recv, chunk_elems, s,
                                        num_cu_of_current_device(), land);
    if (e != hipSuccess)
        return fail_hip(e, "gradient reduce launch");
    return CF_OK;
}

// dW (+)= left^T right: the chunk GEMM with the contraction over the m_chunk rows of both operands.
cf_status wgrad_step_impl(const Resolved &r, int step, const void *left, const void *right, float *dW, hipStream_t s,
                          const CopyJob *job = nullptr)
{
    if (cf_status st = check_step(r, step))
        return st;
    if (left == nullptr || right == nullptr || dW == nullptr)
        return fail(CF_ERR_NULL_PTR, "left, right and dW must not be NULL");
    if (!aligned16(left) || !aligned16(right) || !aligned16(dW))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    if (!r.bf16_in)
        return fail(CF_ERR_UNSUPPORTED, "the weight-gradient step takes bf16 operands");
    if (r.k == 0 || r.n == 0)
        return CF_OK;
    cf::GemmParams gp;
    gp.a_t = true;
    gp.A = left;
    gp.W = right;
    gp.recv = step > 0 ? dW : nullptr;             // in place: every element is read, then written, by one lane
    gp.out = dW;
    gp.lda = r.lda;
    gp.ldw = r.ldw;
    gp.ldo = r.ldo;
    gp.M = (int)r.k;                               // rows of dW
    gp.N = (int)r.n;
    gp.K = (int)r.mc;                              // contraction: the slice's rows
    if (gp.K == 0) {                               // nothing to contract: the gradient of an empty slice is zero
        if (step == 0)
            for (int64_t row = 0; row < r.k; ++row) {
                hipError_t e = cf::launch_set_words(reinterpret_cast<unsigned *>(dW + row * r.ldo), (int)r.n, 0u, s);
                if (e != hipSuccess)
                    return fail_hip(e, "zero fill");
            }
        return CF_OK;
    }
    if (!cf::gemm_bf16_takes_recv_list(gp, true))
        return fail(CF_ERR_UNSUPPORTED, "the weight-gradient step needs operands below 2 GiB (direct-to-LDS kernel)");
    {
        const Workspace ws = workspace_for(s);
        if (ws.ptr != nullptr && ws.bytes > WS_COUNTER_BYTES) {
            gp.counters = static_cast<unsigned *>(ws.ptr);
            gp.ws = reinterpret_cast<float *>(static_cast<char *>(ws.ptr) + WS_COUNTER_BYTES);
            gp.ws_bytes = ws.bytes - WS_COUNTER_BYTES;
            gp.max_tiles = (int)(WS_TILE_COUNTER_BYTES / sizeof(unsigned));
        }
    }
    const int ncu = num_cu_of_current_device();
    if (job != nullptr && job->wait_flag != nullptr) {
        gp.wait_flag = job->wait_flag;
        gp.status = job->status;
        gp.spin_limit = spin_limit();
        gp.wait_at_start = true;
    }
    if (job != nullptr && job->bytes > 0) {
        gp.cp_src = job->src;
        gp.cp_dst = job->dst;
        gp.cp_bytes = job->bytes;
        gp.cp_wgs = ncu / 4;
    }
    hipError_t e = cf::launch_gemm_bf16(gp, true, false, s, ncu);
    if (e != hipSuccess)
        return fail_hip(e, "weight-gradient GEMM launch");
    return CF_OK;
}

cf_status accumulate(float *dst, const float *src, int64_t elems, hipStream_t s)
{
    hipError_t e = cf::launch_dp_reduce(dst, src, elems, s, num_cu_of_current_device());
    if (e != hipSuccess)
        return fail_hip(e, "accumulate launch");
    return CF_OK;
}

cf_status rs_pair_step_impl(const Resolved &r, int step, const void *A, const void *W, const float *recv, float *acc,
                            float *out, hipStream_t s)
{
    if (cf_status st = check_pair_p(r.p))
        return st;
    if (cf_status st = check_step(r, step))
        return st;
    if (A == nullptr || W == nullptr || out == nullptr)
        return fail(CF_ERR_NULL_PTR, "A, W and out must not be NULL");
    if (step == 0 && recv != nullptr)
        return fail(CF_ERR_NULL_PTR, "recv must be NULL at step 0 (nothing has been received yet)");
    const bool last = step == r.p - 1;
    const bool deferred = step > 0 && !last && recv == nullptr && acc == nullptr;   // summed by the last step
    if (step > 0 && recv == nullptr && !deferred)
        return fail(CF_ERR_NULL_PTR, "recv must not be NULL at step %d", step);
    if (r.p > 2 && step > 0 && acc == nullptr && !deferred)
        return fail(CF_ERR_NULL_PTR, "acc must not be NULL at step %d when p > 2", step);
    if (!aligned16(A) || !aligned16(W) || !aligned16(out) || !aligned16(recv) || !aligned16(acc))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    const bool use_acc = r.p > 2 && !deferred;
    if (use_acc && r.ldo != r.n)
        return fail(CF_ERR_UNSUPPORTED, "the pairwise accumulate needs packed partial sums (ldo == n)");
    // in place is fine for the buffer the last step's epilogue adds (every element is read, then written,
    // by the same lane); anything else would be overwritten while still needed
    if ((!last && (out == recv || (use_acc && out == acc))) || (last && use_acc && out == recv))
        return fail(CF_ERR_INVALID_ARG, "out may alias only the buffer the last step adds (acc; recv when p == 2)");
    const size_t elems = (size_t)r.mc * r.n;
    if (use_acc && step >= 1 && elems > 0) {
        if (step == 1) {
            if (recv != acc)                       // the first arrival initialises the accumulator
                CF_HIP(hipMemcpyAsync(acc, recv, elems * sizeof(float), hipMemcpyDeviceToDevice, s));
        } else {
            if (recv == acc)
                return fail(CF_ERR_INVALID_ARG, "recv may equal acc at step 1 only");
            if (cf_status st = accumulate(acc, recv, (int64_t)elems, s))
                return st;
        }
    }
    const int l = pair_slice(r.p, r.rank, step);
    const char *a_rows = static_cast<const char *>(A) + (size_t)l * r.mc * r.lda * in_elem(r);
    const float *add = !last ? nullptr : (use_acc ? acc : recv);   // p == 1: recv is NULL at step 0
    return launch_gemm(r, a_rows, W, add, out, s);
}

// Last step of the pairwise schedule with every round's arrival kept: out = (sum of arrivals) + own product.
cf_status rs_pair_last_step_impl(const Resolved &r, const void *A, const void *W, const float *const *recv_each,
                                 float *out, hipStream_t s)
{
    if (cf_status st = check_pair_p(r.p))
        return st;
    if (A == nullptr || W == nullptr || out == nullptr)
        return fail(CF_ERR_NULL_PTR, "A, W and out must not be NULL");
    const int count = r.p - 1;
    if (count > 0 && recv_each == nullptr)
        return fail(CF_ERR_NULL_PTR, "recv_each must not be NULL when p > 1");
    if (!aligned16(A) || !aligned16(W) || !aligned16(out))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    for (int t = 0; t < count; ++t) {
        if (recv_each[t] == nullptr)
            return fail(CF_ERR_NULL_PTR, "recv_each[%d] is NULL", t);
        if (!aligned16(recv_each[t]))
            return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
        if (recv_each[t] == out)
            return fail(CF_ERR_INVALID_ARG, "recv_each[%d] aliases out", t);
    }
    if (count > 1 && r.ldo != r.n)
        return fail(CF_ERR_UNSUPPORTED, "summing several received partials needs packed rows (ldo == n)");
    const char *a_rows = static_cast<const char *>(A) + (size_t)r.rank * r.mc * r.lda * in_elem(r);
    if (count <= 1)
        return launch_gemm(r, a_rows, W, count ? recv_each[0] : nullptr, out, s);
    cf::GemmParams probe;
    probe.A = a_rows;
    probe.W = W;
    probe.out = out;
    fill_shape(probe, r);
    if (r.bf16_in && count - 1 <= cf::GemmParams::MAX_RECV_MORE && cf::gemm_bf16_takes_recv_list(probe, r.w_kn))
        return launch_gemm(r, a_rows, W, recv_each[0], out, s, nullptr, recv_each + 1, count - 1);
    // other kernels: sum the arrivals in `out` with elementwise passes, then add the product in place
    const size_t elems = (size_t)r.mc * r.n;
    if (elems == 0)
        return CF_OK;
    CF_HIP(hipMemcpyAsync(out, recv_each[0], elems * sizeof(float), hipMemcpyDeviceToDevice, s));
    for (int t = 1; t < count; ++t)
        if (cf_status st = accumulate(out, recv_each[t], (int64_t)elems, s))
            return st;
    return launch_gemm(r, a_rows, W, out, out, s);
}

cf_status dp_pair_step_impl(int p, int rank, int step, float *bucket, int64_t chunk_elems, const float *recv,
                            hipStream_t s)
{
    if (p < 1)
        return fail(CF_ERR_INVALID_ARG, "p = %d must be >= 1", p);
    if (cf_status st = check_pair_p(p))
        return st;
    if (rank < 0 || rank >= p)
        return fail(CF_ERR_INVALID_ARG, "rank = %d not in [0, %d)", rank, p);
    if (step < 0 || step >= p)
        return fail(CF_ERR_INVALID_ARG, "step = %d not in [0, %d)", step, p);
    if (chunk_elems < 0)
        return fail(CF_ERR_INVALID_ARG, "chunk_elems < 0");
    if (step == 0 || chunk_elems == 0)
        return CF_OK;
    if (bucket == nullptr || recv == nullptr)
        return fail(CF_ERR_NULL_PTR, "bucket and recv must not be NULL at step %d", step);
    if ((reinterpret_cast<uintptr_t>(bucket) | reinterpret_cast<uintptr_t>(recv)) & 3u)
        return fail(CF_ERR_MISALIGNED, "fp32 pointers must be 4-byte aligned");
    return accumulate(bucket + (int64_t)rank * chunk_elems, recv, chunk_elems, s);
}

// Device address of this GPU's copy of `scratch`.  Looked up once per device with that device current (the
// first call on a device also zeroes the arrival counters with a small fill kernel on `s`; the kernels leave
// them at zero afterwards).  Later calls only read the table: no HIP call that could allocate.
cf_status static_scratch_of_current_device(hipStream_t s, Workspace *out)
{
    static std::mutex mu;
    static void *ptr_of[64];
    int dev = 0;
    CF_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64)
        return fail(CF_ERR_UNSUPPORTED, "device ordinal %d beyond the table of per-device scratch pointers", dev);
    std::lock_guard<std::mutex> lk(mu);
    if (ptr_of[dev] == nullptr) {
        void *ptr = nullptr;
        CF_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr)
            return fail(CF_ERR_HIP, "hipGetSymbolAddress returned a null device address for the static scratch");
        hipError_t e = cf::launch_set_words(static_cast<unsigned *>(ptr), (int)(WS_COUNTER_BYTES / sizeof(unsigned)), 0u, s);
        if (e != hipSuccess)
            return fail_hip(e, "clearing the arrival counters of the static scratch");
        ptr_of[dev] = ptr;
    }
    out->ptr = ptr_of[dev];
    out->bytes = STATIC_SCRATCH_BYTES;
    return CF_OK;
}

// ---------------------------------------------------------------------------
// events and graphs owned by the library
// ---------------------------------------------------------------------------
std::mutex g_mu;
std::unordered_map<int, std::vector<hipEvent_t>> g_events;   // per device

struct GraphEntry {
    hipGraph_t graph;
    hipGraphExec_t exec;
};
// captured rank steps by argument set; at most MAX_GRAPHS are kept (a caller that keeps changing its
// arguments gets CF_ERR_INVALID_ARG instead of an ever-growing cache: commfuse_destroy_cache empties it)
constexpr size_t MAX_GRAPHS = 4096;
std::map<std::vector<unsigned char>, GraphEntry> g_graphs;

cf_status get_events(size_t count, std::vector<hipEvent_t> *out)
{
    int dev = 0;
    CF_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_mu);
    std::vector<hipEvent_t> &pool = g_events[dev];
    while (pool.size() < count) {
        hipEvent_t ev;
        CF_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        pool.push_back(ev);
    }
    out->assign(pool.begin(), pool.begin() + count);
    return CF_OK;
}

// Query-split attention (Alg. 4) in front of every reduce-scatter step: the attention of the step's query
// slice is written to `attn_out`, which is then the chunk GEMM's left operand.
struct AttnCtx {
    cf::AttnParams ap;     // Q, K, V, out, geometry; `l` is filled in per step
};

// n_slices > 1: slices l .. l+n_slices-1 in one launch, their outputs one after the other in ctx.ap.out
cf_status launch_attention(const AttnCtx &ctx, int l, hipStream_t s, int n_slices = 1)
{
    cf::AttnParams ap = ctx.ap;
    ap.l = l;
    ap.n_slices = n_slices;
    ap.out_slice_stride = (int64_t)ap.batch * ap.c * ap.ldo;
    {
        const Workspace ws = workspace_for(s);
        if (ws.ptr != nullptr && ws.bytes > WS_COUNTER_BYTES) {
            ap.counters = static_cast<unsigned *>(ws.ptr);
            ap.ws = reinterpret_cast<float *>(static_cast<char *>(ws.ptr) + WS_COUNTER_BYTES);
            ap.ws_bytes = ws.bytes - WS_COUNTER_BYTES;
            ap.max_groups = (int)(WS_TILE_COUNTER_BYTES / sizeof(unsigned));
        }
    }
    hipError_t e = cf::launch_attn_slice(ap, s, num_cu_of_current_device());
    if (e != hipSuccess)
        return fail_hip(e, "attention launch");
    return CF_OK;
}

// Enqueues the S = m*p (sub-)steps on the two streams (see commfuse_run_schedule in the header).
// Sub-step j belongs to hop j / m; hop 0 receives nothing and the last hop sends nothing.
cf_status enqueue_schedule(const Resolved &r, int kind, const cf_buffers *b, hipStream_t cs, hipStream_t xs_in,
                           uint32_t flags, const AttnCtx *attn = nullptr)
{
    const int p = r.p, m = r.m, S = r.p * r.m;
    // CF_FUSED_COPY: the delivery for step j+1 rides in the launch of step j; one stream, no events.
    const bool fused = (flags & CF_FUSED_COPY) != 0 && !(flags & (CF_NO_COPY | CF_NO_COMPUTE));
    // CF_DEVICE_WAIT: the compute stream never waits for the copy stream between steps; each delivery
    // is followed by a flag write, and the step kernel that needs it waits for the flag on the device.
    const bool dwait = (flags & CF_DEVICE_WAIT) != 0 && !(flags & CF_NO_COMPUTE) && !fused;
    unsigned *dw_flags = nullptr, *dw_status = nullptr;
    if (dwait) {
        const Workspace ws = workspace_for(cs);
        if (ws.ptr == nullptr || ws.bytes < WS_COUNTER_BYTES)
            return fail(CF_ERR_INVALID_ARG, "CF_DEVICE_WAIT needs a registered workspace (commfuse_set_workspace)");
        dw_flags = reinterpret_cast<unsigned *>(static_cast<char *>(ws.ptr) + WS_FLAG_OFFSET);
        dw_status = reinterpret_cast<unsigned *>(static_cast<char *>(ws.ptr) + WS_STATUS_OFFSET);
    }
    const bool serial = (flags & CF_SERIAL) != 0 || xs_in == cs || fused;
    hipStream_t xs = serial ? cs : xs_in;
    const bool do_copy = !(flags & CF_NO_COPY);
    const bool do_compute = !(flags & CF_NO_COMPUTE);
    const bool poison = (flags & CF_POISON) != 0;

    const bool pair = is_pair_kind(kind);                                                // (m == 1 for these)
    const bool keep_all = kind == CF_KIND_RS_PAIR && b->recv_each != nullptr && p > 1;   // deferred aggregation
    // ring kinds with a landing buffer per hop: no buffer is reused within the call, so no delivery ever waits
    // for a kernel, and (with CF_DEVICE_WAIT and no sinks) nothing but kernels is enqueued on the compute stream
    const bool each = !pair && !is_dp_kind(kind) && b->recv_each != nullptr && p > 1;
    size_t slot_bytes;                               // one (sub-)step's delivery
    if (is_rs_kind(kind))                            // row blocks travel with their row stride, padding included
        slot_bytes = (size_t)r.mc * r.ldo * sizeof(float);
    else if (kind == CF_KIND_AG || kind == CF_KIND_WGRAD_X)
        slot_bytes = (size_t)r.mc * r.lda * in_elem(r);
    else if (kind == CF_KIND_WGRAD_G)
        slot_bytes = (size_t)r.mc * r.ldw * in_elem(r);
    else
        slot_bytes = (size_t)r.mc * sizeof(float);
    auto receives = [&](int j) { return j >= m && j < S; };          // sub-step j consumes a delivery
    auto sends = [&](int j) { return j >= 0 && j < S - m; };         // sub-step j produces something to send
    // block (j % m) of the hop buffer that holds hop (j / m)'s m blocks stacked by rows
    auto stage_of = [&](int j) { return static_cast<const char *>(b->peer_stage[j / m - 1]) + (size_t)(j % m) * slot_bytes; };
    auto sink_of = [&](int j) { return static_cast<char *>(b->peer_sink[j / m]) + (size_t)(j % m) * slot_bytes; };
    // where the delivery of sub-step j lands / is read from
    auto landing = [&](int j) -> void * {
        return each ? static_cast<char *>(b->recv_each[j / m - 1]) + (size_t)(j % m) * slot_bytes : b->slot[j & 1];
    };
    const bool need_done = !each || (b->peer_sink != nullptr && do_copy && !(kind == CF_KIND_AG || is_wgrad_kind(kind)));
    // B_out of sub-step j (Alg. 2 "B_out <- O"): a buffer of its own per sending hop (send_each), else the
    // two alternating send slots
    auto send_buf = [&](int j) -> float * {
        return b->send_each != nullptr ? b->send_each[j / m] + (size_t)(j % m) * r.mc * r.ldo : b->send_slot[j & 1];
    };

    // event layout: [0] start, [1] end, ready[j] = 2+j, done[j] = 2+S+j, sunk[j] = 2+2S+j
    std::vector<hipEvent_t> ev;
    if (cf_status st = get_events(2 + 3 * (size_t)S, &ev))
        return st;
    hipEvent_t ev_start = ev[0], ev_end = ev[1];
    auto ready = [&](int j) { return ev[2 + j]; };
    auto done = [&](int j) { return ev[2 + S + j]; };
    auto sunk = [&](int j) { return ev[2 + 2 * S + j]; };

    if (dwait) {                                     // all delivery flags down before any copy raises one
        hipError_t e = cf::launch_set_words(dw_flags, S, 0u, cs);
        if (e != hipSuccess)
            return fail_hip(e, "flag reset");
    }
    if (!serial) {
        CF_HIP(hipEventRecord(ev_start, cs));
        CF_HIP(hipStreamWaitEvent(xs, ev_start, 0));
    }

    // what rank r-1 delivers for sub-step j+1 lands in slot[(j+1) % 2]
    auto deliver = [&](int j) -> cf_status {
        if (!(receives(j + 1) && do_copy) || fused)
            return CF_OK;
        // pairwise reduce-scatter: every arrival is kept (recv_each), or the first one initialises the
        // accumulator, which is O itself
        void *dst = keep_all ? b->recv_each[j] : (kind == CF_KIND_RS_PAIR && j == 0) ? b->O : landing(j + 1);
        // the slot was last read by the kernel of sub-step j-1 (if that one read a slot at all)
        if (!serial && do_compute && receives(j - 1) && !keep_all && !each)
            CF_HIP(hipStreamWaitEvent(xs, done(j - 1), 0));
        if (slot_bytes == 0)
            return CF_OK;
        if (poison) {
            hipError_t e = cf::launch_fill_ff(dst, slot_bytes, xs);
            if (e != hipSuccess)
                return fail_hip(e, "poison fill");
        }
        CF_HIP(hipMemcpyAsync(dst, stage_of(j + 1), slot_bytes, hipMemcpyDeviceToDevice, xs));
        if (dwait && !serial) {
            hipError_t e = cf::launch_set_words(dw_flags + (j + 1), 1, 1u, xs);   // after the copy, same stream
            if (e != hipSuccess)
                return fail_hip(e, "flag write");
        }
        if (!serial)
            CF_HIP(hipEventRecord(ready(j + 1), xs));
        return CF_OK;
    };

    auto kernel = [&](int j) -> cf_status {
        if (!do_compute)
            return CF_OK;
        const bool last = j == S - 1;
        if (!serial && do_copy && receives(j) && !dwait && (!keep_all || last))
            CF_HIP(hipStreamWaitEvent(cs, ready(j), 0));   // deliveries are in order on the copy stream
        cf_status st = CF_OK;
        CopyJob job;
        if (dwait && !serial && receives(j)) {     // the kernel itself waits for the delivery of sub-step j
            job.wait_flag = dw_flags + j;
            job.status = dw_status;
            job.wait_at_start = kind != CF_KIND_RS;  // the slice is an operand; B_in is needed by the add only
        }
        if (fused && receives(j + 1)) {            // what the neighbour delivers for sub-step j+1
            job.src = stage_of(j + 1);
            job.dst = landing(j + 1);
            job.bytes = slot_bytes;
        }
        // B_out slot (j % 2) was last sent at sub-step j-2 (a send buffer per hop is never reused)
        const bool wait_sunk = !serial && do_copy && b->peer_sink != nullptr && sends(j) && sends(j - 2) &&
                               b->send_each == nullptr;
        if (kind == CF_KIND_RS) {
            if (wait_sunk)
                CF_HIP(hipStreamWaitEvent(cs, sunk(j - 2), 0));
            const float *recv = receives(j) ? static_cast<const float *>(landing(j)) : nullptr;
            float *out = sends(j) ? send_buf(j) : static_cast<float *>(b->O) + (size_t)(j % m) * r.mc * r.ldo;
            if (attn != nullptr) {                 // Alg. 4: attention of slice l, then the projection of its output
                st = launch_attention(*attn, chunk_index(CF_KIND_RS, p, r.rank, j), cs);
                if (st == CF_OK)
                    st = launch_gemm(r, attn->ap.out, b->W, recv, out, cs, &job);
            } else {
                st = rs_step_impl(r, j, b->A_or_own_shard, b->W, recv, out, cs, &job);
            }
        } else if (kind == CF_KIND_AG) {
            const void *shard = receives(j) ? landing(j)
                                            : static_cast<const char *>(b->A_or_own_shard) + (size_t)(j % m) * slot_bytes;
            st = ag_step_impl(r, j, shard, b->W, b->O, cs, &job);
        } else if (is_wgrad_kind(kind)) {
            const void *hand = receives(j) ? landing(j)
                                           : static_cast<const char *>(b->A_or_own_shard) + (size_t)(j % m) * slot_bytes;
            const int c = subslice_index(CF_KIND_AG, p, m, r.rank, j);
            const size_t local_row = (size_t)(kind == CF_KIND_WGRAD_X ? r.ldw : r.lda) * in_elem(r);
            const void *local = static_cast<const char *>(b->W) + (size_t)c * r.mc * local_row;
            st = kind == CF_KIND_WGRAD_X ? wgrad_step_impl(r, j, hand, local, static_cast<float *>(b->O), cs, &job)
                                         : wgrad_step_impl(r, j, local, hand, static_cast<float *>(b->O), cs, &job);
        } else if (kind == CF_KIND_RS_PAIR) {
            if (wait_sunk)
                CF_HIP(hipStreamWaitEvent(cs, sunk(j - 2), 0));
            float *acc = static_cast<float *>(b->O);
            const float *recv = j == 0 ? nullptr : (j == 1 ? acc : static_cast<const float *>(b->slot[j & 1]));
            float *out = !last ? send_buf(j) : acc;
            if (!keep_all)
                st = rs_pair_step_impl(r, j, b->A_or_own_shard, b->W, recv, acc, out, cs);
            else if (!last)
                st = rs_pair_step_impl(r, j, b->A_or_own_shard, b->W, nullptr, nullptr, out, cs);
            else
                st = rs_pair_last_step_impl(r, b->A_or_own_shard, b->W,
                                            reinterpret_cast<const float *const *>(b->recv_each), acc, cs);
        } else if (kind == CF_KIND_DP_PAIR) {
            st = dp_pair_step_impl(p, r.rank, j, static_cast<float *>(b->O), r.mc,
                                   j > 0 ? static_cast<const float *>(b->slot[j & 1]) : nullptr, cs);
        } else {
            st = dp_step_impl(p, r.rank, j, static_cast<float *>(b->O), r.mc,
                              receives(j) ? static_cast<const float *>(b->slot[j & 1]) : nullptr, cs, m);
        }
        if (st != CF_OK)
            return st;
        if (!serial && need_done)
            CF_HIP(hipEventRecord(done(j), cs));
        return CF_OK;
    };

    // emulated send of sub-step j: B_out (RS), the slice in hand (AG), the local slice (DP)
    auto send = [&](int j) -> cf_status {
        if (!(b->peer_sink != nullptr && sends(j) && do_copy))
            return CF_OK;
        const void *src;
        if (is_rs_kind(kind)) {
            src = send_buf(j);
        } else if (kind == CF_KIND_AG || is_wgrad_kind(kind)) {
            src = receives(j) ? landing(j)
                              : static_cast<const char *>(b->A_or_own_shard) + (size_t)(j % m) * slot_bytes;
        } else {
            const int l = pair ? pair_slice(p, r.rank, j) : subslice_index(CF_KIND_DP, p, m, r.rank, j);
            src = static_cast<const float *>(b->O) + (int64_t)l * r.mc;
        }
        if (slot_bytes == 0)
            return CF_OK;
        if (!serial && do_compute && kind != CF_KIND_AG && !is_wgrad_kind(kind))
            CF_HIP(hipStreamWaitEvent(xs, done(j), 0));
        // (all-gather: the slice in hand was delivered on this same stream, so it is already ordered)
        CF_HIP(hipMemcpyAsync(sink_of(j), src, slot_bytes, hipMemcpyDeviceToDevice, xs));
        if (!serial)
            CF_HIP(hipEventRecord(sunk(j), xs));
        return CF_OK;
    };

    for (int j = 0; j < S; ++j) {
        cf_status st;
        if (serial) {
            if ((st = kernel(j)) || (st = send(j)) || (st = deliver(j)))
                return st;
        } else {
            // the delivery for sub-step j+1 is in flight while the kernel of sub-step j runs
            if ((st = deliver(j)) || (st = kernel(j)) || (st = send(j)))
                return st;
        }
    }
    if (!serial) {
        CF_HIP(hipEventRecord(ev_end, xs));
        CF_HIP(hipStreamWaitEvent(cs, ev_end, 0));
    }
    return CF_OK;
}

// CF_PERSISTENT: all (sub-)steps of a rank step in ONE launch of the chunk-GEMM kernel (its work-item loop) --
// reduce-scatter, all-gather, pairwise reduce-scatter with deferred aggregation, the projection of the attention
// layer (after one attention launch for all slices) -- or, for the weight gradient, as one GEMM over the gathered
// operand; the deliveries are enqueued before it on the same stream.  The steps of one launch run side by side,
// so every sending step of a reduce-scatter kind stores its B_out into a buffer of its own (cf_buffers.send_each);
// the emulated sends into peer_sink, if any, are copied from those after the launch.
cf_status enqueue_persistent(const Resolved &r, int kind, const cf_buffers *b, hipStream_t cs, hipStream_t xs,
                             uint32_t flags, const AttnCtx *attn = nullptr)
{
    const int p = r.p, m = r.m, S = r.p * r.m;
    const bool do_copy = !(flags & CF_NO_COPY) && p > 1;
    const bool do_compute = !(flags & CF_NO_COMPUTE);
    const bool poison = (flags & CF_POISON) != 0;
    const size_t slot_bytes = is_dp_kind(kind)         ? (size_t)r.mc * sizeof(float)
                              : is_rs_kind(kind)       ? (size_t)r.mc * r.ldo * sizeof(float)
                              : kind == CF_KIND_WGRAD_G ? (size_t)r.mc * r.ldw * in_elem(r)
                                                        : (size_t)r.mc * r.lda * in_elem(r);
    // Weight gradient: the moving operand must sit in "gathered" order -- one [p*m_chunk x width] buffer, the
    // own slice in row block `rank`, hop i's landing buffer in row block (rank - i) mod p, the row block the
    // local operand pairs it with.  The p chunk GEMMs dW += slice^T local_slice are then ONE GEMM with the
    // contraction over all p*m_chunk rows: dW is written once instead of read and written p times.
    uintptr_t gathered = 0;
    if (is_wgrad_kind(kind)) {
        const size_t hop_bytes = slot_bytes * m;
        gathered = reinterpret_cast<uintptr_t>(b->A_or_own_shard) - (uintptr_t)r.rank * hop_bytes;
        for (int i = 1; i < p; ++i)
            if (reinterpret_cast<uintptr_t>(b->recv_each[i - 1]) != gathered + (uintptr_t)chunk_index(CF_KIND_AG, p, r.rank, i) * hop_bytes)
                return fail(CF_ERR_UNSUPPORTED,
                            "CF_PERSISTENT for the weight gradient needs the gathered layout: recv_each[%d] must be row block "
                            "%d of the buffer whose row block %d is the own slice", i - 1, chunk_index(CF_KIND_AG, p, r.rank, i), r.rank);
    }
    auto receives = [&](int j) { return j >= m && j < S; };
    auto sends = [&](int j) { return j >= 0 && j < S - m; };
    auto landing = [&](int j) -> void * {
        return static_cast<char *>(b->recv_each[j / m - 1]) + (size_t)(j % m) * slot_bytes;
    };
    auto stage_of = [&](int j) { return static_cast<const char *>(b->peer_stage[j / m - 1]) + (size_t)(j % m) * slot_bytes; };
    // CF_FUSED_COPY with the one-launch reduce-scatter or all-gather: the delivery is carried by the consumer, no
    // copy is launched.  Reduce-scatter: the waves that need B_in read it from the neighbour's buffer (peer_stage)
    // under the main loop, add it, and store it to the landing buffer; only where the launch runs the kernel that
    // brings B_in in through LDS (256x256 tile, a k range long enough).  All-gather: the kernel takes its left
    // operand from the neighbour's buffer, and each k-tile that comes in through LDS is stored on to the landing
    // buffer by one of the workgroups that load it (k a multiple of the k-tile).  Otherwise the deliveries are
    // enqueued in front as without the flag.
    bool carried = false;
    if ((flags & CF_FUSED_COPY) && (kind == CF_KIND_RS || kind == CF_KIND_AG) && attn == nullptr && do_copy && do_compute &&
        slot_bytes > 0 && r.mc > 0 && r.n > 0 && r.k > 0) {
        cf::GemmParams probe;
        probe.W = b->W;
        fill_shape(probe, r);
        probe.n_steps = S;
        carried = cf::gemm_bf16_carries_delivery(probe, r.w_kn, r.bf16_out, num_cu_of_current_device(), kind == CF_KIND_RS);
    }
    // A reduce-scatter launch that cannot stream B_in (a short k range, another tile, the projection of the attention
    // layer) carries its deliveries the other way: the epilogue reads B_in from the neighbour's buffer, and the same
    // work item copies its tile's part of it to the landing buffer beside its GEMM (no counter: nobody waits for it).
    bool carried_beside = false;
    if ((flags & CF_FUSED_COPY) && kind == CF_KIND_RS && !carried && do_copy && do_compute && slot_bytes > 0 && r.mc > 0 &&
        r.n > 0 && r.k > 0 && r.ldo == r.n) {
        cf::GemmParams probe;
        probe.W = b->W;
        fill_shape(probe, r);
        probe.n_steps = S;
        carried_beside = cf::gemm_bf16_lands_beside(probe, r.w_kn, r.bf16_out, num_cu_of_current_device());
    }
    // The gradient bucket with CF_FUSED_COPY: the add kernels read the arrivals from the neighbours' buffers and
    // store them on to the landing buffers in the same pass (ring: 16 bytes per element instead of a copy's 8 plus
    // the add's 12; pairwise, p - 1 arrivals in one pass: 8 p instead of 12 p - 4).
    if ((flags & CF_FUSED_COPY) && is_dp_kind(kind) && do_copy && do_compute && slot_bytes > 0)
        carried = true;
    // The pairwise reduce-scatter with CF_FUSED_COPY: the arrival of round t travels while step t - 1 computes, so the
    // work items of step t - 1 land it -- each its own output tile's part, from the partner's buffer to the landing
    // buffer, after its own stores -- and count the tile up; the last step's work item waits for its tile's count
    // before it sums the arrivals.  Needs the registered workspace (a counter per output tile, the status word).
    unsigned *pair_ready = nullptr, *pair_status = nullptr;
    int pair_tiles = 0;
    if ((flags & CF_FUSED_COPY) && kind == CF_KIND_RS_PAIR && do_copy && do_compute && slot_bytes > 0 && r.mc > 0 &&
        r.n > 0 && r.k > 0) {
        cf::GemmParams probe;
        probe.W = b->W;
        fill_shape(probe, r);
        probe.n_steps = S;
        pair_tiles = cf::gemm_bf16_tiles_landing_arrivals(probe, r.w_kn, num_cu_of_current_device());
        const Workspace ws = workspace_for(cs);
        if (pair_tiles > 0 && ws.ptr != nullptr && ws.bytes >= WS_COUNTER_BYTES &&
            (size_t)pair_tiles <= WS_TILE_COUNTER_BYTES / sizeof(unsigned)) {
            pair_ready = static_cast<unsigned *>(ws.ptr);
            pair_status = reinterpret_cast<unsigned *>(static_cast<char *>(ws.ptr) + WS_STATUS_OFFSET);
            carried = true;
        }
    }
    // Without CF_SERIAL (reduce-scatter and all-gather on two streams): the rank step as a few launches, each a group
    // of consecutive (sub-)steps that fills the chip about once, and the deliveries of a group copied on the copy
    // stream under the launches of the groups before it -- Fig. 1's overlap with a group of steps where the paper has
    // one step.  One event per group orders the two streams; every hop has its own landing buffer, so the copy
    // stream never waits for a kernel.
    int group = S;
    const bool grouped = !(flags & CF_SERIAL) && xs != cs && (kind == CF_KIND_RS || kind == CF_KIND_AG) && attn == nullptr &&
                         !carried && !carried_beside && p > 1 && slot_bytes > 0 && r.mc > 0 && r.n > 0 && r.k > 0;
    if (grouped) {
        cf::GemmParams probe;
        probe.W = b->W;
        fill_shape(probe, r);
        probe.n_steps = S;
        group = cf::gemm_bf16_steps_per_launch(probe, r.w_kn, num_cu_of_current_device());
    }
    const int n_groups = (S + group - 1) / group;
    std::vector<hipEvent_t> ev;
    if (grouped) {
        if (cf_status st = get_events(1 + (size_t)n_groups, &ev))
            return st;
        CF_HIP(hipEventRecord(ev[0], cs));               // the copy stream starts behind what the compute stream holds
        CF_HIP(hipStreamWaitEvent(xs, ev[0], 0));
    }
    if (grouped && do_copy) {
        for (int g = 0; g < n_groups; ++g) {             // the deliveries of group g: one batched copy launch, then its event
            const void *srcs[cf::GemmParams::MAX_STEPS];
            void *dsts[cf::GemmParams::MAX_STEPS];
            int n = 0;
            for (int j = g * group; j < S && j < (g + 1) * group; ++j)
                if (receives(j)) {
                    srcs[n] = stage_of(j);
                    dsts[n++] = landing(j);
                    if (poison) {
                        hipError_t e = cf::launch_fill_ff(landing(j), slot_bytes, xs);
                        if (e != hipSuccess)
                            return fail_hip(e, "poison fill");
                    }
                }
            if (n > 0 && cf::copy_batch_takes(srcs, dsts, n, slot_bytes)) {
                hipError_t e = cf::launch_copy_batch(srcs, dsts, n, slot_bytes, xs);
                if (e != hipSuccess)
                    return fail_hip(e, "delivery copy launch");
            } else {
                for (int i = 0; i < n; ++i)
                    CF_HIP(hipMemcpyAsync(dsts[i], srcs[i], slot_bytes, hipMemcpyDeviceToDevice, xs));
            }
            CF_HIP(hipEventRecord(ev[1 + g], xs));
        }
        if (!do_compute)                                 // copies only: the compute stream still ends behind them
            CF_HIP(hipStreamWaitEvent(cs, ev[n_groups], 0));
    }
    if (do_copy && slot_bytes > 0 && !carried && !carried_beside && !grouped) {
        // all deliveries of the rank step are due now: one batched copy launch where the buffers allow it
        // (at most 16 hops of 16-byte-aligned whole hop buffers), else one hipMemcpyAsync per (sub-)step
        const void *srcs[cf::GemmParams::MAX_STEPS];
        void *dsts[cf::GemmParams::MAX_STEPS];
        for (int i = 1; i < p; ++i) {
            srcs[i - 1] = b->peer_stage[i - 1];
            dsts[i - 1] = b->recv_each[i - 1];
        }
        const bool batched = cf::copy_batch_takes(srcs, dsts, p - 1, slot_bytes * m);
        for (int j = m; j < S; ++j) {
            void *dst = landing(j);
            if (poison) {
                hipError_t e = cf::launch_fill_ff(dst, slot_bytes, cs);
                if (e != hipSuccess)
                    return fail_hip(e, "poison fill");
            }
            const char *src = static_cast<const char *>(b->peer_stage[j / m - 1]) + (size_t)(j % m) * slot_bytes;
            if (!batched)
                CF_HIP(hipMemcpyAsync(dst, src, slot_bytes, hipMemcpyDeviceToDevice, cs));
        }
        if (batched) {
            hipError_t e = cf::launch_copy_batch(srcs, dsts, p - 1, slot_bytes * m, cs);
            if (e != hipSuccess)
                return fail_hip(e, "delivery copy launch");
        }
    }
    // Gradient bucket: nothing to fuse into -- the adds of a rank step, each on the landing buffer of its own hop
    // (ring: every hop's slice is a different one, Alg. 2 with the identity; pairwise: all arrivals are summed
    // into the own slice in round order), behind the one batched delivery
    if (do_compute && kind == CF_KIND_DP_PAIR && p > 1 && r.mc > 0) {
        // every round's arrival goes into the own slice: one pass that reads them all (same order of additions)
        const float *srcs[cf::GemmParams::MAX_STEPS];
        float *lands[cf::GemmParams::MAX_STEPS];
        for (int j = 1; j < p; ++j) {
            srcs[j - 1] = carried ? reinterpret_cast<const float *>(stage_of(j)) : static_cast<const float *>(landing(j));
            lands[j - 1] = static_cast<float *>(landing(j));
        }
        if (cf_status st = check_pair_p(p))
            return st;
        hipError_t e = cf::launch_dp_reduce_multi(static_cast<float *>(b->O) + (int64_t)r.rank * r.mc, srcs, p - 1, r.mc, cs,
                                                  num_cu_of_current_device(), carried ? lands : nullptr);
        if (e != hipSuccess)
            return fail_hip(e, "gradient reduce launch");
        return CF_OK;
    }
    if (do_compute && is_dp_kind(kind)) {
        float *bucket = static_cast<float *>(b->O);
        for (int j = m; j < S; ++j) {
            const float *recv = carried ? reinterpret_cast<const float *>(stage_of(j)) : static_cast<const float *>(landing(j));
            cf_status st = kind == CF_KIND_DP_PAIR ? dp_pair_step_impl(p, r.rank, j, bucket, r.mc, recv, cs)
                                                   : dp_step_impl(p, r.rank, j, bucket, r.mc, recv, cs, m,
                                                                  carried ? static_cast<float *>(landing(j)) : nullptr);
            if (st != CF_OK)
                return st;
        }
        return CF_OK;
    }
    if (is_dp_kind(kind))
        return CF_OK;
    if (do_compute && is_wgrad_kind(kind)) {
        Resolved all = r;
        all.m = 1;
        all.mc = r.mc * S;                           // all rows of the gathered and the local operand
        const void *moving = reinterpret_cast<const void *>(gathered);
        if (cf_status st = kind == CF_KIND_WGRAD_X ? wgrad_step_impl(all, 0, moving, b->W, static_cast<float *>(b->O), cs)
                                                   : wgrad_step_impl(all, 0, b->W, moving, static_cast<float *>(b->O), cs))
            return st;
    }
    // Alg. 4: the attention of a slice depends on nothing that travels, so the attention of ALL p query slices
    // is one launch with a chip-filling grid (no key split, no merge); its output [p slices x B*S/p x heads*D_h]
    // is then the left operand of the persistent projection + reduce-scatter kernel, slice by slice.
    if (do_compute && attn != nullptr && r.mc > 0)
        if (cf_status st = launch_attention(*attn, 0, cs, p))
            return st;
    if (do_compute && !is_wgrad_kind(kind) && r.mc > 0 && r.n > 0) {
        if (r.k == 0)
            return fail(CF_ERR_UNSUPPORTED, "CF_PERSISTENT needs k > 0");
      for (int g0 = 0; g0 < S; g0 += group) {            // one launch per group of steps (all steps: one group)
        const int g1 = g0 + group < S ? g0 + group : S;
        cf::GemmParams gp;
        gp.W = b->W;
        fill_shape(gp, r);
        gp.n_steps = g1 - g0;
        gp.num_cu = num_cu_of_current_device();
        for (int jj = g0; jj < g1; ++jj) {
            const int j = jj - g0;                       // the step's place in this launch
            if (kind == CF_KIND_RS_PAIR) {
                // Appendix A(a) with deferred aggregation: steps 0..p-2 are plain chunk GEMMs for the partners'
                // slices, the last step adds every arrival to the product for the own slice (m = 1 here)
                const bool last = j == p - 1;
                gp.A_step[j] = static_cast<const char *>(b->A_or_own_shard) +
                               (size_t)pair_slice(p, r.rank, j) * r.mc * r.lda * in_elem(r);
                gp.recv_step[j] = last && p > 1 ? static_cast<const float *>(b->recv_each[0]) : nullptr;
                gp.out_step[j] = last ? b->O : static_cast<void *>(b->send_each[j]);
                gp.flag_step[j] = nullptr;
                if (last)
                    for (int t = 1; t < p - 1; ++t)
                        gp.recv_more[gp.n_recv_more++] = static_cast<const float *>(b->recv_each[t]);
                if (carried && !last) {              // this step's work items land the arrival of round j + 1
                    gp.tail_src[j] = static_cast<const float *>(b->peer_stage[j]);
                    gp.tail_dst[j] = static_cast<float *>(b->recv_each[j]);
                }
                if (carried && last) {
                    gp.tile_ready = pair_ready;
                    gp.ready_count = p - 1;
                    gp.max_tiles = (int)(WS_TILE_COUNTER_BYTES / sizeof(unsigned));
                    gp.status = pair_status;
                    gp.spin_limit = spin_limit();
                }
                continue;
            }
            const int c = subslice_index(kind, p, m, r.rank, jj);
            if (kind == CF_KIND_RS) {
                gp.A_step[j] = static_cast<const char *>(b->A_or_own_shard) + (size_t)c * r.mc * r.lda * in_elem(r);
                gp.recv_step[j] = receives(jj) ? static_cast<const float *>(landing(jj)) : nullptr;
                if (carried && receives(jj)) {       // read from the neighbour's buffer, land it here
                    gp.recv_step[j] = reinterpret_cast<const float *>(stage_of(jj));
                    gp.land_step[j] = landing(jj);
                }
                if (carried_beside && receives(jj)) { // ... in the epilogue, and landed by a copy beside the GEMM
                    gp.recv_step[j] = reinterpret_cast<const float *>(stage_of(jj));
                    gp.tail_src[j] = gp.recv_step[j];
                    gp.tail_dst[j] = static_cast<float *>(landing(jj));
                }
                gp.out_step[j] = sends(jj) ? static_cast<void *>(b->send_each[jj / m] + (size_t)(jj % m) * r.mc * r.ldo)
                                           : static_cast<void *>(static_cast<float *>(b->O) + (size_t)(jj % m) * r.mc * r.ldo);
            } else {
                gp.A_step[j] = receives(jj) ? landing(jj)
                                            : static_cast<const char *>(b->A_or_own_shard) + (size_t)(jj % m) * slot_bytes;
                if (carried && receives(jj)) {       // the slice is read from the neighbour's buffer and landed here
                    gp.A_step[j] = stage_of(jj);
                    gp.land_step[j] = landing(jj);
                }
                gp.recv_step[j] = nullptr;
                gp.out_step[j] = static_cast<char *>(b->O) + (size_t)c * r.mc * r.ldo * (r.bf16_out ? 2 : 4);
            }
            gp.flag_step[j] = nullptr;               // everything was delivered before the launch
        }
        if (grouped && do_copy)                          // this group's deliveries have landed
            CF_HIP(hipStreamWaitEvent(cs, ev[1 + g0 / group], 0));
        if (gp.tile_ready != nullptr) {                  // the tiles' counters start at zero (a fill kernel: capturable)
            hipError_t e0 = cf::launch_set_words(gp.tile_ready, pair_tiles, 0u, cs);
            if (e0 != hipSuccess)
                return fail_hip(e0, "counter fill");
        }
        hipError_t e = cf::launch_gemm_bf16(gp, r.w_kn, r.bf16_out, cs, gp.num_cu);
        if (e != hipSuccess)
            return fail_hip(e, "persistent rank-step launch");
      }
    }
    // emulated sends (Alg. 2 "p2p_send(B_out)", Alg. 1 "p2p_send(B_out)" of the slice in hand): hop i < p-1 into
    // peer_sink[i], all hops as one batched copy where the buffers allow it
    if (b->peer_sink != nullptr && do_copy && slot_bytes > 0) {
        const void *srcs[cf::GemmParams::MAX_STEPS];
        void *dsts[cf::GemmParams::MAX_STEPS];
        for (int i = 0; i < p - 1; ++i) {
            srcs[i] = is_rs_kind(kind) ? static_cast<const void *>(b->send_each[i])
                                       : (i == 0 ? b->A_or_own_shard : static_cast<const void *>(b->recv_each[i - 1]));
            dsts[i] = b->peer_sink[i];
        }
        if (cf::copy_batch_takes(srcs, dsts, p - 1, slot_bytes * m)) {
            hipError_t e = cf::launch_copy_batch(srcs, dsts, p - 1, slot_bytes * m, cs);
            if (e != hipSuccess)
                return fail_hip(e, "send copy launch");
        } else {
            for (int i = 0; i < p - 1; ++i)
                CF_HIP(hipMemcpyAsync(dsts[i], srcs[i], slot_bytes * m, hipMemcpyDeviceToDevice, cs));
        }
    }
    return CF_OK;
}

cf_status check_buffers(const Resolved &r, int kind, const cf_buffers *b, uint32_t flags)
{
    if (b == nullptr)
        return fail(CF_ERR_NULL_PTR, "buffers is NULL");
    if (b->O == nullptr)
        return fail(CF_ERR_NULL_PTR, "buffers->O is NULL");
    if (!is_dp_kind(kind) && (b->A_or_own_shard == nullptr || b->W == nullptr))
        return fail(CF_ERR_NULL_PTR, "buffers->A_or_own_shard / W is NULL");
    if (b->recv_each != nullptr && is_dp_kind(kind) && !(flags & CF_PERSISTENT))
        return fail(CF_ERR_INVALID_ARG, "buffers->recv_each is used by the gradient-bucket kinds with CF_PERSISTENT only");
    const bool keep_all = b->recv_each != nullptr;
    if (r.p > 1) {
        if (keep_all) {
            for (int i = 0; i < r.p - 1; ++i)
                if (b->recv_each[i] == nullptr || b->recv_each[i] == b->O)
                    return fail(CF_ERR_NULL_PTR, "recv_each[%d] is NULL or aliases O", i);
        } else {
            if (b->slot[0] == nullptr || b->slot[1] == nullptr)
                return fail(CF_ERR_NULL_PTR, "buffers->slot[0..1] must be set when p > 1");
            if (b->slot[0] == b->slot[1])
                return fail(CF_ERR_INVALID_ARG, "the two slots must be distinct buffers");
        }
        if (!(flags & CF_NO_COPY)) {
            if (b->peer_stage == nullptr)
                return fail(CF_ERR_NULL_PTR, "buffers->peer_stage is NULL");
            for (int i = 0; i < r.p - 1; ++i) {
                if (b->peer_stage[i] == nullptr)
                    return fail(CF_ERR_NULL_PTR, "peer_stage[%d] is NULL", i);
                if (b->peer_sink != nullptr && b->peer_sink[i] == nullptr)
                    return fail(CF_ERR_NULL_PTR, "peer_sink[%d] is NULL", i);
            }
        }
        if (is_rs_kind(kind) && b->send_each != nullptr) {
            for (int i = 0; i < r.p - 1; ++i) {
                if (b->send_each[i] == nullptr || b->send_each[i] == b->O)
                    return fail(CF_ERR_NULL_PTR, "send_each[%d] is NULL or aliases O", i);
                if (!aligned16(b->send_each[i]))
                    return fail(CF_ERR_MISALIGNED, "send_each[%d] must be 16-byte aligned", i);
                for (int q = 0; q < r.p - 1; ++q)
                    if ((q < i && b->send_each[q] == b->send_each[i]) ||
                        (keep_all && b->recv_each[q] == static_cast<void *>(b->send_each[i])))
                        return fail(CF_ERR_INVALID_ARG, "send_each[%d] aliases another send or landing buffer", i);
            }
        } else if (is_rs_kind(kind)) {
            if (flags & CF_PERSISTENT)
                return fail(CF_ERR_INVALID_ARG, "CF_PERSISTENT needs buffers->send_each (a B_out buffer per sending step)");
            if (b->send_slot[0] == nullptr || b->send_slot[1] == nullptr)
                return fail(CF_ERR_NULL_PTR, "buffers->send_slot[0..1] must be set for the reduce-scatter path");
            if (b->send_slot[0] == b->send_slot[1])
                return fail(CF_ERR_INVALID_ARG, "the two send slots must be distinct buffers");
        }
    }
    if (is_pair_kind(kind) && !is_dp_kind(kind) && r.ldo != r.n)
        return fail(CF_ERR_UNSUPPORTED, "the pairwise schedule needs packed partial sums (ldo == n)");
    return CF_OK;
}

void append_bytes(std::vector<unsigned char> &v, const void *p, size_t n)
{
    const unsigned char *c = static_cast<const unsigned char *>(p);
    v.insert(v.end(), c, c + n);
}

// Flag checks, buffer checks and (CF_GRAPH) capture-once / replay shared by the schedule entry points.
// `key` arrives holding what identifies the descriptor; the rest of the argument set is appended here.
cf_status run_schedule_common(const Resolved &r, int kind, const cf_buffers *bufs, hipStream_t cs, hipStream_t xs,
                              uint32_t flags, const AttnCtx *attn, std::vector<unsigned char> &key)
{
    if (flags & ~(uint32_t)(CF_NO_COPY | CF_NO_COMPUTE | CF_SERIAL | CF_POISON | CF_GRAPH | CF_FUSED_COPY | CF_DEVICE_WAIT |
                            CF_PERSISTENT))
        return fail(CF_ERR_INVALID_ARG, "unknown flag bits 0x%x", flags);
    if (is_pair_kind(kind)) {
        if (cf_status st = check_pair_p(r.p))
            return st;
        const bool one_launch = (flags & CF_PERSISTENT) && !(flags & CF_DEVICE_WAIT);
        if ((flags & (CF_FUSED_COPY | CF_DEVICE_WAIT)) && !one_launch)
            return fail(CF_ERR_UNSUPPORTED, "CF_FUSED_COPY / CF_DEVICE_WAIT are not available for the pairwise kinds (but "
                                            "CF_FUSED_COPY with CF_PERSISTENT is)");
    }
    if (flags & CF_DEVICE_WAIT) {
        if (flags & CF_FUSED_COPY)
            return fail(CF_ERR_UNSUPPORTED, "CF_DEVICE_WAIT and CF_FUSED_COPY exclude each other");
        // A captured graph has no edge between a flag write and the kernel that polls the flag, so a replay
        // may queue the writer behind the waiting kernel; two live streams cannot be ordered that way.
        if (flags & CF_GRAPH)
            return fail(CF_ERR_UNSUPPORTED, "CF_DEVICE_WAIT cannot be captured into a graph (CF_GRAPH)");
        if (is_dp_kind(kind) || !(is_wgrad_kind(kind) ? wgrad_can_carry_copy(r) : step_can_carry_copy(r)) ||
            r.p * r.m > WS_MAX_FLAGS)
            return fail(CF_ERR_UNSUPPORTED, "CF_DEVICE_WAIT needs the bf16 chunk-GEMM kernels (kind RS or AG, bf16 operands)");
    }
    if (flags & CF_FUSED_COPY) {
        if (flags & CF_POISON)
            return fail(CF_ERR_UNSUPPORTED, "CF_FUSED_COPY cannot be combined with CF_POISON");
        const bool dp_one_launch = is_dp_kind(kind) && (flags & CF_PERSISTENT);   // the add kernels carry the deliveries
        if (!dp_one_launch && (is_dp_kind(kind) || !(is_wgrad_kind(kind) ? wgrad_can_carry_copy(r) : step_can_carry_copy(r))))
            return fail(CF_ERR_UNSUPPORTED, "CF_FUSED_COPY needs the bf16 chunk-GEMM kernels (kind RS or AG, bf16 operands), or "
                                            "CF_PERSISTENT for the gradient-bucket kinds");
    }
    if (flags & CF_PERSISTENT) {
        if (flags & CF_DEVICE_WAIT)
            return fail(CF_ERR_UNSUPPORTED, "CF_PERSISTENT excludes CF_DEVICE_WAIT");
        if (attn != nullptr && r.m != 1)
            return fail(CF_ERR_UNSUPPORTED, "CF_PERSISTENT with the attention layer needs m = 1");
        const bool ok_kind = is_dp_kind(kind)      ? true
                             : is_wgrad_kind(kind) ? wgrad_can_carry_copy(r)
                                                   : (kind == CF_KIND_RS || kind == CF_KIND_AG || kind == CF_KIND_RS_PAIR) &&
                                                         step_can_carry_copy(r) && r.p - 2 <= cf::GemmParams::MAX_RECV_MORE;
        if (!ok_kind || r.p * r.m > cf::GemmParams::MAX_STEPS)
            return fail(CF_ERR_UNSUPPORTED,
                        "CF_PERSISTENT needs bf16 operands (kinds RS, AG, RS_PAIR, weight gradient; the gradient-bucket kinds take "
                        "fp32) and at most %d (sub-)steps",
                        cf::GemmParams::MAX_STEPS);
        if (bufs != nullptr && bufs->peer_sink != nullptr && is_dp_kind(kind))
            return fail(CF_ERR_UNSUPPORTED, "CF_PERSISTENT does not feed peer_sink for the gradient-bucket kinds");
        if (bufs != nullptr && r.p > 1 && bufs->recv_each == nullptr)
            return fail(CF_ERR_INVALID_ARG, "CF_PERSISTENT needs buffers->recv_each (a landing buffer per hop)");
        // A kernel that holds its compute units for a whole rank step starves the blit kernels of concurrent
        // deliveries (its workgroups can take every register of a CU; measured: the copies then crawl on the
        // few CUs left over and the kernel's bounded waits time out).  So the deliveries are enqueued before it.
        if (!(flags & (CF_SERIAL | CF_NO_COPY | CF_NO_COMPUTE)) && xs != cs && r.p > 1 &&
            !((kind == CF_KIND_RS || kind == CF_KIND_AG) && attn == nullptr))
            return fail(CF_ERR_UNSUPPORTED, "CF_PERSISTENT needs CF_SERIAL for this kind (the deliveries are enqueued before the kernel)");
    }
    if (cf_status st = check_buffers(r, kind, bufs, flags))
        return st;
    if (!(flags & CF_GRAPH))
        return (flags & CF_PERSISTENT) ? enqueue_persistent(r, kind, bufs, cs, xs, flags, attn)
                                       : enqueue_schedule(r, kind, bufs, cs, xs, flags, attn);

    // CF_GRAPH: the same enqueue sequence, captured once per distinct argument set.
    if (cs == nullptr || (xs == nullptr && !(flags & CF_SERIAL)))
        return fail(CF_ERR_INVALID_ARG, "CF_GRAPH needs explicit (non-default) streams");
    append_bytes(key, &kind, sizeof(kind));
    append_bytes(key, &flags, sizeof(flags));
    append_bytes(key, &cs, sizeof(cs));
    append_bytes(key, &xs, sizeof(xs));
    append_bytes(key, &bufs->A_or_own_shard, sizeof(void *));
    append_bytes(key, &bufs->W, sizeof(void *));
    append_bytes(key, &bufs->O, sizeof(void *));
    append_bytes(key, bufs->slot, sizeof(bufs->slot));
    append_bytes(key, bufs->send_slot, sizeof(bufs->send_slot));
    if (attn != nullptr) {
        append_bytes(key, &attn->ap.Q, sizeof(void *));
        append_bytes(key, &attn->ap.K, sizeof(void *));
        append_bytes(key, &attn->ap.V, sizeof(void *));
        append_bytes(key, &attn->ap.out, sizeof(void *));
    }
    {   // so are the tuning overrides (tile shape, k-split, work-item order, spin limit, ...)
        const cf::Tuning tn = cf::tuning();
        append_bytes(key, &tn, sizeof(tn));
    }
    {   // the registered workspace is baked into the captured kernels (split-K partials, delivery flags)
        const Workspace ws = workspace_for(cs);
        append_bytes(key, &ws.ptr, sizeof(ws.ptr));
        append_bytes(key, &ws.bytes, sizeof(ws.bytes));
    }
    for (int i = 0; i < r.p - 1; ++i) {
        const void *st = bufs->peer_stage ? bufs->peer_stage[i] : nullptr;
        const void *sk = bufs->peer_sink ? bufs->peer_sink[i] : nullptr;
        const void *re = bufs->recv_each ? bufs->recv_each[i] : nullptr;
        const void *se = bufs->send_each ? bufs->send_each[i] : nullptr;
        append_bytes(key, &st, sizeof(st));
        append_bytes(key, &sk, sizeof(sk));
        append_bytes(key, &re, sizeof(re));
        append_bytes(key, &se, sizeof(se));
    }
    hipGraphExec_t exec = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_graphs.find(key);
        if (it != g_graphs.end())
            exec = it->second.exec;
        else if (g_graphs.size() >= MAX_GRAPHS)
            return fail(CF_ERR_INVALID_ARG, "CF_GRAPH: %zu captured argument sets are cached already; call "
                                            "commfuse_destroy_cache() to release them", g_graphs.size());
    }
    if (exec == nullptr) {
        // events must exist before capture starts (creation is not a capturable operation)
        std::vector<hipEvent_t> tmp;
        if (cf_status st = get_events(2 + 3 * (size_t)r.p * r.m, &tmp))
            return st;
        CF_HIP(hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal));
        const uint32_t fl = flags & ~(uint32_t)CF_GRAPH;
        cf_status st = (fl & CF_PERSISTENT) ? enqueue_persistent(r, kind, bufs, cs, xs, fl, attn)
                                            : enqueue_schedule(r, kind, bufs, cs, xs, fl, attn);
        hipGraph_t graph = nullptr;
        hipError_t e = hipStreamEndCapture(cs, &graph);
        if (st != CF_OK) {
            if (graph)
                (void)hipGraphDestroy(graph);
            return st;
        }
        if (e != hipSuccess)
            return fail_hip(e, "hipStreamEndCapture");
        e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        if (e != hipSuccess) {
            (void)hipGraphDestroy(graph);
            return fail_hip(e, "hipGraphInstantiate");
        }
        std::lock_guard<std::mutex> lk(g_mu);
        g_graphs.emplace(key, GraphEntry{graph, exec});
    }
    CF_HIP(hipGraphLaunch(exec, cs));
    return CF_OK;
}

// cf_attn_desc -> the reduce-scatter layer it projects into, and the attention geometry.
cf_status resolve_attn(const cf_attn_desc *d, Resolved *out, cf::AttnParams *ap)
{
    if (d == nullptr)
        return fail(CF_ERR_NULL_PTR, "descriptor is NULL");
    if (d->p < 1 || d->rank < 0 || d->rank >= d->p)
        return fail(CF_ERR_INVALID_ARG, "need p >= 1 and rank in [0, p)");
    if (d->batch < 1 || d->heads < 1 || d->seq < 1 || d->n < 0)
        return fail(CF_ERR_INVALID_ARG, "batch, heads and seq must be positive, n non-negative");
    if (d->seq % d->p != 0)
        return fail(CF_ERR_INVALID_ARG, "p = %d must divide the sequence length %d", d->p, d->seq);
    if (d->head_dim != 128)
        return fail(CF_ERR_UNSUPPORTED, "head_dim %d: the attention kernel is written for 128", d->head_dim);
    if (!(d->scale > 0.0f) || !(d->scale < 1e30f))
        return fail(CF_ERR_INVALID_ARG, "scale must be a positive finite number");
    cf_layer_desc ld;
    memset(&ld, 0, sizeof(ld));
    ld.p = d->p;
    ld.rank = d->rank;
    ld.m_chunk = (int64_t)d->batch * (d->seq / d->p);
    ld.n = d->n;
    ld.k = (int64_t)d->heads * d->head_dim;
    ld.ldw = d->ldw;
    ld.ldo = d->ldo;
    ld.in_dtype = CF_BF16;
    ld.out_dtype = CF_F32;
    ld.w_layout = d->w_layout;
    if (cf_status st = resolve(&ld, CF_KIND_RS, out))
        return st;
    ap->Q = ap->K = ap->V = nullptr;
    ap->out = nullptr;
    ap->batch = d->batch;
    ap->heads = d->heads;
    ap->S = d->seq;
    ap->head_dim = d->head_dim;
    ap->c = d->seq / d->p;
    ap->l = 0;
    ap->ldo = out->k;                              // attention output rows are the projection's packed left operand
    ap->scale = d->scale;
    if (!cf::attn_slice_supported(*ap))
        return fail(CF_ERR_UNSUPPORTED, "a (batch, head) matrix of K or V must stay below 2 GiB");
    return CF_OK;
}

cf_status check_attn_ptrs(const void *Q, const void *K, const void *V, const void *attn_out)
{
    if (Q == nullptr || K == nullptr || V == nullptr || attn_out == nullptr)
        return fail(CF_ERR_NULL_PTR, "Q, K, V and attn_out must not be NULL");
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(attn_out))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    return CF_OK;
}

}  // namespace

namespace cf {

static Tuning read_tuning_from_environment()
{
    Tuning t;
    memset(&t, 0, sizeof(t));                      // (padding too: the struct is hashed byte-wise into graph keys)
    t.deep = t.prefetch = t.xcd_steps = t.k_rotate = t.stream_recv = t.attn_qt = t.carry = t.mfma16 = -1;
    int bm = 0, bn = 0;
    if (const char *e = getenv("COMMFUSE_TILE"))
        if (sscanf(e, "%dx%d", &bm, &bn) == 2) {
            t.tile_bm = bm;
            t.tile_bn = bn;
        }
    if (const char *e = getenv("COMMFUSE_DEEP"))
        t.deep = atoi(e) != 0;
    if (const char *e = getenv("COMMFUSE_SPLITK")) {
        const int sk = atoi(e);
        if (sk >= 1 && sk <= 8)
            t.splitk = sk;
    }
    if (const char *e = getenv("COMMFUSE_KERNEL"))
        t.staged = strcmp(e, "staged") == 0;
    if (const char *e = getenv("COMMFUSE_PREFETCH"))
        t.prefetch = atoi(e) < 0 ? 0 : atoi(e);
    if (const char *e = getenv("COMMFUSE_XCD_STEPS"))
        t.xcd_steps = atoi(e) != 0;
    if (const char *e = getenv("COMMFUSE_K_ROTATE"))
        t.k_rotate = atoi(e) != 0;
    if (const char *e = getenv("COMMFUSE_XCD_BANDS")) {
        const int v = atoi(e);
        t.xcd_bands = (v == 1 || v == 2 || v == 4) ? v : 0;
    }
    if (const char *e = getenv("COMMFUSE_CARRY"))
        t.carry = atoi(e) != 0;
    if (const char *e = getenv("COMMFUSE_MFMA16"))
        t.mfma16 = atoi(e) != 0;
    if (const char *e = getenv("COMMFUSE_PERSIST_WGS"))
        t.persist_wgs = atoi(e) > 0 ? atoi(e) : 0;
    if (const char *e = getenv("COMMFUSE_STREAM_RECV"))
        t.stream_recv = atoi(e) != 0;
    if (const char *e = getenv("COMMFUSE_TILE_F32"))
        if (sscanf(e, "%dx%d", &bm, &bn) == 2)
            t.tile_f32_bm = bm;
    if (const char *e = getenv("COMMFUSE_SPIN_LIMIT")) {
        const long v = atol(e);
        if (v > 0)
            t.spin_limit = (unsigned)v;
    }
    if (const char *e = getenv("COMMFUSE_ATTN_QT"))
        t.attn_qt = atoi(e);
    if (const char *e = getenv("COMMFUSE_ATTN_WAVES"))
        t.attn_waves = atoi(e) == 8 ? 8 : 4;
    if (const char *e = getenv("COMMFUSE_ATTN_KSPLIT"))
        t.attn_ksplit = atoi(e);
    return t;
}

Tuning tuning()
{
    static const bool live = [] {
        const char *e = getenv("COMMFUSE_TUNING_LIVE");
        return e != nullptr && atoi(e) != 0;
    }();
    static const Tuning once = read_tuning_from_environment();
    return live ? read_tuning_from_environment() : once;
}

}  // namespace cf

extern "C" {

int commfuse_version(void) { return 100; }

const char *commfuse_last_error(void) { return g_err; }

int commfuse_chunk_index(int kind, int p, int rank, int step)
{
    if (!known_kind(kind))
        return fail(CF_ERR_INVALID_ARG, "kind %d", kind);
    if (p < 1 || rank < 0 || rank >= p || step < 0 || step >= p)
        return fail(CF_ERR_INVALID_ARG, "need p >= 1, rank and step in [0, p)");
    if (is_pair_kind(kind)) {
        if (cf_status st = check_pair_p(p))
            return st;
        return pair_slice(p, rank, step);
    }
    return chunk_index(kind, p, rank, step);
}

int commfuse_subslice_index(int kind, int p, int m, int rank, int step)
{
    if (kind != CF_KIND_RS && kind != CF_KIND_AG && kind != CF_KIND_DP)
        return fail(CF_ERR_INVALID_ARG, "kind %d (ring kinds only)", kind);
    if (p < 1 || m < 1 || m > 4096 || rank < 0 || rank >= p || step < 0 || step >= p * m)
        return fail(CF_ERR_INVALID_ARG, "need p >= 1, m in [1, 4096], rank in [0, p), step in [0, m*p)");
    return subslice_index(kind, p, m, rank, step);
}

int commfuse_pair_partner(int p, int rank, int round)
{
    if (p < 2 || (p & 1))
        return fail(CF_ERR_INVALID_ARG, "the pairwise schedule needs an even p >= 2, not %d", p);
    if (rank < 0 || rank >= p || round < 1 || round > p - 1)
        return fail(CF_ERR_INVALID_ARG, "need rank in [0, p) and round in [1, p-1]");
    return pair_partner(p, rank, round);
}

cf_status commfuse_rs_pair_step(const cf_layer_desc *desc, int step, const void *A, const void *W,
                                const float *recv, float *acc, float *out, void *hip_stream)
{
    Resolved r;
    if (cf_status st = resolve(desc, CF_KIND_RS_PAIR, &r))
        return st;
    return rs_pair_step_impl(r, step, A, W, recv, acc, out, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_rs_pair_last_step(const cf_layer_desc *desc, const void *A, const void *W,
                                     const float *const *recv_each, float *out, void *hip_stream)
{
    Resolved r;
    if (cf_status st = resolve(desc, CF_KIND_RS_PAIR, &r))
        return st;
    return rs_pair_last_step_impl(r, A, W, recv_each, out, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_wgrad_step(const cf_layer_desc *desc, int step, const void *left, const void *right, float *dW,
                              void *hip_stream)
{
    Resolved r;
    if (cf_status st = resolve(desc, CF_KIND_WGRAD_X, &r))
        return st;
    return wgrad_step_impl(r, step, left, right, dW, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_dp_pair_step(int p, int rank, int step, float *bucket, int64_t chunk_elems, const float *recv,
                                void *hip_stream)
{
    return dp_pair_step_impl(p, rank, step, bucket, chunk_elems, recv, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_rs_step(const cf_layer_desc *desc, int step, const void *A, const void *W, const float *recv,
                           float *out, void *hip_stream)
{
    Resolved r;
    if (cf_status st = resolve(desc, CF_KIND_RS, &r))
        return st;
    return rs_step_impl(r, step, A, W, recv, out, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_rs_step_noalloc(const cf_layer_desc *desc, int step, const void *A, const void *W,
                                   const float *recv, float *out, void *hip_stream)
{
    Resolved r;
    if (cf_status st = resolve(desc, CF_KIND_RS, &r))
        return st;
    // the largest step whose k-split partials fit the library's scratch for every split choice
    if ((size_t)r.mc * (size_t)r.n * sizeof(float) * WS_MAX_SPLITS > STATIC_PARTIAL_BYTES)
        return fail(CF_ERR_INVALID_ARG,
                    "commfuse_rs_step_noalloc: a step output of %lld x %lld fp32 elements exceeds the static scratch "
                    "(at most %zu elements per step); use commfuse_rs_step with a registered workspace",
                    (long long)r.mc, (long long)r.n, STATIC_PARTIAL_BYTES / sizeof(float) / WS_MAX_SPLITS);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Workspace own;
    if (cf_status st = static_scratch_of_current_device(s, &own))
        return st;
    return rs_step_impl(r, step, A, W, recv, out, s, nullptr, &own);
}

cf_status commfuse_ag_step(const cf_layer_desc *desc, int step, const void *shard, const void *W, void *O,
                           void *hip_stream)
{
    Resolved r;
    if (cf_status st = resolve(desc, CF_KIND_AG, &r))
        return st;
    return ag_step_impl(r, step, shard, W, O, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_dp_reduce_step(int p, int rank, int step, float *bucket, int64_t chunk_elems, const float *recv,
                                  void *hip_stream)
{
    return dp_step_impl(p, rank, step, bucket, chunk_elems, recv, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_run_schedule(const cf_layer_desc *desc, int kind, const cf_buffers *bufs, void *compute_stream,
                                void *copy_stream, uint32_t flags)
{
    if (!known_kind(kind))
        return fail(CF_ERR_INVALID_ARG, "kind %d", kind);
    Resolved r;
    if (cf_status st = resolve(desc, kind, &r))
        return st;
    std::vector<unsigned char> key;
    append_bytes(key, desc, sizeof(*desc));
    return run_schedule_common(r, kind, bufs, static_cast<hipStream_t>(compute_stream),
                               static_cast<hipStream_t>(copy_stream), flags, nullptr, key);
}

cf_status commfuse_attn_slice(const cf_attn_desc *desc, int slice, const void *Q, const void *K, const void *V,
                              void *attn_out, void *hip_stream)
{
    Resolved r;
    AttnCtx ctx;
    if (cf_status st = resolve_attn(desc, &r, &ctx.ap))
        return st;
    if (slice < 0 || slice >= r.p)
        return fail(CF_ERR_INVALID_ARG, "slice = %d not in [0, %d)", slice, r.p);
    if (cf_status st = check_attn_ptrs(Q, K, V, attn_out))
        return st;
    ctx.ap.Q = Q;
    ctx.ap.K = K;
    ctx.ap.V = V;
    ctx.ap.out = attn_out;
    return launch_attention(ctx, slice, static_cast<hipStream_t>(hip_stream));
}

cf_status commfuse_attn_rs_step(const cf_attn_desc *desc, int step, const void *Q, const void *K, const void *V,
                                const void *Wo, const float *recv, float *out, void *attn_out, void *hip_stream)
{
    Resolved r;
    AttnCtx ctx;
    if (cf_status st = resolve_attn(desc, &r, &ctx.ap))
        return st;
    if (cf_status st = check_step(r, step))
        return st;
    if (cf_status st = check_attn_ptrs(Q, K, V, attn_out))
        return st;
    if (Wo == nullptr || out == nullptr)
        return fail(CF_ERR_NULL_PTR, "Wo and out must not be NULL");
    if (step == 0 && recv != nullptr)
        return fail(CF_ERR_NULL_PTR, "recv must be NULL at step 0 (nothing has been received yet)");
    if (step > 0 && recv == nullptr)
        return fail(CF_ERR_NULL_PTR, "recv must not be NULL at step %d", step);
    if (recv == out)
        return fail(CF_ERR_INVALID_ARG, "out may not alias recv");
    if (!aligned16(Wo) || !aligned16(out) || !aligned16(recv))
        return fail(CF_ERR_MISALIGNED, "tensor pointers must be 16-byte aligned");
    ctx.ap.Q = Q;
    ctx.ap.K = K;
    ctx.ap.V = V;
    ctx.ap.out = attn_out;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (cf_status st = launch_attention(ctx, chunk_index(CF_KIND_RS, r.p, r.rank, step), s))
        return st;
    return launch_gemm(r, attn_out, Wo, recv, out, s);
}

cf_status commfuse_run_attn_schedule(const cf_attn_desc *desc, const cf_attn_buffers *ab, void *compute_stream,
                                     void *copy_stream, uint32_t flags)
{
    Resolved r;
    AttnCtx ctx;
    if (cf_status st = resolve_attn(desc, &r, &ctx.ap))
        return st;
    if (ab == nullptr)
        return fail(CF_ERR_NULL_PTR, "buffers is NULL");
    if (cf_status st = check_attn_ptrs(ab->Q, ab->K, ab->V, ab->attn_out))
        return st;
    ctx.ap.Q = ab->Q;
    ctx.ap.K = ab->K;
    ctx.ap.V = ab->V;
    ctx.ap.out = ab->attn_out;
    cf_buffers b;
    memset(&b, 0, sizeof(b));
    b.A_or_own_shard = ab->attn_out;
    b.W = ab->Wo;
    b.O = ab->O;
    b.peer_stage = ab->peer_stage;
    b.slot[0] = ab->slot[0];
    b.slot[1] = ab->slot[1];
    b.send_slot[0] = ab->send_slot[0];
    b.send_slot[1] = ab->send_slot[1];
    b.peer_sink = ab->peer_sink;
    b.recv_each = ab->recv_each;
    b.send_each = ab->send_each;
    std::vector<unsigned char> key;
    append_bytes(key, desc, sizeof(*desc));
    const char tag[8] = "attn";
    append_bytes(key, tag, sizeof(tag));
    return run_schedule_common(r, CF_KIND_RS, &b, static_cast<hipStream_t>(compute_stream),
                               static_cast<hipStream_t>(copy_stream), flags, &ctx, key);
}

size_t commfuse_workspace_bytes(const cf_layer_desc *desc, int kind)
{
    Resolved r;
    if (is_wgrad_kind(kind)) {                     // k-splits of a [k x n] gradient tile
        if (resolve(desc, kind, &r) != CF_OK || !r.bf16_in)
            return 0;
        return WS_COUNTER_BYTES + (size_t)WS_MAX_SPLITS * (size_t)r.k * (size_t)r.n * sizeof(float);
    }
    if (kind != CF_KIND_RS && kind != CF_KIND_AG && kind != CF_KIND_RS_PAIR)
        return 0;                                  // the gradient path needs none
    if (resolve(desc, kind, &r) != CF_OK || !r.bf16_in)
        return 0;
    return WS_COUNTER_BYTES + (size_t)WS_MAX_SPLITS * (size_t)r.mc * (size_t)r.n * sizeof(float);
}

cf_status commfuse_set_workspace(void *device_ptr, size_t bytes, void *hip_stream)
{
    hipStream_t key = static_cast<hipStream_t>(hip_stream);
    if (device_ptr == nullptr || bytes == 0) {
        std::lock_guard<std::mutex> lk(g_ws_mu);
        if (key != nullptr)
            g_ws_of_stream.erase(key);
        else
            g_ws = Workspace{};
        return CF_OK;
    }
    if (!aligned16(device_ptr))
        return fail(CF_ERR_MISALIGNED, "workspace must be 16-byte aligned");
    if (bytes <= WS_COUNTER_BYTES)
        return fail(CF_ERR_INVALID_ARG, "workspace must exceed %zu bytes", WS_COUNTER_BYTES);
    // arrival counters start at zero; the kernels leave them at zero
    CF_HIP(hipMemsetAsync(device_ptr, 0, WS_COUNTER_BYTES, static_cast<hipStream_t>(hip_stream)));
    std::lock_guard<std::mutex> lk(g_ws_mu);
    Workspace &w = key != nullptr ? g_ws_of_stream[key] : g_ws;
    w.ptr = device_ptr;
    w.bytes = bytes;
    return CF_OK;
}

cf_status commfuse_device_status(void *hip_stream)
{
    void *ws = workspace_for(static_cast<hipStream_t>(hip_stream)).ptr;
    if (ws == nullptr)
        return CF_OK;
    unsigned word = 0;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    CF_HIP(hipMemcpyAsync(&word, static_cast<char *>(ws) + WS_STATUS_OFFSET, sizeof(word), hipMemcpyDeviceToHost, s));
    CF_HIP(hipStreamSynchronize(s));
    if (word != 0) {
        CF_HIP(hipMemsetAsync(static_cast<char *>(ws) + WS_STATUS_OFFSET, 0, sizeof(word), s));
        CF_HIP(hipStreamSynchronize(s));
        return fail(CF_ERR_HIP, "a step kernel gave up waiting for its delivery (status 0x%x): results are invalid", word);
    }
    return CF_OK;
}

void commfuse_destroy_cache(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto &kv : g_graphs) {
        (void)hipGraphExecDestroy(kv.second.exec);
        (void)hipGraphDestroy(kv.second.graph);
    }
    g_graphs.clear();
    for (auto &kv : g_events)
        for (hipEvent_t ev : kv.second)
            (void)hipEventDestroy(ev);
    g_events.clear();
}

}  // extern "C"

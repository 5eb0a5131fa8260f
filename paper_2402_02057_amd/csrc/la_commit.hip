// Appending the accepted tokens of a step to the KV cache (the step's own keys and values of
// those rows become prefix rows of the next step: Sec. 3.3 evaluates the candidates at the
// positions they will hold once accepted, so nothing is recomputed).
//
// A copy of at most N rows per KV head, driven by the device-side result of la_verify_step:
// one workgroup per appended row, 16 bytes per thread and trip.
#include "la_internal.h"
#include "la_rope_common.h"

namespace la {
namespace {

struct CommitParams {
    unsigned char* k_cache;
    unsigned char* v_cache;
    const unsigned char* step_k;
    const unsigned char* step_v;
    const int* best;
    const int* n_out;
    long long capacity;   // rows per KV head in the cache
    const int* block_table;  // paged cache (else nullptr): [n_pages][kv_heads][page_size][head_dim]
    int page_size, n_pages;
    int P, W, N, G, kv_heads;
    int row_bytes;        // head_dim * 2
};

__device__ __forceinline__ void commit_row(const CommitParams& p, int i)
{
    // i-th appended row: cache row P + i
    int n = *p.n_out;
    n = n < 1 ? 1 : (n > p.N ? p.N : n);    // (a valid result is 1..N; never index past the step)
    if (i >= n) return;
    int src = 0;                            // step row it comes from: the current token ...
    if (i > 0) {                            // ... or token i-1 of the winning candidate
        int g = *p.best;
        g = g < 0 ? 0 : (g >= p.G ? p.G - 1 : g);
        if (p.G == 0) return;               // (cannot happen with n > 1)
        src = 1 + p.W * (p.N - 1) + g * (p.N - 1) + (i - 1);
    }
    const int pieces = p.row_bytes / 16;    // 16-byte pieces per head row
    for (int x = threadIdx.x; x < p.kv_heads * pieces; x += blockDim.x) {
        const int h = x / pieces, c = x - h * pieces;
        const size_t from = ((size_t)src * p.kv_heads + h) * p.row_bytes + (size_t)c * 16;
        size_t to_row;
        if (p.block_table) {   // (the host checked that the table covers P + N rows; entries are clamped)
            const int t = p.P + i;
            int page = p.block_table[t / p.page_size];
            page = page < 0 ? 0 : (page >= p.n_pages ? p.n_pages - 1 : page);
            to_row = ((size_t)page * p.kv_heads + h) * (size_t)p.page_size + (size_t)(t % p.page_size);
        } else {
            to_row = (size_t)h * (size_t)p.capacity + (size_t)(p.P + i);
        }
        const size_t to = to_row * p.row_bytes + (size_t)c * 16;
        *reinterpret_cast<uint4*>(p.k_cache + to) = *reinterpret_cast<const uint4*>(p.step_k + from);
        *reinterpret_cast<uint4*>(p.v_cache + to) = *reinterpret_cast<const uint4*>(p.step_v + from);
    }
}

__global__ __launch_bounds__(256) void kv_commit_kernel(CommitParams p) { commit_row(p, blockIdx.x); }

// The same append for a step whose keys were left unrotated in memory (the attention kernel turned
// them on the way in): the key rows are turned here, by the position they take in the cache, P + i,
// which is the position the step evaluated them at (current token: P; token i - 1 of a candidate:
// P + i).  A work item is eight pairs of one KV head's key row, with the arithmetic of the pass of
// its own, and the same two 16-byte pieces of the value row, copied as they are.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
struct CommitRope {
    const float* cos;
    const float* sin;
    int interleaved;
};

__global__ __launch_bounds__(256) void kv_commit_rope_kernel(CommitParams p, CommitRope rp)
{
    const int i = blockIdx.x;
    int n = *p.n_out;
    n = n < 1 ? 1 : (n > p.N ? p.N : n);
    if (i >= n) return;
    int src = 0;
    if (i > 0) {
        int g = *p.best;
        g = g < 0 ? 0 : (g >= p.G ? p.G - 1 : g);
        if (p.G == 0) return;
        src = 1 + p.W * (p.N - 1) + g * (p.N - 1) + (i - 1);
    }
    const int units = p.row_bytes / 32;     // units of eight pairs per head row
    const float* cs = rp.cos + (size_t)(p.P + i) * (p.row_bytes / 4);
    const float* sn = rp.sin + (size_t)(p.P + i) * (p.row_bytes / 4);
    for (int x = threadIdx.x; x < p.kv_heads * units; x += blockDim.x) {
        const int h = x / units, c = x - h * units;
        const int pa = rp.interleaved ? 2 * c : c, pb = rp.interleaved ? 2 * c + 1 : c + units;
        const size_t from = ((size_t)src * p.kv_heads + h) * p.row_bytes;
        const size_t to = ((size_t)h * (size_t)p.capacity + (size_t)(p.P + i)) * p.row_bytes;
        const bf16x8 xa = *reinterpret_cast<const bf16x8*>(p.step_k + from + pa * 16);
        const bf16x8 xb = *reinterpret_cast<const bf16x8*>(p.step_k + from + pb * 16);
        const float4 c0 = *reinterpret_cast<const float4*>(cs + c * 8), c1 = *reinterpret_cast<const float4*>(cs + c * 8 + 4);
        const float4 s0 = *reinterpret_cast<const float4*>(sn + c * 8), s1 = *reinterpret_cast<const float4*>(sn + c * 8 + 4);
        const float co[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        const float si[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        bf16x8 ya, yb;
        rope_eight_pairs(xa, xb, co, si, rp.interleaved != 0, ya, yb);
        *reinterpret_cast<bf16x8*>(p.k_cache + to + pa * 16) = ya;
        *reinterpret_cast<bf16x8*>(p.k_cache + to + pb * 16) = yb;
        *reinterpret_cast<uint4*>(p.v_cache + to + pa * 16) = *reinterpret_cast<const uint4*>(p.step_v + from + pa * 16);
        *reinterpret_cast<uint4*>(p.v_cache + to + pb * 16) = *reinterpret_cast<const uint4*>(p.step_v + from + pb * 16);
    }
}

// Several appends in one launch (the layers of a model after a step, or several sequences):
// blockIdx.y names the append, blockIdx.x its row.  What differs between appends travels as a
// kernel argument, kCommitBatch of them at a time.
constexpr int kCommitBatch = 32;
struct CommitOne {
    unsigned char* k_cache;
    unsigned char* v_cache;
    const unsigned char* step_k;
    const unsigned char* step_v;
    const int* best;
    const int* n_out;
    const int* block_table;
    long long capacity;
    int P;
};
struct CommitBatchParams {
    CommitOne one[kCommitBatch];
    int page_size, n_pages, W, N, G, kv_heads, row_bytes;
};

__global__ __launch_bounds__(256) void kv_commit_batch_kernel(CommitBatchParams b)
{
    const CommitOne& o = b.one[blockIdx.y];
    CommitParams p;
    p.k_cache = o.k_cache;
    p.v_cache = o.v_cache;
    p.step_k = o.step_k;
    p.step_v = o.step_v;
    p.best = o.best;
    p.n_out = o.n_out;
    p.capacity = o.capacity;
    p.block_table = o.block_table;
    p.page_size = b.page_size;
    p.n_pages = b.n_pages;
    p.P = o.P; p.W = b.W; p.N = b.N; p.G = b.G; p.kv_heads = b.kv_heads;
    p.row_bytes = b.row_bytes;
    commit_row(p, blockIdx.x);
}

}  // namespace

la_status launch_kv_commit(void* k_cache, void* v_cache, long long capacity, const int* block_table,
                           int page_size, int n_pages, const void* step_k, const void* step_v, int P, int W,
                           int N, int G, int kv_heads, int head_dim, const int* best, const int* n_out,
                           hipStream_t stream)
{
    CommitParams p;
    p.k_cache = (unsigned char*)k_cache;
    p.v_cache = (unsigned char*)v_cache;
    p.step_k = (const unsigned char*)step_k;
    p.step_v = (const unsigned char*)step_v;
    p.best = best;
    p.n_out = n_out;
    p.capacity = capacity;
    p.block_table = block_table;
    p.page_size = page_size;
    p.n_pages = n_pages;
    p.P = P; p.W = W; p.N = N; p.G = G; p.kv_heads = kv_heads;
    p.row_bytes = head_dim * 2;
    hipLaunchKernelGGL(kv_commit_kernel, dim3((unsigned)N), dim3(256), 0, stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_kv_commit launch: %s", hipGetErrorString(e));
    return LA_OK;
}

la_status launch_kv_commit_rope(void* k_cache, void* v_cache, long long capacity, const void* step_k,
                                const void* step_v, const float* cos, const float* sin, int interleaved, int P,
                                int W, int N, int G, int kv_heads, int head_dim, const int* best, const int* n_out,
                                hipStream_t stream)
{
    CommitParams p;
    p.k_cache = (unsigned char*)k_cache;
    p.v_cache = (unsigned char*)v_cache;
    p.step_k = (const unsigned char*)step_k;
    p.step_v = (const unsigned char*)step_v;
    p.best = best;
    p.n_out = n_out;
    p.capacity = capacity;
    p.block_table = nullptr;
    p.page_size = 0;
    p.n_pages = 0;
    p.P = P; p.W = W; p.N = N; p.G = G; p.kv_heads = kv_heads;
    p.row_bytes = head_dim * 2;
    CommitRope rp;
    rp.cos = cos;
    rp.sin = sin;
    rp.interleaved = interleaved;
    hipLaunchKernelGGL(kv_commit_rope_kernel, dim3((unsigned)N), dim3(256), 0, stream, p, rp);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_kv_commit_rope launch: %s", hipGetErrorString(e));
    return LA_OK;
}

la_status launch_kv_commit_batch(const CommitSeq* seqs, int n_seqs, int page_size, int n_pages, int W, int N,
                                 int G, int kv_heads, int head_dim, hipStream_t stream)
{
    for (int i0 = 0; i0 < n_seqs; i0 += kCommitBatch) {
        const int n = n_seqs - i0 < kCommitBatch ? n_seqs - i0 : kCommitBatch;
        CommitBatchParams b;
        for (int i = 0; i < n; ++i) {
            const CommitSeq& s = seqs[i0 + i];
            CommitOne& o = b.one[i];
            o.k_cache = (unsigned char*)s.k_cache;
            o.v_cache = (unsigned char*)s.v_cache;
            o.step_k = (const unsigned char*)s.step_k;
            o.step_v = (const unsigned char*)s.step_v;
            o.best = s.best;
            o.n_out = s.n_out;
            o.block_table = s.block_table;
            o.capacity = s.capacity;
            o.P = s.P;
        }
        for (int i = n; i < kCommitBatch; ++i) b.one[i] = b.one[0];  // never indexed: the grid has n layers
        b.page_size = page_size; b.n_pages = n_pages;
        b.W = W; b.N = N; b.G = G; b.kv_heads = kv_heads;
        b.row_bytes = head_dim * 2;
        hipLaunchKernelGGL(kv_commit_batch_kernel, dim3((unsigned)N, (unsigned)n), dim3(256), 0, stream, b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(LA_EHIP, "la_kv_commit_batch launch: %s", hipGetErrorString(e));
    }
    return LA_OK;
}

}  // namespace la

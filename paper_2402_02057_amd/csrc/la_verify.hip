// Greedy verification reduction for gfx950: per-row argmax over the vocabulary and the
// longest accepted prefix of every candidate n-gram (Sec. 2 "Guess-And-Verify"; the
// accept/stop rule Algorithm 3 applies to each candidate), in one launch.
//
// A workgroup of 16 waves scans one segment of one logits row - up to 32768 elements, so a
// whole row of a 32000-entry vocabulary - with every 16-byte load requested before the first
// comparison.  (Many small segments would fill the machine better, but each costs device-scope
// atomics on a handful of addresses, and those serialise: measured, they dominated.)  A
// segment's winner is folded into one 64-bit key per row with atomicMax,
//     key = (order-preserving image of the fp32 value) << 32 | (0xFFFFFFFF - index),
// so the largest value wins and, among equal values, the lowest index: the result does
// not depend on the order in which workgroups finish.  Each candidate has a ticket counter;
// the workgroup that finishes last among a candidate's (N-1) x segments workgroups turns that
// candidate's keys into `accepted` and `accept_len` and zeroes keys and ticket again, so the
// workspace is clean for the next call without a memset.  Keys and tickets are touched only
// by device-scope atomics that return their old value (the ticket is taken after the key
// update has come back), so no cache write-back or invalidate is needed: those cost tens of
// microseconds on this part, more than the whole scan.
//
// verify_step_kernel ends a greedy step in one launch (Algorithm 3 in full, plus the greedy
// tokens of Algorithm 2's lookahead branch): the same row scan over 1 + W + G(N-1) rows, a
// two-level ticket (eight workgroups per first-level counter, so that no address sees more than
// a handful of atomics), and the workgroup that arrives last reads all row maxima at once and
// walks the candidates.
#include "la_internal.h"

namespace la {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kVecPerThread = 8;                          // float4 loads in flight per thread
constexpr int kMaxSeg = kThreads * kVecPerThread * 4;     // elements per segment

__device__ __forceinline__ unsigned long long pack_key(float v, int idx)
{
    if (v == 0.0f) v = 0.0f;  // -0.0 and +0.0 compare equal: give them one image
    unsigned b = __float_as_uint(v);
    unsigned ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return ((unsigned long long)ord << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)idx);
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long x, int mask)
{
    unsigned lo = __shfl_xor((unsigned)x, mask, 64);
    unsigned hi = __shfl_xor((unsigned)(x >> 32), mask, 64);
    return ((unsigned long long)hi << 32) | lo;
}

// The largest value of p[v0 .. v1) with the lowest index among equals, as a packed key, in every
// lane of each wave (waves still have to be combined).  Per thread, indices are visited in
// increasing order and only a strictly larger value replaces the best, so the earliest of equal
// values is kept.
template <bool kVec>
__device__ __forceinline__ unsigned long long scan_segment(const float* __restrict__ p, int v0, int v1, int tid)
{
    float best = 0.0f;
    int best_idx = -1;
    if (kVec) {
        const float4* p4 = reinterpret_cast<const float4*>(p) + (v0 >> 2);
        const int nvec = (v1 - v0) >> 2;  // V % 4 == 0 on this path; nvec >= 1
        float4 x[kVecPerThread];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) x[j] = p4[min(tid + j * kThreads, nvec - 1)];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
            const int i = tid + j * kThreads;
            if (i < nvec) {
                const int base = v0 + (i << 2);
                if (best_idx < 0) { best = x[j].x; best_idx = base; }
                if (x[j].x > best) { best = x[j].x; best_idx = base; }
                if (x[j].y > best) { best = x[j].y; best_idx = base + 1; }
                if (x[j].z > best) { best = x[j].z; best_idx = base + 2; }
                if (x[j].w > best) { best = x[j].w; best_idx = base + 3; }
            }
        }
    } else {
        for (int i = v0 + tid; i < v1; i += kThreads) {
            const float x = p[i];
            if (best_idx < 0 || x > best) { best = x; best_idx = i; }
        }
    }
    unsigned long long key = best_idx < 0 ? 0ull : pack_key(best, best_idx);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const unsigned long long o = shfl_xor_u64(key, m);
        key = o > key ? o : key;
    }
    return key;
}

// rows = G * n1 logits rows of V floats; row r is cut into nseg segments of seg_len
// (a multiple of 4) elements; blockIdx.x = r * nseg + segment.
template <bool kVec>
__global__ __launch_bounds__(kThreads) void verify_kernel(
    const float* __restrict__ logits, const int* __restrict__ cand_tokens, int G, int n1, int V,
    int seg_len, int nseg, unsigned long long* keys, unsigned* tickets,
    int* __restrict__ accept_len, int* __restrict__ accepted)
{
    const int row = blockIdx.x / nseg;
    const int seg = blockIdx.x - row * nseg;
    const int v0 = seg * seg_len;
    const int v1 = min(V, v0 + seg_len);
    const float* p = logits + (size_t)row * V;
    const int tid = threadIdx.x;

    const unsigned long long key = scan_segment<kVec>(p, v0, v1, tid);
    __shared__ unsigned long long wave_key[kWaves];
    __shared__ unsigned last_flag;
    if ((tid & 63) == 0) wave_key[tid >> 6] = key;
    __syncthreads();
    if (tid == 0) {
        unsigned long long k = wave_key[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) k = wave_key[w] > k ? wave_key[w] : k;
        // returning atomics: the ticket is requested only after the key update has come back
        const unsigned long long before = atomicMax(&keys[row], k);
        asm volatile("" ::"v"((unsigned)before) : "memory");  // consume the returned value first
        const int g = row / n1;
        const unsigned t = atomicAdd(&tickets[g], 1u);
        last_flag = (t == (unsigned)(n1 * nseg) - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!last_flag) return;

    // Last workgroup of candidate g: its N-1 keys are final.  The first wave reads them, one
    // key per lane and all at once, with returning atomics (other workgroups updated them with
    // device-scope atomics, which act at the memory side, not in this XCD's L2).
    if (tid < 64) {
        const int g = row / n1;
        int len = 0;
        bool run = true;  // still inside the leading run of matches
        for (int k0 = 0; k0 < n1; k0 += 64) {
            const int k = k0 + tid;
            bool match = false;
            if (k < n1) {
                const unsigned long long key = atomicMax(&keys[g * n1 + k], 0ull);
                const int tok = (int)(0xFFFFFFFFu - (unsigned)key);
                accepted[g * n1 + k] = tok;
                match = tok == cand_tokens[g * n1 + k];
                atomicExch(&keys[g * n1 + k], 0ull);  // clean for the next call
            }
            const int here = min(64, n1 - k0);
            const unsigned long long mask = __builtin_amdgcn_ballot_w64(match);
            // number of leading set bits among the `here` lanes in use
            const unsigned long long inv = ~mask & (here == 64 ? ~0ull : ((1ull << here) - 1ull));
            const int lead = inv == 0ull ? here : (int)__builtin_ctzll(inv);
            if (run) len += lead;
            run = run && lead == here;
        }
        if (tid == 0) {
            accept_len[g] = len;
            atomicExch(&tickets[g], 0u);
        }
    }
}

// Row r of the step: 0 = output at the current token, 1 .. W = outputs at the newest lookahead
// tokens, 1 + W + g*n1 + k = output at candidate g's token k.  blockIdx.x = r * nseg + segment.
// keys: one per row; l1: one counter per `fan` workgroups; l2: one counter.
template <bool kVec>
__global__ __launch_bounds__(kThreads) void verify_step_kernel(
    const float* __restrict__ logits_cur, const float* __restrict__ logits_look,
    const float* __restrict__ logits_cand, const int* __restrict__ cand_tokens, int W, int n1, int G, int V,
    int seg_len, int nseg, int rows, unsigned fan, unsigned long long* keys, unsigned* l1, unsigned* l2,
    int* __restrict__ out_tokens, int* __restrict__ n_out, int* __restrict__ best_out,
    int* __restrict__ new_window, int* __restrict__ accept_len)
{
    extern __shared__ int tok[];  // rows greedy tokens, then one packed result per wave
    const int row = blockIdx.x / nseg;
    const int seg = blockIdx.x - row * nseg;
    const int v0 = seg * seg_len;
    const int v1 = min(V, v0 + seg_len);
    const float* p = row == 0 ? logits_cur
                              : (row <= W ? logits_look + (size_t)(row - 1) * V
                                          : logits_cand + (size_t)(row - 1 - W) * V);
    const int tid = threadIdx.x;
    const unsigned long long key = scan_segment<kVec>(p, v0, v1, tid);

    __shared__ unsigned long long wave_key[kWaves];
    __shared__ unsigned last_flag;
    if ((tid & 63) == 0) wave_key[tid >> 6] = key;
    __syncthreads();
    if (tid == 0) {
        unsigned long long k = wave_key[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) k = wave_key[w] > k ? wave_key[w] : k;
        // returning atomics: a ticket is requested only after the key update has come back
        const unsigned long long before = atomicMax(&keys[row], k);
        asm volatile("" ::"v"((unsigned)before) : "memory");
        // first-level counters take `fan` workgroups each; a few dozen arrivals on one address
        // still cost less than a second dependent round trip, so small launches use one level
        const unsigned blocks = gridDim.x, grp = blockIdx.x / fan;
        const unsigned n_groups = (blocks + fan - 1u) / fan;
        const unsigned grp_size = min(fan, blocks - grp * fan);
        unsigned last = 0u;
        if (atomicAdd(&l1[grp], 1u) == grp_size - 1u) {
            atomicExch(&l1[grp], 0u);  // clean for the next call
            last = n_groups == 1u ? 1u : (atomicAdd(l2, 1u) == n_groups - 1u ? 1u : 0u);
        }
        last_flag = last;
    }
    __syncthreads();
    if (!last_flag) return;

    // ---- last workgroup: every row's key is final.  Read them all at once with returning atomics
    //      (other workgroups updated them with device-scope atomics, which act at the memory
    //      side, not in this XCD's L2), and leave them zero.
    for (int r = tid; r < rows; r += kThreads) {
        const unsigned long long k = atomicMax(&keys[r], 0ull);
        tok[r] = (int)(0xFFFFFFFFu - (unsigned)k);
        atomicExch(&keys[r], 0ull);
    }
    __syncthreads();
    for (int j = tid; j < W; j += kThreads) new_window[j] = tok[1 + j];

    // Accept length of every candidate: slot 0 is judged by the current token's output, slot s by
    // the output at the candidate's token s-1.  The winner is the longest, first among equals:
    // largest (len << 32 | ~g).
    unsigned long long win = 0ull;
    for (int g = tid; g < G; g += kThreads) {
        int len = 0;
        while (len < n1 && (len == 0 ? tok[0] : tok[1 + W + g * n1 + len - 1]) == cand_tokens[g * n1 + len]) ++len;
        if (accept_len) accept_len[g] = len;
        const unsigned long long mine = ((unsigned long long)(unsigned)len << 32) | (0xFFFFFFFFu - (unsigned)g);
        win = mine > win ? mine : win;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const unsigned long long o = shfl_xor_u64(win, m);
        win = o > win ? o : win;
    }
    if ((tid & 63) == 0) wave_key[tid >> 6] = win;
    __syncthreads();
    if (tid == 0) {
        unsigned long long w = wave_key[0];
#pragma unroll
        for (int i = 1; i < kWaves; ++i) w = wave_key[i] > w ? wave_key[i] : w;
        int len = 0, best = -1;
        if (G > 0) {
            len = (int)(w >> 32);
            best = (int)(0xFFFFFFFFu - (unsigned)w);
        }
        for (int s = 0; s < len; ++s) out_tokens[s] = cand_tokens[best * n1 + s];
        // the model's own token at the first unaccepted slot: correction, or bonus after a full match
        out_tokens[len] = len == 0 ? tok[0] : tok[1 + W + best * n1 + len - 1];
        *n_out = len + 1;
        *best_out = best;
        if (gridDim.x > fan) atomicExch(l2, 0u);
    }
}

}  // namespace

la_status launch_verify(const float* logits, const int* cand_tokens, int G, int N, int V,
                        int* accept_len, int* accepted, hipStream_t stream)
{
    const int n1 = N - 1;
    const int rows = G * n1;
    // as few segments per row as the per-thread load budget allows
    int nseg = (V + kMaxSeg - 1) / kMaxSeg;
    int seg_len = (V + nseg - 1) / nseg;
    seg_len = (seg_len + 3) & ~3;
    nseg = (V + seg_len - 1) / seg_len;
    const long long blocks = (long long)rows * nseg;
    if (blocks > 0x7fffffffll) return fail(LA_EINVAL, "la_verify: too many workgroups");

    // workspace: one 64-bit key per row, then one ticket per candidate
    const size_t bytes = (size_t)rows * 8 + (size_t)G * 4;
    char* ws = (char*)zeroed_workspace(bytes, stream);
    if (!ws) return LA_ENOMEM;
    unsigned long long* keys = (unsigned long long*)ws;
    unsigned* ticket = (unsigned*)(ws + (size_t)rows * 8);

    const bool vec = (V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
    if (vec)
        hipLaunchKernelGGL(verify_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           logits, cand_tokens, G, n1, V, seg_len, nseg, keys, ticket, accept_len,
                           accepted);
    else
        hipLaunchKernelGGL(verify_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           logits, cand_tokens, G, n1, V, seg_len, nseg, keys, ticket, accept_len,
                           accepted);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_verify launch: %s", hipGetErrorString(e));
    return LA_OK;
}

la_status launch_verify_step(const float* logits_cur, const float* logits_look, const float* logits_cand,
                             const int* cand_tokens, int W, int N, int G, int V, int* out_tokens, int* n_out,
                             int* best, int* new_window, int* accept_len, hipStream_t stream)
{
    const int n1 = N - 1;
    const long long rows = 1ll + W + (long long)G * n1;
    int nseg = (V + kMaxSeg - 1) / kMaxSeg;
    int seg_len = (V + nseg - 1) / nseg;
    seg_len = (seg_len + 3) & ~3;
    nseg = (V + seg_len - 1) / seg_len;
    const long long blocks = rows * nseg;
    // the last workgroup keeps one token per row in LDS
    if (rows > 12 * 1024 || blocks > 0x7fffffffll)
        return fail(LA_EUNSUPPORTED, "la_verify_step: %lld rows is too many", rows);

    // workspace: one 64-bit key per row, one counter per `fan` workgroups, one more counter
    const unsigned fan = blocks <= 128 ? (unsigned)blocks : 8u;
    const size_t n_groups = (size_t)((blocks + fan - 1) / fan);
    const size_t bytes = (size_t)rows * 8 + n_groups * 4 + 4;
    char* ws = (char*)zeroed_workspace(bytes, stream);
    if (!ws) return LA_ENOMEM;
    unsigned long long* keys = (unsigned long long*)ws;
    unsigned* l1 = (unsigned*)(ws + (size_t)rows * 8);
    unsigned* l2 = l1 + n_groups;

    const bool vec = (V % 4 == 0) && ((((uintptr_t)logits_cur | (uintptr_t)logits_look | (uintptr_t)logits_cand) & 15) == 0);
    const size_t lds = (size_t)rows * sizeof(int);
    if (vec)
        hipLaunchKernelGGL(verify_step_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), lds, stream,
                           logits_cur, logits_look, logits_cand, cand_tokens, W, n1, G, V, seg_len, nseg,
                           (int)rows, fan, keys, l1, l2, out_tokens, n_out, best, new_window, accept_len);
    else
        hipLaunchKernelGGL(verify_step_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), lds, stream,
                           logits_cur, logits_look, logits_cand, cand_tokens, W, n1, G, V, seg_len, nseg,
                           (int)rows, fan, keys, l1, l2, out_tokens, n_out, best, new_window, accept_len);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_verify_step launch: %s", hipGetErrorString(e));
    return LA_OK;
}

}  // namespace la

// Greedy verification reduction for gfx950: per-row argmax over the vocabulary and the
// longest accepted prefix of every candidate n-gram (Sec. 2, the guess-and-verify paragraph; the
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
// workspace is clean for the next call without a memset.  (Where one workgroup covers a whole
// row and N-1 <= 16, the keys are not needed at all: each row hands its match bit to the
// candidate's counter together with its arrival, one atomic in place of three dependent ones.)
// Keys and tickets are touched only
// by device-scope atomics that return their old value (the ticket is taken after the key
// update has come back), so no cache write-back or invalidate is needed: those cost tens of
// microseconds on this part, more than the whole scan.
//
// verify_step_kernel ends a greedy step in one launch (Algorithm 3 in full, plus the greedy
// tokens of Algorithm 2's lookahead branch): the same row scan over 1 + W + G(N-1) rows, a
// two-level ticket (eight workgroups per first-level counter, so that no address sees more than
// a handful of atomics), and the workgroup that arrives last reads all row maxima at once and
// walks the candidates.
//
// verify_sample_kernel is sampling verification (Algorithm 4) in one launch.  Every workgroup
// reduces one row segment to the softmax statistics (maximum, sum of exponentials), publishes
// them and takes a ticket; the workgroup that arrives last walks the positions - per position
// one parallel gather of the first survivor's row at the survivors' tokens, then the accept
// tests in order - and finally draws the last token by inverse CDF over one row: chunk sums,
// a block-wide scan, and a walk through the chunk that holds the target.
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
    const int want = cand_tokens[row];  // requested before the scan, used after it

    const unsigned long long key = scan_segment<kVec>(p, v0, v1, tid);
    __shared__ unsigned long long wave_key[kWaves];
    __shared__ unsigned last_flag;
    if ((tid & 63) == 0) wave_key[tid >> 6] = key;
    __syncthreads();
    if (nseg == 1 && n1 <= 16) {
        // One workgroup per row: its winner is final.  The row writes its own `accepted` entry
        // and hands the candidate's counter its arrival (upper half) and its match bit (lower
        // half) in ONE returning atomic; whoever completes the count has every match bit of the
        // candidate in the returned word and needs nothing else from memory.
        if (tid == 0) {
            unsigned long long k = wave_key[0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) k = wave_key[w] > k ? wave_key[w] : k;
            const int tok = (int)(0xFFFFFFFFu - (unsigned)k);
            const int g = row / n1, pos = row - g * n1;
            accepted[row] = tok;
            const unsigned mine = tok == want ? 1u << pos : 0u;
            const unsigned old = atomicAdd(&tickets[g], 0x10000u | mine);
            if ((old >> 16) == (unsigned)n1 - 1u) {
                const unsigned miss = ~(old | mine) & ((1u << n1) - 1u);
                accept_len[g] = miss ? (int)__builtin_ctz(miss) : n1;
                atomicExch(&tickets[g], 0u);  // clean for the next call
            }
        }
        return;
    }
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
__device__ __forceinline__ void verify_step_body(
    const float* __restrict__ logits_cur, const float* __restrict__ logits_look,
    const float* __restrict__ logits_cand, const int* __restrict__ cand_tokens, int W, int n1, int G, int V,
    int seg_len, int nseg, int rows, unsigned fan, unsigned long long* keys, unsigned* l1, unsigned* l2,
    int* __restrict__ out_tokens, int* __restrict__ n_out, int* __restrict__ best_out,
    int* __restrict__ new_window, int* __restrict__ accept_len, int* tok)
{
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

template <bool kVec>
__global__ __launch_bounds__(kThreads) void verify_step_kernel(
    const float* __restrict__ logits_cur, const float* __restrict__ logits_look,
    const float* __restrict__ logits_cand, const int* __restrict__ cand_tokens, int W, int n1, int G, int V,
    int seg_len, int nseg, int rows, unsigned fan, unsigned long long* keys, unsigned* l1, unsigned* l2,
    int* __restrict__ out_tokens, int* __restrict__ n_out, int* __restrict__ best_out,
    int* __restrict__ new_window, int* __restrict__ accept_len)
{
    extern __shared__ int tok[];  // rows greedy tokens
    verify_step_body<kVec>(logits_cur, logits_look, logits_cand, cand_tokens, W, n1, G, V, seg_len, nseg, rows, fan,
                           keys, l1, l2, out_tokens, n_out, best_out, new_window, accept_len, tok);
}

// The ends of several sequences' steps in one launch: blockIdx.y names the sequence, blockIdx.x
// the row segment as above; every sequence has its own keys and counters in the workspace
// (ws_stride bytes apart) and its own last workgroup.  What differs between sequences travels
// as a kernel argument, kVerifyBatch of them at a time.
constexpr int kVerifyBatch = 32;
struct VerifyOne {
    const float* logits_cur;
    const float* logits_look;
    const float* logits_cand;
    const int* cand_tokens;
    int* out_tokens;
    int* n_out;
    int* best;
    int* new_window;
    int* accept_len;
};
struct VerifyBatchParams {
    VerifyOne one[kVerifyBatch];
    unsigned char* ws;
    size_t ws_stride, l1_offset, l2_offset;
    int W, n1, G, V, seg_len, nseg, rows;
    unsigned fan;
};

template <bool kVec>
__global__ __launch_bounds__(kThreads) void verify_step_batch_kernel(VerifyBatchParams b)
{
    extern __shared__ int tok[];
    const VerifyOne& o = b.one[blockIdx.y];
    unsigned char* ws = b.ws + (size_t)blockIdx.y * b.ws_stride;
    verify_step_body<kVec>(o.logits_cur, o.logits_look, o.logits_cand, o.cand_tokens, b.W, b.n1, b.G, b.V, b.seg_len,
                           b.nseg, b.rows, b.fan, (unsigned long long*)ws, (unsigned*)(ws + b.l1_offset),
                           (unsigned*)(ws + b.l2_offset), o.out_tokens, o.n_out, o.best, o.new_window, o.accept_len,
                           tok);
}

constexpr float kLog2e = 1.4426950408889634f;

// Softmax statistics of two disjoint sets, merged: (max, sum of exp(x - max)).
__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2)
{
    const float mn = fmaxf(m, m2);
    if (mn == -__builtin_huge_valf()) { m = mn; z = 0.0f; return; }
    z = z * __builtin_amdgcn_exp2f((m - mn) * kLog2e) + z2 * __builtin_amdgcn_exp2f((m2 - mn) * kLog2e);
    m = mn;
}

__device__ __forceinline__ float expw(float logit, float inv_t, float m)
{
    return __builtin_amdgcn_exp2f((logit * inv_t - m) * kLog2e);
}

// Row r: 0 = output at the current token, 1 + g*n1 + k = output at candidate g's token k.
// blockIdx.x = r * nseg + segment.  stats: one packed (max, sum) per workgroup.
template <bool kVec>
__device__ __forceinline__ void verify_sample_body(
    const float* __restrict__ logits_cur, const float* __restrict__ logits_cand,
    const int* __restrict__ cand_tokens, const float* __restrict__ u_test, const float* __restrict__ u_final,
    float inv_t, int n1, int G, int V, int seg_len, int nseg, int rows, unsigned fan, int lds_copy,
    unsigned long long* stats, unsigned* l1, unsigned* l2, int* __restrict__ out_tokens, int* __restrict__ n_out,
    float* dyn)  // dynamic LDS; last workgroup: row max [rows], row sum [rows], tokens [G], survivors [G]
{
    __shared__ float wave_m[kWaves], wave_z[kWaves], wave_tot[kWaves];
    __shared__ unsigned last_flag;
    __shared__ int sh_len, sh_jrow, sh_n_rej, sh_found, sh_last;
    __shared__ float sh_rej_mass, tile_part[kWaves][kVecPerThread], tile_tot[kVecPerThread];

    const int row = blockIdx.x / nseg;
    const int seg = blockIdx.x - row * nseg;
    const int v0 = seg * seg_len;
    const int v1 = min(V, v0 + seg_len);
    const float* p = row == 0 ? logits_cur : logits_cand + (size_t)(row - 1) * V;
    const int tid = threadIdx.x;
    const float kNegInf = -__builtin_huge_valf();

    // ---- statistics of this segment
    float m = kNegInf, z = 0.0f;
    if (kVec) {
        const float4* p4 = reinterpret_cast<const float4*>(p) + (v0 >> 2);
        const int nvec = (v1 - v0) >> 2;
        float4 x[kVecPerThread];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) x[j] = p4[min(tid + j * kThreads, nvec - 1)];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j)
            if (tid + j * kThreads < nvec)
                m = fmaxf(m, fmaxf(fmaxf(x[j].x, x[j].y), fmaxf(x[j].z, x[j].w)) * inv_t);
        // (inv_t > 0, so the maximum of the scaled values is the scaled maximum)
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j)
            if (tid + j * kThreads < nvec)
                z += expw(x[j].x, inv_t, m) + expw(x[j].y, inv_t, m) + expw(x[j].z, inv_t, m) + expw(x[j].w, inv_t, m);
    } else {
        for (int i = v0 + tid; i < v1; i += kThreads) m = fmaxf(m, p[i] * inv_t);
        for (int i = v0 + tid; i < v1; i += kThreads) z += expw(p[i], inv_t, m);
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) merge_stats(m, z, __shfl_xor(m, s, 64), __shfl_xor(z, s, 64));
    if ((tid & 63) == 0) { wave_m[tid >> 6] = m; wave_z[tid >> 6] = z; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w) merge_stats(m, z, wave_m[w], wave_z[w]);
        const unsigned long long packed =
            ((unsigned long long)__float_as_uint(z) << 32) | (unsigned long long)__float_as_uint(m);
        // returning atomics: the ticket is requested only after the statistics have been published
        const unsigned long long before = atomicExch(&stats[blockIdx.x], packed);
        asm volatile("" ::"v"((unsigned)before) : "memory");
        const unsigned blocks = gridDim.x, grp = blockIdx.x / fan;
        const unsigned n_groups = (blocks + fan - 1u) / fan;
        const unsigned grp_size = min(fan, blocks - grp * fan);
        unsigned last = 0u;
        if (atomicAdd(&l1[grp], 1u) == grp_size - 1u) {
            atomicExch(&l1[grp], 0u);
            last = n_groups == 1u ? 1u : (atomicAdd(l2, 1u) == n_groups - 1u ? 1u : 0u);
        }
        last_flag = last;
    }
    __syncthreads();
    if (!last_flag) return;
    if (tid == 0 && gridDim.x > fan) atomicExch(l2, 0u);

    // ---- last workgroup.  Row statistics: fetch every workgroup's pair (leaving zero behind) and
    //      merge the segments of a row in order.
    float* row_m = dyn;
    float* row_z = dyn + rows;
    int* tok = reinterpret_cast<int*>(dyn + 2 * rows);       // tokens examined at this position
    int* alive = reinterpret_cast<int*>(dyn + 2 * rows + max(G, 1));  // surviving candidates, in order
    for (int r = tid; r < rows; r += kThreads) {
        float mr = kNegInf, zr = 0.0f;
        for (int sgm = 0; sgm < nseg; ++sgm) {
            const unsigned long long v = atomicExch(&stats[r * nseg + sgm], 0ull);
            merge_stats(mr, zr, __uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
        }
        row_m[r] = mr;
        row_z[r] = zr;
    }
    for (int g = tid; g < G; g += kThreads) alive[g] = g;
    // the candidates' tokens and draws are read several times along dependent chains: keep a copy
    // in LDS when it fits (lds_copy says so)
    const int* ct = cand_tokens;
    const float* ut = u_test;
    if (lds_copy) {
        int* ct_l = alive + max(G, 1);
        float* ut_l = reinterpret_cast<float*>(ct_l + G * n1);
        for (int k = tid; k < G * n1; k += kThreads) { ct_l[k] = cand_tokens[k]; ut_l[k] = u_test[k]; }
        ct = ct_l;
        ut = ut_l;
    }
    __syncthreads();

    // ---- the walk over the positions (Algorithm 4's outer loop), by the first wave: the accept
    //      tests of a position are examined 64 at a time - each lane's probability needs only the
    //      mass ruled out before it (a prefix sum) - and the first lane that passes wins
    if (tid < 64) {
        const int lane = tid;
        int n_alive = G, len = 0, acc = 0, jrow = 0, n_rej = 0;
        float rej_mass = 0.0f;  // weight ruled out of the row the last token is drawn from
        for (int i = 0; i < n1 && n_alive > 0; ++i) {
            jrow = i == 0 ? 0 : 1 + alive[0] * n1 + (i - 1);   // the first survivor's i-th distribution
            const float* prow = jrow == 0 ? logits_cur : logits_cand + (size_t)(jrow - 1) * V;
            const float mrow = row_m[jrow], zrow = row_z[jrow];
            float rejected = 0.0f;  // weight ruled out so far at this position
            acc = -1;
            for (int base = 0; base < n_alive && acc < 0; base += 64) {
                const int j = base + lane;
                const bool valid = j < n_alive;
                const int t = valid ? ct[alive[j] * n1 + i] : -1;
                // a candidate token outside the vocabulary (a padding id, say) has probability zero: it
                // is never accepted, rules nothing out, and its logit is never read
                const bool in_vocab = valid && (unsigned)t < (unsigned)V;
                const float e = in_vocab ? expw(prow[t], inv_t, mrow) : 0.0f;
                const float u = valid ? ut[i * G + j] : 2.0f;
                if (valid) tok[j] = t;
                __builtin_amdgcn_wave_barrier();
                bool dup = false;  // proposed again after having been ruled out: probability zero now
                for (int k = 0; k < j && valid; ++k) dup = dup || tok[k] == t;
                const float contrib = (valid && !dup) ? e : 0.0f;
                float incl = contrib;
#pragma unroll
                for (int sft = 1; sft < 64; sft <<= 1) {
                    const float o = __shfl_up(incl, sft, 64);
                    if (lane >= sft) incl += o;
                }
                const float before = rejected + (incl - contrib);
                const float pj = dup ? 0.0f : e / (zrow - before);
                const unsigned long long pass = __builtin_amdgcn_ballot_w64(valid && u < pj);
                if (pass != 0ull) acc = base + (int)__builtin_ctzll(pass);
                rejected += __shfl(incl, 63, 64);
            }
            if (acc < 0) { n_rej = n_alive; rej_mass = rejected; break; }
            const int t = tok[acc];
            if (lane == 0) out_tokens[len] = t;
            ++len;
            // later candidates with the same token survive (compacted in place, in order)
            int kept = 0;
            for (int base = acc - (acc & 63); base < n_alive; base += 64) {
                const int k = base + lane;
                const int who = k < n_alive ? alive[k] : 0;
                const bool keep = k >= acc && k < n_alive && ct[who * n1 + i] == t;
                const unsigned long long km = __builtin_amdgcn_ballot_w64(keep);
                __builtin_amdgcn_wave_barrier();
                if (keep) alive[kept + (int)__builtin_popcountll(km & ((1ull << lane) - 1ull))] = who;
                kept += (int)__builtin_popcountll(km);
                __builtin_amdgcn_wave_barrier();
            }
            n_alive = kept;
        }
        if (acc >= 0) {
            // every position accepted (or no candidates): the next distribution of the first survivor
            jrow = len == 0 ? 0 : 1 + alive[0] * n1 + (len - 1);
            n_rej = 0;
            rej_mass = 0.0f;
        }
        if (lane == 0) { sh_len = len; sh_jrow = jrow; sh_n_rej = n_rej; sh_rej_mass = rej_mass; }
    }
    __syncthreads();
    const int len = sh_len, jrow = sh_jrow, n_rej = sh_n_rej;

    // ---- draw the last token from row jrow without the ruled-out tokens (tok[0 .. n_rej), repeats
    //      possible): inverse CDF in index order; the target is the draw times the row's remaining
    //      weight.
    const float* prow = jrow == 0 ? logits_cur : logits_cand + (size_t)(jrow - 1) * V;
    const float mrow = row_m[jrow];
    const float target = u_final[0] * (row_z[jrow] - sh_rej_mass);
    auto ruled_out = [&](int v) {
        bool r = false;
        for (int k = 0; k < n_rej; ++k) r = r || tok[k] == v;
        return r;
    };
    if (tid == 0) { sh_found = -1; sh_last = -1; }
    if (kVec) {
        // Coalesced 16-byte loads, as in the scan: within a tile of 4096 elements thread t holds
        // elements 4t .. 4t+3, so index order is (tile, thread, element).  Per super-tile of 8
        // tiles: the tile totals (8 block reductions at once) locate the tile, one scan over the
        // threads of that tile locates the thread.
        float run = 0.0f;   // weight of everything before the current tile (same in all threads)
        bool done = false;  // (uniform)
        for (int st = 0; st < V && !done; st += kMaxSeg) {
            const float4* p4 = reinterpret_cast<const float4*>(prow + st);
            const int nvec = (min(V, st + kMaxSeg) - st) >> 2;
            float4 x[kVecPerThread];
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j) x[j] = p4[min(tid + j * kThreads, nvec - 1)];
            float e[kVecPerThread][4], ssum[kVecPerThread];
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j) {
                const bool in = tid + j * kThreads < nvec;
                e[j][0] = in ? expw(x[j].x, inv_t, mrow) : 0.0f;
                e[j][1] = in ? expw(x[j].y, inv_t, mrow) : 0.0f;
                e[j][2] = in ? expw(x[j].z, inv_t, mrow) : 0.0f;
                e[j][3] = in ? expw(x[j].w, inv_t, mrow) : 0.0f;
            }
            for (int k = 0; k < n_rej; ++k) {  // ruled-out tokens that are this thread's elements
                const int off = tok[k] - st;
                if (off >= 0 && off < kMaxSeg && ((off >> 2) & (kThreads - 1)) == tid) {
#pragma unroll
                    for (int j = 0; j < kVecPerThread; ++j)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (off == (j * kThreads + tid) * 4 + c) e[j][c] = 0.0f;
                }
            }
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j) {
                ssum[j] = (e[j][0] + e[j][1]) + (e[j][2] + e[j][3]);
                float r = ssum[j];
#pragma unroll
                for (int sft = 32; sft >= 1; sft >>= 1) r += __shfl_xor(r, sft, 64);
                if ((tid & 63) == 0) tile_part[tid >> 6][j] = r;
            }
            __syncthreads();
            if (tid < kVecPerThread) {
                float t = 0.0f;
                for (int w = 0; w < kWaves; ++w) t += tile_part[w][tid];
                tile_tot[tid] = t;
            }
            __syncthreads();
            int jstar = -1;
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j) {
                if (jstar < 0) {
                    if (target < run + tile_tot[j]) jstar = j; else run += tile_tot[j];
                }
            }
            if (jstar >= 0) {
                done = true;
                float mine = 0.0f, ee[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int j = 0; j < kVecPerThread; ++j)
                    if (j == jstar) { mine = ssum[j]; ee[0] = e[j][0]; ee[1] = e[j][1]; ee[2] = e[j][2]; ee[3] = e[j][3]; }
                float incl = mine;
#pragma unroll
                for (int sft = 1; sft < 64; sft <<= 1) {
                    const float o = __shfl_up(incl, sft, 64);
                    if ((tid & 63) >= sft) incl += o;
                }
                if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
                __syncthreads();
                float base = run;
                for (int w = 0; w < (tid >> 6); ++w) base += wave_tot[w];
                // [lo, hi) of consecutive threads tile the tile's range exactly: a thread's lo is the
                // very value its predecessor computed as hi
                const float prev_incl = __shfl_up(incl, 1, 64);
                const float lo = base + ((tid & 63) == 0 ? 0.0f : prev_incl), hi = base + incl;
                if (mine > 0.0f && lo <= target && target < hi) {
                    float c = lo;
                    int pick = -1, last_pos = -1;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (ee[k] > 0.0f && pick < 0) last_pos = k;
                        c += ee[k];
                        if (pick < 0 && ee[k] > 0.0f && c > target) pick = k;
                    }
                    sh_found = st + (jstar * kThreads + tid) * 4 + (pick >= 0 ? pick : last_pos);
                }
                // should rounding leave the target between the threads' intervals and the tile's
                // total, the answer is the tile's last token with positive weight
                // (one LDS atomic per wave: a thousand of them on one word take microseconds)
                int last_here = -1;
                if (mine > 0.0f) {
                    int lp = 0;
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (ee[k] > 0.0f) lp = k;
                    last_here = st + (jstar * kThreads + tid) * 4 + lp;
                }
#pragma unroll
                for (int sft = 32; sft >= 1; sft >>= 1) last_here = max(last_here, __shfl_xor(last_here, sft, 64));
                if ((tid & 63) == 0 && last_here >= 0) atomicMax(&sh_last, last_here);
            }
        }
    } else {
        // rows that cannot be read 16 bytes at a time: a thread owns a contiguous chunk (slower:
        // the loads of a wave do not coalesce)
        const int chunk = (V + kThreads - 1) / kThreads;
        const int c0 = min(V, tid * chunk), c1 = min(V, c0 + chunk);
        float mine = 0.0f;
        for (int v = c0; v < c1; ++v)
            if (!ruled_out(v)) mine += expw(prow[v], inv_t, mrow);
        float incl = mine;
#pragma unroll
        for (int sft = 1; sft < 64; sft <<= 1) {
            const float o = __shfl_up(incl, sft, 64);
            if ((tid & 63) >= sft) incl += o;
        }
        if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
        __syncthreads();
        float base = 0.0f;
        for (int w = 0; w < (tid >> 6); ++w) base += wave_tot[w];
        const float prev_incl = __shfl_up(incl, 1, 64);
        const float lo = base + ((tid & 63) == 0 ? 0.0f : prev_incl), hi = base + incl;
        if (mine > 0.0f && lo <= target && target < hi) {
            float c = lo;
            int pick = -1, last_pos = -1;
            for (int v = c0; v < c1 && pick < 0; ++v) {
                if (ruled_out(v)) continue;
                const float e = expw(prow[v], inv_t, mrow);
                if (e > 0.0f) last_pos = v;
                c += e;
                if (e > 0.0f && c > target) pick = v;
            }
            sh_found = pick >= 0 ? pick : last_pos;
        }
    }
    __syncthreads();
    if (tid == 0) {
        int pick = sh_found >= 0 ? sh_found : sh_last;
        if (pick < 0) {
            // rounding left the target at or beyond the total: the last token with positive weight
            for (int v = V - 1; v >= 0 && pick < 0; --v)
                if (!ruled_out(v) && expw(prow[v], inv_t, mrow) > 0.0f) pick = v;
            if (pick < 0) pick = 0;
        }
        out_tokens[len] = pick;
        *n_out = len + 1;
    }
}

template <bool kVec>
__global__ __launch_bounds__(kThreads) void verify_sample_kernel(
    const float* __restrict__ logits_cur, const float* __restrict__ logits_cand,
    const int* __restrict__ cand_tokens, const float* __restrict__ u_test, const float* __restrict__ u_final,
    float inv_t, int n1, int G, int V, int seg_len, int nseg, int rows, unsigned fan, int lds_copy,
    unsigned long long* stats, unsigned* l1, unsigned* l2, int* __restrict__ out_tokens, int* __restrict__ n_out)
{
    extern __shared__ float dyn[];
    verify_sample_body<kVec>(logits_cur, logits_cand, cand_tokens, u_test, u_final, inv_t, n1, G, V, seg_len, nseg,
                             rows, fan, lds_copy, stats, l1, l2, out_tokens, n_out, dyn);
}

// Sampling verification for several sequences in one launch: blockIdx.y names the sequence; each
// has its own statistics and counters in the workspace (ws_stride bytes apart), its own draws
// and temperature, and its own last workgroup.
struct SampleOne {
    const float* logits_cur;
    const float* logits_cand;
    const int* cand_tokens;
    const float* u_test;
    const float* u_final;
    int* out_tokens;
    int* n_out;
    float inv_t;
};
struct SampleBatchParams {
    SampleOne one[kVerifyBatch];
    unsigned char* ws;
    size_t ws_stride, l1_offset, l2_offset;
    int n1, G, V, seg_len, nseg, rows, lds_copy;
    unsigned fan;
};

template <bool kVec>
__global__ __launch_bounds__(kThreads) void verify_sample_batch_kernel(SampleBatchParams b)
{
    extern __shared__ float dyn[];
    const SampleOne& o = b.one[blockIdx.y];
    unsigned char* ws = b.ws + (size_t)blockIdx.y * b.ws_stride;
    verify_sample_body<kVec>(o.logits_cur, o.logits_cand, o.cand_tokens, o.u_test, o.u_final, o.inv_t, b.n1, b.G, b.V,
                             b.seg_len, b.nseg, b.rows, b.fan, b.lds_copy, (unsigned long long*)ws,
                             (unsigned*)(ws + b.l1_offset), (unsigned*)(ws + b.l2_offset), o.out_tokens, o.n_out, dyn);
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
    if (!ws) return last_failure();
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
    if (!ws) return last_failure();
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

la_status launch_verify_step_batch(const VerifySeq* seqs, int n_seqs, int W, int N, int G, int V,
                                   hipStream_t stream)
{
    const int n1 = N - 1;
    const long long rows = 1ll + W + (long long)G * n1;
    int nseg = (V + kMaxSeg - 1) / kMaxSeg;
    int seg_len = (V + nseg - 1) / nseg;
    seg_len = (seg_len + 3) & ~3;
    nseg = (V + seg_len - 1) / seg_len;
    const long long blocks = rows * nseg;
    if (rows > 12 * 1024 || blocks > 0x7fffffffll)
        return fail(LA_EUNSUPPORTED, "la_verify_step_batch: %lld rows is too many", rows);
    const unsigned fan = blocks <= 128 ? (unsigned)blocks : 8u;
    const size_t n_groups = (size_t)((blocks + fan - 1) / fan);
    // per sequence: one 64-bit key per row, one counter per `fan` workgroups, one more counter
    const size_t l1_offset = (size_t)rows * 8, l2_offset = l1_offset + n_groups * 4;
    const size_t ws_stride = (l2_offset + 4 + 7) & ~(size_t)7;
    for (int i0 = 0; i0 < n_seqs; i0 += kVerifyBatch) {
        const int n = n_seqs - i0 < kVerifyBatch ? n_seqs - i0 : kVerifyBatch;
        VerifyBatchParams b;
        bool vec = V % 4 == 0;
        for (int i = 0; i < n; ++i) {
            const VerifySeq& q = seqs[i0 + i];
            b.one[i] = VerifyOne{q.logits_cur, q.logits_look, q.logits_cand, q.cand_tokens, q.out_tokens,
                                 q.n_out,      q.best,        q.new_window,  q.accept_len};
            vec = vec && ((((uintptr_t)q.logits_cur | (uintptr_t)q.logits_look | (uintptr_t)q.logits_cand) & 15) == 0);
        }
        for (int i = n; i < kVerifyBatch; ++i) b.one[i] = b.one[0];  // never indexed: the grid has n layers
        // (launches on one stream run in order, so they can share the workspace)
        b.ws = (unsigned char*)zeroed_workspace(ws_stride * (size_t)n, stream);
        if (!b.ws) return last_failure();
        b.ws_stride = ws_stride; b.l1_offset = l1_offset; b.l2_offset = l2_offset;
        b.W = W; b.n1 = n1; b.G = G; b.V = V; b.seg_len = seg_len; b.nseg = nseg; b.rows = (int)rows;
        b.fan = fan;
        const size_t lds = (size_t)rows * sizeof(int);
        const dim3 grid((unsigned)blocks, (unsigned)n);
        if (vec) hipLaunchKernelGGL(verify_step_batch_kernel<true>, grid, dim3(kThreads), lds, stream, b);
        else hipLaunchKernelGGL(verify_step_batch_kernel<false>, grid, dim3(kThreads), lds, stream, b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(LA_EHIP, "la_verify_step_batch launch: %s", hipGetErrorString(e));
    }
    return LA_OK;
}

la_status launch_verify_sample(const float* logits_cur, const float* logits_cand, const int* cand_tokens,
                               const float* u_test, const float* u_final, float temperature, int N, int G,
                               int V, int* out_tokens, int* n_out, hipStream_t stream)
{
    const int n1 = N - 1;
    const long long rows = 1ll + (long long)G * n1;
    int nseg = (V + kMaxSeg - 1) / kMaxSeg;
    int seg_len = (V + nseg - 1) / nseg;
    seg_len = (seg_len + 3) & ~3;
    nseg = (V + seg_len - 1) / seg_len;
    const long long blocks = rows * nseg;
    // the last workgroup keeps two floats per row and two words per candidate in LDS, and a copy of
    // the candidates' tokens and draws if that still fits
    size_t lds = ((size_t)rows * 2 + (size_t)(G > 0 ? G : 1) * 2) * sizeof(float);
    if (lds > 48 * 1024 || blocks > 0x7fffffffll)
        return fail(LA_EUNSUPPORTED, "la_verify_sample: %lld rows is too many", rows);
    const int lds_copy = lds + (size_t)G * n1 * 8 <= 48 * 1024 ? 1 : 0;
    if (lds_copy) lds += (size_t)G * n1 * 8;

    const unsigned fan = blocks <= 128 ? (unsigned)blocks : 8u;
    const size_t n_groups = (size_t)((blocks + fan - 1) / fan);
    const size_t bytes = (size_t)blocks * 8 + n_groups * 4 + 4;
    char* ws = (char*)zeroed_workspace(bytes, stream);
    if (!ws) return last_failure();
    unsigned long long* stats = (unsigned long long*)ws;
    unsigned* l1 = (unsigned*)(ws + (size_t)blocks * 8);
    unsigned* l2 = l1 + n_groups;

    const float inv_t = 1.0f / temperature;
    const bool vec = (V % 4 == 0) && ((((uintptr_t)logits_cur | (uintptr_t)logits_cand) & 15) == 0);
    if (vec)
        hipLaunchKernelGGL(verify_sample_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), lds, stream,
                           logits_cur, logits_cand, cand_tokens, u_test, u_final, inv_t, n1, G, V, seg_len,
                           nseg, (int)rows, fan, lds_copy, stats, l1, l2, out_tokens, n_out);
    else
        hipLaunchKernelGGL(verify_sample_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), lds, stream,
                           logits_cur, logits_cand, cand_tokens, u_test, u_final, inv_t, n1, G, V, seg_len,
                           nseg, (int)rows, fan, lds_copy, stats, l1, l2, out_tokens, n_out);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_verify_sample launch: %s", hipGetErrorString(e));
    return LA_OK;
}

la_status launch_verify_sample_batch(const SampleSeq* seqs, int n_seqs, int N, int G, int V, hipStream_t stream)
{
    const int n1 = N - 1;
    const long long rows = 1ll + (long long)G * n1;
    int nseg = (V + kMaxSeg - 1) / kMaxSeg;
    int seg_len = (V + nseg - 1) / nseg;
    seg_len = (seg_len + 3) & ~3;
    nseg = (V + seg_len - 1) / seg_len;
    const long long blocks = rows * nseg;
    size_t lds = ((size_t)rows * 2 + (size_t)(G > 0 ? G : 1) * 2) * sizeof(float);
    if (lds > 48 * 1024 || blocks > 0x7fffffffll)
        return fail(LA_EUNSUPPORTED, "la_verify_sample_batch: %lld rows is too many", rows);
    const int lds_copy = lds + (size_t)G * n1 * 8 <= 48 * 1024 ? 1 : 0;
    if (lds_copy) lds += (size_t)G * n1 * 8;
    const unsigned fan = blocks <= 128 ? (unsigned)blocks : 8u;
    const size_t n_groups = (size_t)((blocks + fan - 1) / fan);
    const size_t l1_offset = (size_t)blocks * 8, l2_offset = l1_offset + n_groups * 4;
    const size_t ws_stride = (l2_offset + 4 + 7) & ~(size_t)7;
    for (int i0 = 0; i0 < n_seqs; i0 += kVerifyBatch) {
        const int n = n_seqs - i0 < kVerifyBatch ? n_seqs - i0 : kVerifyBatch;
        SampleBatchParams b;
        bool vec = V % 4 == 0;
        for (int i = 0; i < n; ++i) {
            const SampleSeq& q = seqs[i0 + i];
            b.one[i] = SampleOne{q.logits_cur, q.logits_cand, q.cand_tokens, q.u_test,
                                 q.u_final,    q.out_tokens,  q.n_out,       1.0f / q.temperature};
            vec = vec && ((((uintptr_t)q.logits_cur | (uintptr_t)q.logits_cand) & 15) == 0);
        }
        for (int i = n; i < kVerifyBatch; ++i) b.one[i] = b.one[0];  // never indexed: the grid has n layers
        b.ws = (unsigned char*)zeroed_workspace(ws_stride * (size_t)n, stream);
        if (!b.ws) return last_failure();
        b.ws_stride = ws_stride; b.l1_offset = l1_offset; b.l2_offset = l2_offset;
        b.n1 = n1; b.G = G; b.V = V; b.seg_len = seg_len; b.nseg = nseg; b.rows = (int)rows; b.lds_copy = lds_copy;
        b.fan = fan;
        const dim3 grid((unsigned)blocks, (unsigned)n);
        if (vec) hipLaunchKernelGGL(verify_sample_batch_kernel<true>, grid, dim3(kThreads), lds, stream, b);
        else hipLaunchKernelGGL(verify_sample_batch_kernel<false>, grid, dim3(kThreads), lds, stream, b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(LA_EHIP, "la_verify_sample_batch launch: %s", hipGetErrorString(e));
    }
    return LA_OK;
}

}  // namespace la

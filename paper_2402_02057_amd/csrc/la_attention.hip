// Lookahead-step attention for gfx950 (Sec. 2 causal attention under the mask of Sec. 3.3,
// Fig. 2(b)): the current token, the W x (N-1) lookahead window and G candidate n-grams
// attend to the prefix KV cache and to each other in one pass.
//
// Shape of the problem.  The T = 1 + (W+G)(N-1) step rows of the g = heads/kv_heads query
// heads that share one KV head form R = T*g query rows over the same P + T keys, so QK^T and
// PV are dense [R x d] x [d x keys] contractions: they run on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate) while K and V stream from HBM exactly once per
// row block.
//
// Decomposition.  A workgroup owns (KV head, block of RT 32-row tiles, one of XS ranges of
// 64-key chunks).  Chunks are copied HBM -> LDS by direct-to-LDS loads into a ring of stages;
// the 16-byte pieces of a row are stored XOR-swizzled so that both the K operand reads
// (ds_read_b128, one key per lane) and the transposing V reads (ds_read_b64_tr_b16) are free
// of bank conflicts.  Within a workgroup, KS waves share a row tile and take alternate 32-key
// blocks of each chunk; they are merged through LDS at the end.
//
// Per 32-key block a wave computes S^T = K Q^T (keys x rows), so that every lane holds 16
// scores of ONE query row: the row maximum and sum are in-register reductions plus one
// cross-lane step, and the exponentiated scores, converted to bf16, already have the layout
// of the B operand of O^T += V^T P^T - no LDS round trip for P.
//
// Mask.  Prefix keys are visible to every row.  For step keys the visible set of row t is
//   {0} u [0, 1+j] u {t - k*W : k = 0..l}      lookahead (l, j)
//   {0} u [t - k, t]                            candidate token k
// (Algorithm 2's conditioning sets read as index ranges), turned into one 32-bit word per
// (row, key block) from integer ranges in registers; no mask tensor exists anywhere.
//
// Split combine, in the same launch, wave by wave.  With XS > 1 each wave stores the slice(s)
// of the unnormalised accumulator it owns after the key-split merge, rounded to bf16, and
// (max, sum) per row, waits for the stores to be acknowledged by the L2, and takes a ticket of
// its own; the wave that arrives last in its group merges all XS partials in index order (so
// results do not depend on arrival order), normalises and writes bf16.  The L2 of one XCD is
// coherent for all its compute units, but the eight L2s are not coherent with each other
// inside a kernel, and an agent-scope fence (L2 write-back + invalidate) costs tens of
// microseconds here.  So the workgroups of a split group are laid out on one XCD (workgroup
// ids go round-robin over XCDs) and the ticket also carries the XCD id each member read
// from the hardware register: if all ids agree the partials are read straight from the shared
// L2; if not, the last wave ignores the partials and its workgroup recomputes its rows over
// all chunks from the read-only inputs and writes them directly.  The two paths agree to the
// bf16 rounding of the partials, not bit for bit (the recomputed accumulator is never rounded),
// so a result can differ in the last place with where the workgroups happened to run; both are
// within the tolerance of the step.  Tickets return to zero, so no memset is needed between
// calls.
//
// Variants of the same kernel (template parameters): a paged cache (block table), a subset of
// the step's rows, keys and values as 8-bit floats with a scale per KV head (converted exactly
// to bf16 in front of the MFMA), and query rows (optionally the step keys too) rotated on the
// way in (rotary embedding).
#include <stdlib.h>

#include <mutex>
#include <string>

#include "la_internal.h"
#include "la_attention_common.h"
#include "la_rope_common.h"

#ifdef LA_DEV_HOOKS
#include LA_DEV_HOOKS  // developer builds only: timing stamps, never part of the product build
#else
#define LA_STAMP(k) do { } while (0)
#endif

namespace la {
namespace {

// Tickets of different waves sit in different 128-byte lines: atomics on one line are served one
// after the other by the L2 (eight counters side by side cost a microsecond at the 7B shape).
constexpr int kTicketStride = 32;  // in 4-byte words

struct AttnParams {
    const __bf16* q;
    const __bf16* k_cache;
    const __bf16* v_cache;
    const __bf16* step_k;
    const __bf16* step_v;
    __bf16* out;
    // Two pointers whose meaning depends on the kernel variant (the variants exclude each other, and
    // the structure has to stay small: it travels as a kernel argument, sixteen at a time in a batch):
    //   paged cache       block_table: k_cache / v_cache are [n_pages][kv_heads][page][head_dim] and
    //                     prefix key t sits in page block_table[t / page] at slot t % page
    //   row subset        row_ids: T ids of rows of the full (W, N, G) layout
    //   quantised cache   k_scale, v_scale: one fp32 scale per KV head each (8-bit keys and values)
    //   rotating          rope_cos, rope_sin: the rows of the model's tables from the prefix length
    //                     on, [rope_rows][head_dim/2] fp32 each (query rows rotated on the way in)
    union {
        const int* block_table;
        const float* k_scale;
        const float* rope_cos;
    };
    union {
        const int* row_ids;
        const float* v_scale;
        const float* rope_sin;
    };
    int rope_rows;         // positions P .. P + rope_rows - 1 are staged in LDS
    int rope_block;        // LDS bytes reserved per table (rope_rows * head_dim * 2 rounded up to 1 KB)
    int rope_flags;  // bit 0: pairing of the rotation, 0 (x[i], x[i + d/2]), 1 (x[2i], x[2i + 1]);
                     // bit 1: the step keys are rotated in the kernel as well
    void* partials;     // XS > 1: per workgroup and wave, fragment-layout bf16 slices and fp32 (m, l)
    unsigned* tickets;  // XS > 1: one counter (kTicketStride words apart) per (KV head, row block, wave), zero between calls
    int P, W, N, G, T;
    long long cache_rows;  // rows between the caches of consecutive KV heads (>= P; paged: the page size)
    long long page_bytes;  // bytes of one page (all KV heads)
    int page_chunks;       // chunks per page
    int n_pages;           // table entries are clamped to 0 .. n_pages-1
    int table_last;        // last valid index of block_table
    float inv_page_chunks;
    int heads, kv_heads, group;
    int R;                // T * group query rows per KV head
    int n_prefix_chunks;  // ceil(P / KC)
    int n_chunks;         // prefix chunks + step chunks
    int n_row_blocks;
    int XS;
    int total_wg;         // kv_heads * n_row_blocks * XS
    int wg_per_xcd;       // ceil(total_wg / 8)
    float scale_log2;     // log2(e) / sqrt(head_dim)
    // Integer division costs dozens of instructions, and a wave issues about one instruction
    // every four cycles: quotients by these small divisors are taken with a float reciprocal
    // (exact while the dividend stays below 2^21, which the host checks).
    float inv_XS, inv_row_blocks, inv_group, inv_W, inv_n1;
    int chunks_lo, chunks_rem;  // n_chunks = XS * chunks_lo + chunks_rem
    int pre;              // chunks requested before the loop starts (1 .. stages)
    int force_recompute;  // testing: treat every group as spread over several XCDs
};

// Row-subset variant: a row of the full layout as (branch, coordinates), and the pairwise rule
// of Sec. 3.3 written out (the closed-form words above assume consecutive step keys).
struct RowPos {
    int cls;  // 0 current token, 1 lookahead (a = level, b = column), 2 candidate (a = candidate, b = token)
    int a, b;
};

__device__ __forceinline__ RowPos row_position(int t, int W, int N, float inv_W, float inv_n1)
{
    RowPos r;
    const int n_look = W * (N - 1);
    if (t == 0) {
        r.cls = 0; r.a = 0; r.b = 0;
    } else if (t <= n_look) {
        const int x = t - 1;
        r.cls = 1; r.a = div_small(x, inv_W); r.b = x - r.a * W;
    } else {
        const int x = t - 1 - n_look;
        r.cls = 2; r.a = div_small(x, inv_n1); r.b = x - r.a * (N - 1);
    }
    return r;
}

__device__ __forceinline__ bool visible_pair(const RowPos& q, int tk, int W, int N, float inv_W, float inv_n1)
{
    if (tk == 0) return true;  // everyone sees the current token
    const RowPos k = row_position(tk, W, N, inv_W, inv_n1);
    if (q.cls != k.cls) return false;
    if (q.cls == 1) return (k.a == 0 && k.b <= q.b) || (k.b == q.b && k.a <= q.a);
    return q.cls == 2 && k.a == q.a && k.b <= q.b;
}

// KVB: bytes per key / value element (2: bf16; 1: 8-bit float, quantised cache).  Q rows are bf16 always.
template <int D, int RT, int KS, int KC, int NSTAGE, int KVB = 2>
struct Cfg {
    static constexpr int HEAD_DIM = D;
    static constexpr int NW = RT * KS;
    static constexpr int NT = NW * 64;
    static constexpr int RBYTES = D * KVB;                // a key or value row
    static constexpr int QRBYTES = D * 2;                 // a query row
    static constexpr int NCH = RBYTES / 16;               // 16-byte pieces per key / value row
    static constexpr int QNCH = QRBYTES / 16;             // per query row
    static constexpr int KB = KC / 32;                    // 32-key blocks per chunk
    // Key-split waves of a row tile: up to KB of them share a chunk (one or more blocks each);
    // beyond that, groups of KB waves take consecutive chunks of the same iteration.
    static constexpr int CPI = KS > KB ? KS / KB : 1;     // chunks consumed per iteration
    static constexpr int KBW = KS >= KB ? 1 : KB / KS;    // blocks per wave per chunk
    static constexpr int KV_BYTES = KC * RBYTES;          // one of K or V of a chunk
    static constexpr int STAGE_BYTES = 2 * KV_BYTES;
    static constexpr int WLOADS = STAGE_BYTES / 1024;     // 64-lane x 16-byte loads per chunk
    static constexpr int LPW = WLOADS / NW;               // loads per wave per chunk
    static constexpr int TILES = RT;                      // 32-row tiles per workgroup, one per wave group
    static constexpr int ROWS = TILES * 32;
    static constexpr int DB = D / 32;                     // 32-wide blocks of head_dim
    // After the key-split merge a wave owns SPW of its tile's DB (tile, 32-column) slices.
    static constexpr int SPW = KS > 1 ? DB / KS : DB;
    // Key-split merge through LDS: a wave leaves the DB - SPW slices it does not own as bf16 (16
    // values x 64 lanes x 2 bytes each, fragment order) followed by (m, l) of its rows per lane in fp32.
    static constexpr int MERGE_WAVE_BYTES = KS > 1 ? (DB - SPW) * 2048 + 512 : 0;
    static constexpr int MERGE_BYTES = NW * MERGE_WAVE_BYTES;
    // The merge area lies in ring stages that the last iteration of the loop does not read (that
    // iteration reads stages F .. F + CPI - 1 modulo NSTAGE): the longer of the runs below and
    // above them, or the run between them when they wrap around.  FREE_STAGES is the shortest
    // such run over all F; where the area (and the flag word behind it) fits into it, no barrier
    // is needed between the loop and the merge.
    static constexpr int free_stages()
    {
        int least = NSTAGE;
        for (int k = 0; k < NSTAGE; ++k) {
            const int f = (k * CPI) % NSTAGE;  // the first live stage is a multiple of CPI modulo NSTAGE
            int best = 0;
            if (f + CPI <= NSTAGE) {
                const int below = f, above = NSTAGE - CPI - f;
                best = below > above ? below : above;
            } else {
                best = NSTAGE - CPI;  // the live stages wrap around: everything between them is free
            }
            if (best < least) least = best;
        }
        return least;
    }
    static constexpr int FREE_STAGES = free_stages();
    static constexpr bool MERGE_EARLY = KS > 1 && MERGE_BYTES + 16 <= FREE_STAGES * STAGE_BYTES;
    static_assert(!(D == 128 && RT == 2 && KS == 4 && NSTAGE == 4 && KVB == 2) || MERGE_EARLY,
                  "the plan of the benchmark shapes merges without a barrier after the loop");
    // a split's partial in global memory, per wave: its SPW slices as bf16 in fragment order
    // ([8 values][lane], 16 bytes per lane and access) followed by (m, l) of its rows per lane in fp32
    static constexpr int PART_ACC_BYTES = SPW * 16 * 64 * 2;
    static constexpr int PART_WAVE_BYTES = PART_ACC_BYTES + 64 * 8;
    static constexpr int PART_WG_BYTES = NW * PART_WAVE_BYTES;
    static constexpr int Q_BYTES = ROWS * QRBYTES;        // the workgroup's query rows
    static constexpr int Q_OFFSET = NSTAGE * STAGE_BYTES; // they sit behind the stage ring
    static constexpr int QLPW = Q_BYTES / 1024 / NW;      // Q loads per wave
    static constexpr int LDS_MAIN = NSTAGE * STAGE_BYTES + Q_BYTES;
    static constexpr int LDS_BYTES = LDS_MAIN > MERGE_BYTES + 16 ? LDS_MAIN : MERGE_BYTES + 16;
    static_assert(KS >= KB ? KS % KB == 0 : KB % KS == 0, "key-split waves and blocks must divide");
    static_assert(KS == 1 || DB % KS == 0, "key-split waves must divide the head_dim blocks");
    static_assert(NSTAGE >= CPI, "an iteration's chunks must fit the ring");
    static_assert(WLOADS % NW == 0, "chunk loads must divide among the waves");
    static_assert((Q_BYTES / 1024) % NW == 0, "Q loads must divide among the waves");
    static_assert(NSTAGE <= 9, "wait_chunks covers up to 8 younger chunks");
    // rotating variant: the cosine and sine rows of the step's positions, behind everything else
    static constexpr int ROPE_OFFSET = LDS_BYTES;
    static constexpr int ROPE_POS_BYTES = D * 2;           // one position of one table (D/2 fp32)
    static constexpr int ROPE_MAX_BYTES = (160 * 1024 - LDS_BYTES) / 2048 * 2048 < 64 * 1024
                                              ? (160 * 1024 - LDS_BYTES) / 2048 * 2048 : 64 * 1024;  // both tables
    // row-subset variant: the ids of up to ROWSET_MAX rows, staged behind everything else
    static constexpr int ROWSET_MAX = 1024;
    static constexpr int ROWIDS_OFFSET = LDS_BYTES;
    static constexpr int ROWIDS_BYTES = ROWSET_MAX * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of a compute unit");
};


// Write one finished (tile, 32-column) slice: lane (l32, hi) holds, for query row tile*32 + l32 of
// the workgroup, columns db*32 + i4*8 + hi*4 .. +3 in vals[i4*4 .. +3].  The two half-waves of a
// row fill 16 contiguous bytes per i4, 64 per slice.
template <class C, int D = C::HEAD_DIM>
__device__ __forceinline__ void store_slice(const AttnParams& p, int rb, int kvh, int tile, int db, int l32,
                                            int hi, const f32x16& vals, float inv)
{
    const int rr = rb * C::ROWS + tile * 32 + l32;
    if (rr >= p.R) return;
    const int t = div_small(rr, p.inv_group), hh = rr - t * p.group;
    __bf16* row = p.out + ((size_t)t * p.heads + (size_t)kvh * p.group + hh) * D + db * 32 + hi * 4;
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (__bf16)(vals[i4 * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(row + i4 * 8) = v;
    }
}

// Merge the KS key-split waves of a row tile, for the wave whose key index is MYKS.  Every
// wave leaves the slices it does not own in `area` (bf16, fragment layout: [2 halves][lane], 16
// bytes per lane and access) with its (max, sum); after one barrier each wave sums its own SPW
// slices over the KS states, in key order (its own state stays in fp32).  On return
// o[0 .. SPW-1] hold the merged slices MYKS*SPW .. MYKS*SPW+SPW-1 and (m_run, l_run) the merged
// softmax state of the row.
template <class C, int KS, int MYKS>
__device__ __forceinline__ void merge_key_splits(unsigned char* area, int rt, int lane, bool wave_active,
                                                 f32x16 (&o)[C::DB], float& m_run, float& l_run, float scale_log2)
{
    constexpr int DB0 = MYKS * C::SPW;
    constexpr int ML_OFFSET = (C::DB - C::SPW) * 2048;
    unsigned char* const tile = area + rt * KS * C::MERGE_WAVE_BYTES;  // this tile's states
    if (wave_active) {
        unsigned char* dst = tile + MYKS * C::MERGE_WAVE_BYTES;
        int slot = 0;
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
            if (db >= DB0 && db < DB0 + C::SPW) continue;  // stays in registers
#pragma unroll
            for (int i8 = 0; i8 < 2; ++i8) {
                bf16x8 v;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (__bf16)o[db][i8 * 8 + e];
                *reinterpret_cast<bf16x8*>(dst + ((slot * 2 + i8) * 64 + lane) * 16) = v;
            }
            ++slot;
        }
        *reinterpret_cast<f32x2*>(dst + ML_OFFSET + lane * 8) = f32x2{m_run, l_run};
    }
    LA_STAMP(2);
    __syncthreads();
    LA_STAMP(19);
    if (!wave_active) return;
    f32x2 ml[KS];
#pragma unroll
    for (int k = 0; k < KS; ++k)
        ml[k] = k == MYKS ? f32x2{m_run, l_run}
                          : *reinterpret_cast<const f32x2*>(tile + k * C::MERGE_WAVE_BYTES + ML_OFFSET + lane * 8);
    bf16x8 v[C::SPW][KS][2];
#pragma unroll
    for (int u = 0; u < C::SPW; ++u)
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            if (k == MYKS) continue;
            // wave k stored its slices in order, skipping its own k*SPW .. k*SPW+SPW-1
            const int slot = DB0 + u < k * C::SPW ? DB0 + u : DB0 + u - C::SPW;
#pragma unroll
            for (int i8 = 0; i8 < 2; ++i8)
                v[u][k][i8] = *reinterpret_cast<const bf16x8*>(tile + k * C::MERGE_WAVE_BYTES +
                                                               ((slot * 2 + i8) * 64 + lane) * 16);
        }
    float m_all = ml[0][0];
#pragma unroll
    for (int k = 1; k < KS; ++k) m_all = fmaxf(m_all, ml[k][0]);
    const float m_use = (m_all == kNegInf) ? 0.0f : m_all;
    float a[KS];
    float l = 0.0f;
#pragma unroll
    for (int k = 0; k < KS; ++k) {
        a[k] = fast_exp2((ml[k][0] - m_use) * scale_log2);
        l = __builtin_fmaf(ml[k][1], a[k], l);
    }
    m_run = m_all;
    l_run = l;
#pragma unroll
    for (int u = 0; u < C::SPW; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float acc = 0.0f;
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                const float x = k == MYKS ? o[DB0 + u][i] : (float)v[u][k][i >> 3][i & 7];
                acc = k == 0 ? x * a[0] : __builtin_fmaf(x, a[k], acc);
            }
            o[u][i] = acc;
        }
}

// PAGED: the prefix cache is reached through a block table (a kernel of its own: the walk then
// needs a dozen more scalar registers, which the packed kernel would otherwise pay for in spills).
// ROWSET: the step holds a subset of the rows of the (W, N, G) layout (one device's share under
// lookahead parallelism, Sec. 3.4); row ids come from p.row_ids and the mask is evaluated pair by pair.
// The body is shared by the one-step kernel and the batched one: `xcd` is the XCD this workgroup
// runs on (its id modulo 8) and `slot` its index among the step's workgroups on that XCD.
template <int D, int RT, int KS, int KC, int NSTAGE, bool PAGED = false, bool ROWSET = false, int KVB = 2, bool ROPE = false>
__device__ __forceinline__ void step_attention_body(const AttnParams& p, const int xcd, const int slot)
{
    using C = Cfg<D, RT, KS, KC, NSTAGE, KVB>;
    static_assert(KVB == 2 || (KVB == 1 && !PAGED && !ROWSET), "the quantised cache is packed and takes whole steps");
    static_assert(!ROPE || (!PAGED && !ROWSET && KVB == 2), "the rotating variant takes packed bf16 caches and whole steps");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // Consecutive workgroup ids go round-robin over the 8 XCDs (each with its own L2); put
    // the workgroups that stream the same KV head on one XCD.
    LA_STAMP(0);
    int logical = xcd * p.wg_per_xcd + slot;
    if (logical >= p.total_wg) return;
    // (the float arithmetic runs on the vector unit: tell the compiler the results are uniform,
    // or every loop and branch that depends on them is compiled as divergent control flow)
    const int unit = __builtin_amdgcn_readfirstlane(div_small(logical, p.inv_XS));  // (kvh, rb) pair
    const int xs = logical - unit * p.XS;
    const int kvh = __builtin_amdgcn_readfirstlane(div_small(unit, p.inv_row_blocks));
    const int rb = unit - kvh * p.n_row_blocks;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rt = wave / KS;   // row tile of this wave
    const int ks = wave % KS;   // which key blocks of a chunk it takes
    const int hi = lane >> 5;   // upper half-wave
    const int l32 = lane & 31;

    const unsigned lds_base = lds_address(lds);
    const int row_base = rb * C::ROWS + rt * 32;  // first row of this wave (in R space)
    const bool wave_active = row_base < p.R;     // else: only helps loading

    // ---- chunk range of this split
    int c_begin = xs * p.chunks_lo + min(xs, p.chunks_rem);
    int c_end = c_begin + p.chunks_lo + (xs < p.chunks_rem ? 1 : 0);
    bool direct = p.XS == 1;  // this pass covers every key of the rows: write `out` directly

    // ---- load addressing.  A wave-load moves 1 KB: RPW = 64 / NCH consecutive rows of 16-byte
    // pieces.  The LDS side is linear; the swizzle is applied on the global side.  Wave-load j
    // of this wave (j < LPW/2, the same for K and for V) covers chunk rows
    // (wave + j*NW)*RPW .. +RPW-1.
    static_assert(C::LPW % 2 == 0, "a wave loads as much of K as of V");
    const int lane_row = lane / C::NCH;
    const int lane_pc = lane % C::NCH;
    int ld_row[C::LPW / 2];          // the chunk row this lane fetches in wave-load j
    unsigned ld_piece[C::LPW / 2];   // byte offset of its 16-byte piece within that row
#pragma unroll
    for (int j = 0; j < C::LPW / 2; ++j) {
        ld_row[j] = (wave + j * C::NW) * (64 / C::NCH) + lane_row;
        ld_piece[j] = (unsigned)((lane_pc ^ row_swizzle<C::RBYTES>(ld_row[j])) << 4);
    }

    // This KV head's part of the four key/value tensors (wave-uniform).
    const unsigned char* const kc_head = reinterpret_cast<const unsigned char*>(p.k_cache) + (size_t)kvh * (size_t)p.cache_rows * C::RBYTES;
    const unsigned char* const vc_head = reinterpret_cast<const unsigned char*>(p.v_cache) + (size_t)kvh * (size_t)p.cache_rows * C::RBYTES;
    const unsigned char* const sk_head = reinterpret_cast<const unsigned char*>(p.step_k) + (size_t)kvh * C::RBYTES;
    const unsigned char* const sv_head = reinterpret_cast<const unsigned char*>(p.step_v) + (size_t)kvh * C::RBYTES;
    const unsigned step_stride = (unsigned)(p.kv_heads * C::RBYTES);  // step keys are strided by kv_heads
    const int n_prefix_chunks = p.n_prefix_chunks, n_P = p.P, n_T = p.T;

    // ---- the stream of chunks to request, as running wave-uniform state: every scalar
    //      instruction in the loop is paid by all waves of the workgroup, so nothing is
    //      recomputed from the chunk index
    const unsigned char* iss_k;   // K rows of the next chunk to request
    const unsigned char* iss_v;   // V rows
    int iss_rows;                 // rows from there to the end of the tensor (prefix cache or step)
    unsigned iss_stride;          // bytes between rows (the host checks it is below 2^24)
    int iss_prefix_left;          // prefix chunks still to request before the step keys start
    unsigned iss_stage;           // LDS offset of the stage the next chunk goes to
    // paged cache: chunks left in the current page, its index in the block table, and a queue of
    // the raw entries of the next four pages.  The entries are fetched with scalar loads written
    // as assembly, each batch followed by its own wait: left to the compiler they become vector
    // loads (it cannot prove that the kernel's stores leave the table alone), whose wait is a wait
    // for every direct-to-LDS load in flight.  The queue is refilled at the end of an iteration,
    // where no LDS read is pending and the wave is about to wait for its chunks anyway; a page
    // crossing in between only moves registers.  Entries are clamped when used.
    const int* const table = PAGED ? p.block_table : nullptr;
    constexpr int kNoPage = 1 << 30;  // page countdown that never reaches zero: packed cache, step keys
    int iss_page_left = kNoPage, iss_page = 0;
    int iss_ent0 = 0, iss_ent1 = 0, iss_ent2 = 0, iss_ent3 = 0;  // entries of pages iss_page+1 .. iss_page+iss_q
    int iss_q = 0;
    auto table_offset = [&](int i) {  // byte offset of entry i, never past the end of the table
        return (unsigned)__builtin_amdgcn_readfirstlane(min(i, p.table_last) * 4);
    };
    auto page_offset = [&](int raw) {  // clamped: a bad table can give wrong results, not a fault
        return (size_t)min(max(raw, 0), p.n_pages - 1) * (size_t)p.page_bytes;
    };
    auto refill_entries = [&]() {
        asm volatile("s_load_dword %0, %4, %5\n\ts_load_dword %1, %4, %6\n\ts_load_dword %2, %4, %7\n\t"
                     "s_load_dword %3, %4, %8\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(iss_ent0), "=&s"(iss_ent1), "=&s"(iss_ent2), "=&s"(iss_ent3)
                     : "s"(table), "s"(table_offset(iss_page + 1)), "s"(table_offset(iss_page + 2)),
                       "s"(table_offset(iss_page + 3)), "s"(table_offset(iss_page + 4))
                     : "memory");
        iss_q = 4;
    };
    auto seek = [&](int c) {      // next chunk to request := chunk c, into stage 0
        iss_page_left = kNoPage;
        if (c < n_prefix_chunks) {
            int key0 = c * KC;
            iss_rows = n_P - key0;
            size_t page_off = 0;
            if (table) {
                iss_page = div_small(c, p.inv_page_chunks);
                const int within = c - iss_page * p.page_chunks;
                int first;
                asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)"
                             : "=&s"(first)
                             : "s"(table), "s"(table_offset(iss_page))
                             : "memory");
                refill_entries();
                page_off = page_offset(first);
                iss_page_left = p.page_chunks - within;
                key0 = within * KC;
            }
            iss_k = kc_head + page_off + (size_t)key0 * C::RBYTES;
            iss_v = vc_head + page_off + (size_t)key0 * C::RBYTES;
            iss_stride = C::RBYTES;
            iss_prefix_left = n_prefix_chunks - c;
        } else {
            const int key0 = (c - n_prefix_chunks) * KC;
            iss_k = sk_head + (size_t)key0 * step_stride;
            iss_v = sv_head + (size_t)key0 * step_stride;
            iss_rows = n_T - key0;
            iss_stride = step_stride;
            iss_prefix_left = 0;
        }
        iss_stage = 0;
    };
    // Request the next chunk: direct-to-LDS loads, a wave-uniform 64-bit base plus a 32-bit lane
    // offset each.  Rows past the end of the tensor repeat its last row (they are masked later).
    auto issue_next = [&]() {
        const int last_row = min(KC, iss_rows) - 1;  // >= 0
        const unsigned dst = lds_base + iss_stage + (unsigned)wave * 1024u;
#pragma unroll
        for (int j = 0; j < C::LPW / 2; ++j) {
            const unsigned off = __umul24((unsigned)min(ld_row[j], last_row), iss_stride) + ld_piece[j];
            dma16_base(iss_k, off, dst + j * C::NW * 1024);
            dma16_base(iss_v, off, dst + C::KV_BYTES + j * C::NW * 1024);
        }
        iss_stage = iss_stage + C::STAGE_BYTES == (unsigned)(NSTAGE * C::STAGE_BYTES) ? 0u : iss_stage + C::STAGE_BYTES;
        iss_rows -= KC;
        if (--iss_prefix_left == 0) {  // the prefix cache is exhausted: go on with the step keys
            iss_k = sk_head;
            iss_v = sv_head;
            iss_rows = n_T;
            iss_stride = step_stride;
            iss_page_left = kNoPage;
        } else if (PAGED && --iss_page_left == 0) {  // paged cache: the next chunk starts the next page
            if (iss_q == 0) refill_entries();  // (only when more chunks are requested in a row than the queue holds)
            ++iss_page;
            const size_t page_off = page_offset(iss_ent0);
            iss_k = kc_head + page_off;
            iss_v = vc_head + page_off;
            iss_ent0 = iss_ent1;
            iss_ent1 = iss_ent2;
            iss_ent2 = iss_ent3;
            --iss_q;
            iss_page_left = p.page_chunks;
        } else {
            iss_k += (size_t)KC * iss_stride;
            iss_v += (size_t)KC * iss_stride;
        }
    };
    // The workgroup's query rows go to LDS like a chunk (same swizzle as K); rows past the end
    // repeat the last row.
    auto issue_q = [&]() {
        if constexpr (ROPE) {
            // the table rows of the step's positions: two linear blocks, 1 KB per wave-load, lanes
            // past the end repeat the last 16 bytes
            const int per_table = p.rope_block >> 10;
            const unsigned last = (unsigned)(p.rope_rows * C::ROPE_POS_BYTES - 16);
            for (int i = wave; i < 2 * per_table; i += C::NW) {
                const bool is_sin = i >= per_table;
                const int j = is_sin ? i - per_table : i;
                const unsigned off = min((unsigned)(j * 1024 + lane * 16), last);
                dma16_base(is_sin ? p.rope_sin : p.rope_cos, off,
                           lds_base + C::ROPE_OFFSET + (is_sin ? p.rope_block : 0) + j * 1024);
            }
        }
#pragma unroll
        for (int i = 0; i < C::QLPW; ++i) {
            const int wl = wave + i * C::NW;
            const int row = wl * (64 / C::QNCH) + lane / C::QNCH;
            const int lc = (lane % C::QNCH) ^ swizzle<D>(row);
            const int rr = min(rb * C::ROWS + row, p.R - 1);
            const int t = div_small(rr, p.inv_group), hh = rr - t * p.group;
            // (the host checks that q spans less than 2^31 bytes)
            const unsigned off = (unsigned)(((t * p.heads + kvh * p.group + hh) * D + lc * 8) * 2);
            dma16_base(p.q, off, lds_base + C::Q_OFFSET + wl * 1024);
        }
        if constexpr (ROWSET) {  // the row ids travel with Q (entries past the end repeat the last one)
            static_assert(C::ROWSET_MAX % (C::NW * 64) == 0, "whole rounds of wave-loads");
#pragma unroll
            for (int r = 0; r < C::ROWSET_MAX / (C::NW * 64); ++r) {
                const int slot = r * C::NW + wave;
                const int idx = min(slot * 64 + lane, n_T - 1);
                dma4_base(p.row_ids, (unsigned)idx * 4u, lds_base + C::ROWIDS_OFFSET + slot * 256);
            }
        }
    };

    // Quantised cache: a key stands for its code times the head's key scale, which goes into the
    // factor the scores are multiplied with anyway; the value scale is applied to the finished rows.
    // (Read as constants, so that they come through the scalar cache and their wait is not a wait
    // for the loads requested below.)
    float sl2 = p.scale_log2, out_scale = 1.0f;
    if constexpr (KVB == 1) {
        typedef const float __attribute__((address_space(4)))* const_f32;
        sl2 *= ((const_f32)(unsigned long long)p.k_scale)[kvh];
        out_scale = ((const_f32)(unsigned long long)p.v_scale)[kvh];
    }

    // Requests first: the stream from HBM is the critical path.  The chunks of the first
    // iteration, then Q (needed with them), then the rest of the `pre` chunks.
    int n_my = c_end - c_begin;
    int issued = 0;               // chunks of this pass requested so far
    seek(c_begin);
    auto issue_first = [&](bool with_q) {
        const int upfront = min(n_my, p.pre);
        // (paged cache: Q does not depend on the block table, so it goes first and the wait for
        // the table's first entries overlaps its issue)
        // (rotating variant: Q and the tables first as well: they are rotated in LDS while the first
        // chunks are still on their way)
        const bool q_first = table != nullptr || ROPE;
        if (q_first && with_q) issue_q();
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s) {
            if (s == C::CPI && with_q && !q_first) issue_q();
            if (s < upfront) issue_next();
        }
        issued = upfront;
    };
    issue_first(true);
    LA_STAMP(1);

    // Eight pairs of one 16-bit row in LDS (pieces of 16 bytes, swizzled with `sw`), turned in place by
    // the table rows of position digit `digit` staged behind the ring: unit c of D/16.
    auto rotate_unit = [&](unsigned char* row, int sw, int c, int digit) {
        constexpr int UPR = D / 16;  // units of eight pairs per row
        const bool inter = (p.rope_flags & 1) != 0;
        bf16x8* va = reinterpret_cast<bf16x8*>(row + (((inter ? 2 * c : c) ^ sw) << 4));
        bf16x8* vb = reinterpret_cast<bf16x8*>(row + (((inter ? 2 * c + 1 : c + UPR) ^ sw) << 4));
        const float* cs = reinterpret_cast<const float*>(lds + C::ROPE_OFFSET + digit * C::ROPE_POS_BYTES) + c * 8;
        const float* sn = reinterpret_cast<const float*>(lds + C::ROPE_OFFSET + p.rope_block + digit * C::ROPE_POS_BYTES) + c * 8;
        const f32x4 c0 = *reinterpret_cast<const f32x4*>(cs), c1 = *reinterpret_cast<const f32x4*>(cs + 4);
        const f32x4 s0 = *reinterpret_cast<const f32x4*>(sn), s1 = *reinterpret_cast<const f32x4*>(sn + 4);
        const float co[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
        const float si[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
        const bf16x8 xa = *va, xb = *vb;
        bf16x8 ya, yb;
        rope_eight_pairs(xa, xb, co, si, inter, ya, yb);
        *va = ya;
        *vb = yb;
    };

    if constexpr (ROPE) {
        // Q and the table rows are older than every chunk requested so far: wait for them alone,
        // then every thread turns eight pairs of the workgroup's query rows in place (the same
        // arithmetic as the pass of its own).  The barrier of the first iteration orders these
        // writes before the waves read their rows into registers.
        // (a ring requested in full: the first chunk is waited for as well; the counter has 6 bits)
        wait_young<C::LPW, NSTAGE - 1>(min(issued, NSTAGE - 1));
        __syncthreads();
        for (int u = tid; u < C::ROWS * (D / 16); u += C::NT) {
            const int r = u / (D / 16), c = u - r * (D / 16);
            const int rr = min(rb * C::ROWS + r, p.R - 1);
            const int digit = min(step_row_digit(div_small(rr, p.inv_group), p.W, p.N, p.inv_W, p.inv_n1), p.rope_rows - 1);
            rotate_unit(lds + C::Q_OFFSET + r * C::QRBYTES, swizzle<D>(r), c, digit);
        }
    }

    // which step keys this lane's row may see
    const int t_lane = div_small(min(row_base + l32, p.R - 1), p.inv_group);  // step row of this lane's query row
    const RowVis vis = row_visibility(t_lane, p.W, p.N, p.inv_W, p.inv_n1);
    RowPos qpos = {0, 0, 0};  // row-subset variant: filled once the ids have landed
    bf16x8 qreg[D / 16];  // B operand of S^T = K Q^T: row l32, d = k16*16 + hi*8 .. +8

    // o[db]: O^T accumulators of this wave's tile in the main loop; after the key-split merge,
    // o[0 .. SPW-1] are the tile's 32-column slices db0 .. db0+SPW-1 summed over all key splits
    f32x16 o[C::DB];
    float m_run, l_run;
    const int db0 = KS > 1 ? ks * C::SPW : 0;
    // Which of an iteration's chunks this wave takes.  Waves w and w + NW/2 (equal key index,
    // different tiles when RT = 2) share a SIMD: odd tiles take the chunks in rotated order, so
    // that a last iteration with fewer chunks than CPI leaves one busy wave on every SIMD
    // instead of two on half of them.
    const int cw = KS > C::KB ? (ks / C::KB + rt) % C::CPI : 0;
    // which waves ask for the recompute pass (a word of LDS, addressed as such)
    typedef __attribute__((address_space(3))) unsigned lds_u32;
    volatile lds_u32* s_recompute = nullptr;  // (set once a pass knows where its merge area lies)
    unsigned store_mask = ~0u;  // recompute pass: which waves write their slices
    // the wave's counter of this split group
    unsigned* const my_ticket = p.XS > 1 ? p.tickets + ((size_t)unit * C::NW + wave) * kTicketStride : nullptr;

    // LDS read offsets of this lane relative to the start of a stage; the loop adds only the stage.
    //   K operand: key row kb*32 + l32, pieces k16*2 + hi (swizzled).
    //   V^T operand: k-slot e of half `hi` of 16-key step kk is key kb*32 + kk*16 + (e/4)*8 + hi*4 + e%4
    //   (the layout S^T leaves P in).  A 16-lane block reads 4 keys x 16 columns; the transposing
    //   read hands lane n column n.  The swizzle of those rows does not depend on kb or kk.
    const int kb_first = KS >= C::KB ? ks % C::KB : ks;  // this wave's (first) block of a chunk
    // (quantised cache: a 16-byte piece of K feeds two MFMA steps and one transposing read of V
    // covers 8 keys, so half the offsets are in use)
    constexpr int NKOFF = KVB == 2 ? D / 16 : D / 32;
    unsigned k_off[NKOFF], v_off[2][C::DB];
    {
        const int krow = kb_first * 32 + l32;
        const int ksw = row_swizzle<C::RBYTES>(krow);
#pragma unroll
        for (int j = 0; j < NKOFF; ++j)
            k_off[j] = (unsigned)(krow * C::RBYTES + (((j * 2 + hi) ^ ksw) << 4));
        const int b16 = lane >> 4, i16 = lane & 15;
        if constexpr (KVB == 2) {
            const int jj = i16 >> 2, q4 = i16 & 3;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int vrow = kb_first * 32 + hi * 4 + jj + r * 8;  // e = 0..3 (r = 0), 4..7 (r = 1); kk = 0
                const int sw = swizzle<D>(vrow);
#pragma unroll
                for (int db = 0; db < C::DB; ++db) {
                    const int col = db * 32 + (b16 & 1) * 16 + q4 * 4;
                    const int lc = col >> 3, within = (col & 7) * 2;
                    v_off[r][db] = (unsigned)(C::KV_BYTES + vrow * C::RBYTES + ((lc ^ sw) << 4) + within);
                }
            }
        } else {
            // The 8-bit transposing read takes, from the 16 lanes of a block, 8 rows of 16 bytes (lane
            // 2b + h supplies bytes h*8 .. +7 of row b) and hands lane n the 8 bytes of column n.
            // Row b is the key of k-slot b: (b/4)*8 + hi*4 + b%4.
            const int b = i16 >> 1, h = i16 & 1;
            const int vrow = kb_first * 32 + (b >> 2) * 8 + hi * 4 + (b & 3);  // kk = 0
            const int sw = row_swizzle<C::RBYTES>(vrow);
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                const int lc = db * 2 + (b16 & 1);  // 16 columns = one piece
                v_off[0][db] = (unsigned)(C::KV_BYTES + vrow * C::RBYTES + ((lc ^ sw) << 4) + h * 8);
                v_off[1][db] = 0u;
            }
        }
    }

    for (int pass = 0;; ++pass) {
        m_run = kNegInf;
        l_run = 0.0f;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] = 0.0f;
        if (pass > 0) {
            n_my = c_end - c_begin;
            seek(c_begin);
            issue_first(false);
        }

        // Iteration `it` consumes chunks done .. done+CPI-1 of this pass (done = it*CPI).
        int cons_c = c_begin + cw;                     // the chunk this wave takes next
        unsigned cons_stage = (unsigned)cw * C::STAGE_BYTES;  // and the LDS offset of its stage
        for (int it = 0, done = 0; done < n_my; ++it, done += C::CPI) {
            // Wait for this wave's loads of the chunks needed now; younger ones stay in flight.
            wait_young<C::LPW, NSTAGE - C::CPI>(issued - min(n_my, done + C::CPI));
            __syncthreads();  // these chunks are complete in LDS; everyone is done with the last ones
            if (it < 4) LA_STAMP(8 + 2 * it);
            if constexpr (ROPE) {
                // Step keys that come as the projection left them: the chunks of this iteration that
                // hold step rows are turned in place by all threads, once per workgroup, before anyone
                // multiplies with them (row r of step chunk c is step row c*KC + r; rows past the end
                // repeat the last row's position and are masked out anyway).
                if (p.rope_flags & 2) {
                    bool any = false;
#pragma unroll
                    for (int j = 0; j < C::CPI; ++j) {
                        const int c_abs = c_begin + done + j;
                        if (done + j < n_my && c_abs >= n_prefix_chunks) {  // (uniform over the workgroup)
                            any = true;
                            unsigned char* stage = lds + ((done + j) % NSTAGE) * C::STAGE_BYTES;
                            const int t0 = (c_abs - n_prefix_chunks) * KC;
                            for (int u = tid; u < KC * (D / 16); u += C::NT) {
                                const int r = u / (D / 16), c = u - r * (D / 16);
                                const int digit = min(step_row_digit(min(t0 + r, n_T - 1), p.W, p.N, p.inv_W, p.inv_n1), p.rope_rows - 1);
                                rotate_unit(stage + r * C::RBYTES, swizzle<D>(r), c, digit);
                            }
                        }
                    }
                    if (any) __syncthreads();
                }
            }
            if (it == 0 && pass == 0) {
                // Q has landed with the first chunks: move this wave's rows to registers
                const int qrow = rt * 32 + l32;
                const unsigned char* qr = lds + C::Q_OFFSET + qrow * C::QRBYTES;
                const int qsw = swizzle<D>(qrow);
#pragma unroll
                for (int k16 = 0; k16 < D / 16; ++k16) {
                    // the 8 columns of MFMA step k16 in this half-wave: k16*16 + hi*8 .. +7, or, where a
                    // 16-byte piece of 8-bit keys spans two steps, (k16/2)*32 + hi*16 + (k16%2)*8 .. +7
                    const int piece = KVB == 2 ? k16 * 2 + hi : (k16 >> 1) * 4 + hi * 2 + (k16 & 1);
                    qreg[k16] = *reinterpret_cast<const bf16x8*>(qr + ((piece ^ qsw) << 4));
                }
                if constexpr (ROWSET) {
                    const int t_full = 1 + (p.W + p.G) * (p.N - 1);
                    const int tq = *reinterpret_cast<const int*>(lds + C::ROWIDS_OFFSET + t_lane * 4);
                    qpos = row_position(min(max(tq, 0), t_full - 1), p.W, p.N, p.inv_W, p.inv_n1);
                }
            }
            // Up to CPI chunks are requested per iteration, into stages the last iteration freed:
            // the ring has room up to chunk done + NSTAGE - 1.  A computing wave issues its first
            // request behind a batch of MFMAs, which run on meanwhile.
            const int room = min(n_my, done + NSTAGE);
            int slots_left = C::CPI;
            auto issue_slot = [&]() {
                if (issued < room) {
                    issue_next();
                    ++issued;
                }
                --slots_left;
            };
            // With two chunks per iteration the first refill goes out right here: at long prefixes an
            // iteration waits for the data requested one iteration earlier, so every request that
            // leaves sooner shortens it (70B shape -5 %, 13B -2.5 %); the second follows the first
            // batch of MFMAs (both at once measured slower: the requests stall the wave).
            if (slots_left > 1) issue_slot();
            bool compute = done + cw < n_my && wave_active;
            if (compute) {
            const bool is_step = cons_c >= n_prefix_chunks;
            const int chunk_key0 = (cons_c - (is_step ? n_prefix_chunks : 0)) * KC;
            const int limit = is_step ? n_T : n_P;

#pragma unroll
            for (int kbw = 0; kbw < C::KBW; ++kbw) {
                const int kb = KS >= C::KB ? ks % C::KB : ks + kbw * KS;
                const int key0 = chunk_key0 + kb * 32;
                if (key0 >= limit) continue;  // block entirely past the end (wave-uniform)

                // ---- which of this lane's 16 keys of the block its row may see (bit (i/4)*8 + i%4 for
                //      score register i).  A step block that no row of the tile sees at all is
                //      skipped before anything is read: with wide windows most step blocks are.
                const bool full = !is_step && (key0 + 32 <= limit);  // wave-uniform
                unsigned word = 0xFFFFFFFFu;
                if (!full) {
                    if (is_step && ROWSET) {
                        // pair by pair over this lane's 16 keys of the block (ids from LDS, four at a time)
                        word = 0;
#pragma unroll
                        for (int grp = 0; grp < 4; ++grp) {
                            const int c0 = key0 + grp * 8 + hi * 4;
                            const i32x4 g4 = *reinterpret_cast<const i32x4*>(lds + C::ROWIDS_OFFSET + c0 * 4);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const bool ok = c0 + e < n_T && visible_pair(qpos, g4[e], p.W, p.N, p.inv_W, p.inv_n1);
                                word |= (ok ? 1u : 0u) << (grp * 8 + hi * 4 + e);
                            }
                        }
                    } else if (is_step) {
                        word = step_block_word(vis, key0);
                    } else {
                        const int n = limit - key0;  // 1..31
                        word = (1u << n) - 1u;
                    }
                    word = (word >> (hi * 4)) & 0x0F0F0F0Fu;
                    if (is_step && __builtin_amdgcn_ballot_w64(word != 0u) == 0ull) continue;
                }

                // ---- operands: all K pieces of the block, and the V pieces of its first 16 keys,
                //      are requested from LDS before the first MFMA (LDS answers in order)
                const unsigned char* blk = lds + (cons_stage + (unsigned)(kbw * KS * 32 * C::RBYTES));
                bf16x8 kf[KVB == 2 ? D / 16 : 1];
                u32x4 kraw[KVB == 2 ? 1 : D / 32];   // quantised: 16 codes per read, converted at the MFMA
                if constexpr (KVB == 2) {
#pragma unroll
                    for (int k16 = 0; k16 < D / 16; ++k16)
                        kf[k16] = *reinterpret_cast<const bf16x8*>(blk + k_off[k16]);
                } else {
#pragma unroll
                    for (int j = 0; j < D / 32; ++j) kraw[j] = *reinterpret_cast<const u32x4*>(blk + k_off[j]);
                }
                bf16x8 vf[2][KVB == 2 ? C::DB : 1];
                i32x2 vraw[2][KVB == 2 ? 1 : C::DB];
                auto read_v = [&](int kk) {
#pragma unroll
                    for (int db = 0; db < C::DB; ++db) {
                        const unsigned char* a0 = blk + v_off[0][db] + kk * 16 * C::RBYTES;
                        if constexpr (KVB == 2) {
                            const unsigned char* a1 = blk + v_off[1][db] + kk * 16 * C::RBYTES;
                            union { struct { short4v a, b; } s; bf16x8 v; } u;
                            u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (short4v __attribute__((address_space(3)))*)a0);
                            u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (short4v __attribute__((address_space(3)))*)a1);
                            vf[kk][db] = u.v;
                        } else {
                            vraw[kk][db] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                                (i32x2 __attribute__((address_space(3)))*)a0);
                        }
                    }
                };
                read_v(0);

                // ---- S^T block: 32 keys x 32 rows
                f32x16 s;
#pragma unroll
                for (int i = 0; i < 16; ++i) s[i] = 0.0f;
#pragma unroll
                for (int k16 = 0; k16 < D / 16; ++k16) {
                    bf16x8 a;
                    if constexpr (KVB == 2) a = kf[k16];
                    else a = fp8x8_to_bf16(kraw[k16 >> 1][(k16 & 1) * 2], kraw[k16 >> 1][(k16 & 1) * 2 + 1]);
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[k16], s, 0, 0, 0);
                }
                if (slots_left > 0) issue_slot();
                read_v(1);  // in flight during the softmax arithmetic

                // ---- mask, running max, exponentials
                if (!full) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int bit = (i >> 2) * 8 + (i & 3);  // hi*4 already shifted out
                        if (!((word >> bit) & 1u)) s[i] = kNegInf;
                    }
                }
                if (full) settle_mfma_result(s);  // (the mask above is compiler-visible arithmetic on s)
                float mx = max3(s[0], s[1], s[2]);
#pragma unroll
                for (int i = 3; i < 15; i += 2) mx = max3(mx, s[i], s[i + 1]);
                mx = max_across_halves(max2(mx, s[15]));
                // Scores stay unscaled; exp(x/sqrt(d)) = exp2(x * scale_log2).  The reference
                // m_run only moves when the block maximum exceeds it by more than 2^8 in the
                // exponent (or no key was seen yet): softmax is invariant to the reference, and
                // skipping small moves saves rescaling the accumulators nearly every time.
                const bool move = (mx - m_run) * sl2 > 8.0f || m_run == kNegInf;
                const float m_new = move ? mx : m_run;
                const float m_use = (m_new == kNegInf) ? 0.0f : m_new;  // the row has seen no key at all
                const float neg_mc = -m_use * sl2;
                if (__builtin_amdgcn_ballot_w64(move) != 0ull) {
                    const float alpha = fast_exp2(__builtin_fmaf(m_run, sl2, neg_mc));
                    l_run *= alpha;
#pragma unroll
                    for (int db = 0; db < C::DB; ++db)
#pragma unroll
                        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
                }
                m_run = m_new;
                // P in bf16, as the PV product uses it; the row sum adds up those same rounded
                // values (two per instruction), so that numerator and denominator agree
                bf16x8 pf[2];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    pf[i >> 3][i & 7] = (__bf16)fast_exp2(__builtin_fmaf(s[i], sl2, neg_mc));
                {
                    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
                    float psum0 = 0.0f, psum1 = 0.0f;
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        psum0 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{pf[kk][0], pf[kk][1]}, ones, psum0, false);
                        psum1 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{pf[kk][2], pf[kk][3]}, ones, psum1, false);
                        psum0 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{pf[kk][4], pf[kk][5]}, ones, psum0, false);
                        psum1 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{pf[kk][6], pf[kk][7]}, ones, psum1, false);
                    }
                    l_run += psum0 + psum1;
                }

                // ---- O^T += V^T P^T
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int db = 0; db < C::DB; ++db) {
                        bf16x8 a;
                        if constexpr (KVB == 2) a = vf[kk][db];
                        else a = fp8x8_to_bf16((unsigned)vraw[kk][db][0], (unsigned)vraw[kk][db][1]);
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kk], o[db], 0, 0, 0);
                    }
            }
            }
#pragma unroll
            for (int j = 0; j < C::CPI; ++j)
                if (slots_left > 0) issue_slot();
            if (table && iss_q < 4) refill_entries();
            cons_c += C::CPI;
            cons_stage += C::CPI * C::STAGE_BYTES;
            if (cons_stage >= (unsigned)(NSTAGE * C::STAGE_BYTES)) cons_stage -= NSTAGE * C::STAGE_BYTES;
            if (it < 4) LA_STAMP(9 + 2 * it);
        }

        LA_STAMP(3);
        // the two half-waves of a row hold the sums over their own keys
        l_run += __shfl_xor(l_run, 32, 64);

        // ---- where the merge leaves its data: ring stages that nobody reads any more.  The
        //      waves are at most one iteration apart, so once a wave is past the loop the others
        //      read the last iteration's stages at most: anywhere else may be written at once.
        unsigned char* merge_area = lds;
        if constexpr (C::MERGE_EARLY) {
            const int iters = (n_my + C::CPI - 1) / C::CPI;
            const int first = ((iters - 1) * C::CPI) % NSTAGE;       // stages first .. first + CPI - 1 (mod NSTAGE) are live
            if (first + C::CPI <= NSTAGE) {
                const int below = first, above = NSTAGE - C::CPI - first;
                merge_area = lds + (above >= below ? (first + C::CPI) * C::STAGE_BYTES : 0);
            } else {
                merge_area = lds + (first + C::CPI - NSTAGE) * C::STAGE_BYTES;
            }
        } else {
            __syncthreads();  // all stages consumed: LDS is reused below
        }
        LA_STAMP(16);
        s_recompute = (volatile lds_u32*)(merge_area + C::MERGE_BYTES);
        if (tid == 0) *s_recompute = 0u;
        if (KS == 1) __syncthreads();  // (with key-split waves the merge's barrier does this)

        // ---- merge the KS waves of a row tile; the key index is uniform in a wave, and branching
        //      on it keeps every register index a compile-time constant
        if (KS > 1) {
            const float sc = sl2;
            if (ks == 0) merge_key_splits<C, KS, 0>(merge_area, rt, lane, wave_active, o, m_run, l_run, sc);
            if (KS > 1 && ks == 1) merge_key_splits<C, KS, (KS > 1 ? 1 : 0)>(merge_area, rt, lane, wave_active, o, m_run, l_run, sc);
            if (KS > 2 && ks == 2) merge_key_splits<C, KS, (KS > 2 ? 2 : 0)>(merge_area, rt, lane, wave_active, o, m_run, l_run, sc);
            if (KS > 3 && ks == 3) merge_key_splits<C, KS, (KS > 3 ? 3 : 0)>(merge_area, rt, lane, wave_active, o, m_run, l_run, sc);
            static_assert(KS <= 4, "one branch per key index");
        }
        LA_STAMP(4);
        if (direct) break;

        // ---- split combine, wave by wave (no workgroup barrier): a wave stores its slices with its
        //      rows' (m, l), waits for the L2 of this XCD to acknowledge the stores and takes a ticket
        //      of its own; the wave that arrives last in its group merges the XS partials of these
        //      slices in index order (so results do not depend on arrival order)
        if (wave_active) {
            unsigned char* const group_base = reinterpret_cast<unsigned char*>(p.partials) +
                                              (size_t)unit * p.XS * C::PART_WG_BYTES + (size_t)wave * C::PART_WAVE_BYTES;
            {
                unsigned char* dst = group_base + (size_t)xs * C::PART_WG_BYTES;
#pragma unroll
                for (int u = 0; u < C::SPW; ++u)
#pragma unroll
                    for (int i8 = 0; i8 < 2; ++i8) {
                        bf16x8 v;
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (__bf16)o[u][i8 * 8 + e];
                        // (streaming stores: the partials are read once, by one other wave, and measured
                        // faster this way than with the default cache policy)
                        __builtin_nontemporal_store(v, reinterpret_cast<bf16x8*>(dst + ((u * 2 + i8) * 64 + lane) * 16));
                    }
                *reinterpret_cast<f32x2*>(dst + C::PART_ACC_BYTES + lane * 8) = f32x2{m_run, l_run};
            }
            __builtin_amdgcn_s_waitcnt(0);
            LA_STAMP(5);
            unsigned role = 0;  // 0 not last, 1 last and co-located, 2 last but spread over several XCDs
            if (lane == 0) {
                // One atomic carries the arrival count and, to tell whether every member of the group
                // ran on the same XCD (and so shares one L2), the sum and the sum of squares of the
                // members' XCD ids: XS * sum(x^2) == (sum x)^2 holds iff all ids are equal.
                const unsigned x = xcc_id();
                const unsigned mine = 1u | (x << 8) | ((x * x) << 18);
                const unsigned total = atomicAdd(my_ticket, mine) + mine;
                const unsigned cnt = total & 0xffu, sum = (total >> 8) & 0x3ffu, sq = total >> 18;
                if (cnt == (unsigned)p.XS) {
                    *my_ticket = 0u;  // everyone has arrived; clean for the next call
                    role = (sq * (unsigned)p.XS == sum * sum && !p.force_recompute) ? 1u : 2u;
                }
            }
            role = __builtin_amdgcn_readfirstlane(role);
            LA_STAMP(6);
            if (role == 1) {
                // ---- all partials sit in the L2 this XCD shares: four splits per trip to the L2
                constexpr int MB = 4;
                float m_acc = kNegInf, l_acc = 0.0f;
                float acc[C::SPW][16];
#pragma unroll
                for (int u = 0; u < C::SPW; ++u)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[u][i] = 0.0f;
                for (int s0 = 0; s0 < p.XS; s0 += MB) {
                    f32x2 ml[MB];
                    bf16x8 v[MB][C::SPW][2];
#pragma unroll
                    for (int w = 0; w < MB; ++w) {
                        const int s2 = min(s0 + w, p.XS - 1);
                        const unsigned char* src = group_base + (size_t)s2 * C::PART_WG_BYTES;
                        ml[w] = *reinterpret_cast<const f32x2*>(src + C::PART_ACC_BYTES + lane * 8);
#pragma unroll
                        for (int u = 0; u < C::SPW; ++u)
#pragma unroll
                            for (int i8 = 0; i8 < 2; ++i8)
                                v[w][u][i8] = *reinterpret_cast<const bf16x8*>(src + ((u * 2 + i8) * 64 + lane) * 16);
                    }
                    LA_STAMP(18);
                    // batch maximum, then one weight per split: acc = acc * a0 + sum_w v_w * a_w
                    float mb = m_acc;
#pragma unroll
                    for (int w = 0; w < MB; ++w)
                        if (s0 + w < p.XS) mb = fmaxf(mb, ml[w][0]);
                    const float m_use = (mb == kNegInf) ? 0.0f : mb;
                    const float a0 = fast_exp2((m_acc - m_use) * sl2);
                    l_acc *= a0;
                    if (s0 > 0) {
#pragma unroll
                        for (int u = 0; u < C::SPW; ++u)
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc[u][i] *= a0;
                    }
                    m_acc = mb;
#pragma unroll
                    for (int w = 0; w < MB; ++w) {
                        const float aw = s0 + w < p.XS ? fast_exp2((ml[w][0] - m_use) * sl2) : 0.0f;
                        l_acc = __builtin_fmaf(ml[w][1], aw, l_acc);
#pragma unroll
                        for (int u = 0; u < C::SPW; ++u)
#pragma unroll
                            for (int i8 = 0; i8 < 2; ++i8)
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    acc[u][i8 * 8 + e] = __builtin_fmaf((float)v[w][u][i8][e], aw, acc[u][i8 * 8 + e]);
                    }
                }
                const float inv = out_scale / l_acc;
#pragma unroll
                for (int u = 0; u < C::SPW; ++u) {
                    f32x16 vals;
#pragma unroll
                    for (int i = 0; i < 16; ++i) vals[i] = acc[u][i];
                    store_slice<C>(p, rb, kvh, rt, db0 + u, l32, hi, vals, inv);
                }
                LA_STAMP(7);
            }
            // ---- a wave that arrived last in a group spread over several XCDs, whose L2s are not
            //      coherent with each other inside a kernel, cannot trust the partials: the whole
            //      workgroup then recomputes its rows over every chunk from the read-only inputs (which
            //      are always coherent), and the waves that asked for it write their slices directly
            if (role == 2 && lane == 0) atomicOr(reinterpret_cast<unsigned*>(merge_area + C::MERGE_BYTES), 1u << wave);
        }
        __syncthreads();
        store_mask = (unsigned)__builtin_amdgcn_readfirstlane((int)*s_recompute);
        if (store_mask == 0u) return;
        __syncthreads();  // everyone has read the mask before the next pass clears it
        c_begin = 0;
        c_end = p.n_chunks;
        direct = true;
    }

    // ---- normalise and write this wave's slices (>= 1 visible key per row, so l > 0)
    if (wave_active && ((store_mask >> wave) & 1u)) {
        const float inv = out_scale / l_run;
#pragma unroll
        for (int u = 0; u < C::SPW; ++u) store_slice<C>(p, rb, kvh, rt, db0 + u, l32, hi, o[u], inv);
    }
}

template <int D, int RT, int KS, int KC, int NSTAGE, bool PAGED = false, bool ROWSET = false, int KVB = 2, bool ROPE = false>
__global__ __launch_bounds__(RT* KS * 64) void step_attention_kernel(const AttnParams)
{
    const AttnParams& p = warmed_arguments<AttnParams>();
    step_attention_body<D, RT, KS, KC, NSTAGE, PAGED, ROWSET, KVB, ROPE>(p, (int)(blockIdx.x & 7), (int)(blockIdx.x >> 3));
}

// Several independent steps (sequences) in one launch: on every XCD, step i owns the slots
// slot0[i] .. slot0[i+1]-1.  Workgroups are handed out in id order, so the steps start in the
// order given (longest first) and the tail of one overlaps the head of the next.
constexpr int kMaxBatch = 16;
struct BatchSlots {
    int slot0[kMaxBatch + 1];
    int n;
};
struct BatchParams {
    AttnParams seq[kMaxBatch];
    BatchSlots slots;
};

template <int D, int RT, int KS, int KC, int NSTAGE, bool PAGED = false>
__global__ __launch_bounds__(RT* KS * 64) void step_attention_batch_kernel(const BatchParams)
{
    // two misses of the scalar cache: the slot table, then the arguments of this workgroup's step
    const BatchSlots& sl = warmed_arguments<BatchSlots>((unsigned)offsetof(BatchParams, slots));
    const int slot = (int)(blockIdx.x >> 3);
    int i = 0;
#pragma unroll
    for (int k = 1; k < kMaxBatch; ++k)
        if (k < sl.n && slot >= sl.slot0[k]) i = k;
    const AttnParams& p = warmed_arguments<AttnParams>((unsigned)i * (unsigned)sizeof(AttnParams));
    step_attention_body<D, RT, KS, KC, NSTAGE, PAGED>(p, (int)(blockIdx.x & 7), slot - sl.slot0[i]);
}

// Scratch memory of the entry point that allocates nothing (la_step_attention_noalloc): the
// tickets and the split partials of one step, in the library's own image.  Every device the
// library runs on holds one copy until the process ends.  In host code the name below is only a
// handle: its device address is looked up once per device (fixed_workspace) and only that
// pointer is handed to kernels.
constexpr size_t kFixedTicketBytes = (size_t)128 << 10;          // 128 split groups x 8 waves, 128 bytes apart
constexpr size_t kFixedPartialBytes = (size_t)12 << 20;         // 12 MiB of partials
static __device__ __align__(256) unsigned char scratch[kFixedTicketBytes + kFixedPartialBytes];

__global__ void clear_words_kernel(unsigned* words, int n)
{
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < n) words[i] = 0u;
}

// ---------------------------------------------------------------------------------------
// host side

// Testing hooks (la_debug_override; the environment gives their values at the first call): a
// decomposition forced by hand, and the recompute path of a split group forced on.
struct Overrides {
    bool has_plan = false;
    int plan[6] = {0, 0, 0, 0, 0, 0};  // RT, KS, XS, NS, KC, PRE (XS = 0, PRE = 0: heuristic)
    int batch_rows = 0;                // 2 or 4: 32-row tiles per workgroup of a batched launch
    int rowtile = -1;                  // 1 / 0: the kernel without partials forced on / off (-1: heuristic)
    bool force_recompute = false;
};
std::mutex g_config_mutex;  // the overrides, and the once-per-device kernel attributes
Overrides g_overrides;
bool g_overrides_from_env = false;

bool parse_plan(const char* text, Overrides& o)
{
    int v[6] = {0, 0, 0, 0, 0, 0};
    o.has_plan = text && sscanf(text, "%d,%d,%d,%d,%d,%d", &v[0], &v[1], &v[2], &v[3], &v[4], &v[5]) >= 5;
    for (int i = 0; i < 6; ++i) o.plan[i] = o.has_plan ? v[i] : 0;
    return o.has_plan;
}

void overrides_from_env_locked()
{
    if (g_overrides_from_env) return;
    g_overrides_from_env = true;
    parse_plan(getenv("LA_ATTN_PLAN"), g_overrides);
    const char* b = getenv("LA_BATCH_PLAN");
    g_overrides.batch_rows = (b && (b[0] == '2' || b[0] == '4')) ? b[0] - '0' : 0;
    const char* f = getenv("LA_FORCE_RECOMPUTE");
    g_overrides.force_recompute = f && f[0] == '1';
}

Overrides current_overrides()
{
    std::lock_guard<std::mutex> lock(g_config_mutex);
    overrides_from_env_locked();
    return g_overrides;
}

// hipFuncSetAttribute once per kernel and device (`done` is that kernel's own table)
la_status set_lds_attribute_once(const void* kern, int lds_bytes, bool (&done)[16])
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return fail(LA_EHIP, "hipGetDevice failed");
    std::lock_guard<std::mutex> lock(g_config_mutex);
    if (!done[dev]) {
        const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return fail(LA_EHIP, "hipFuncSetAttribute(%d bytes LDS): %s", lds_bytes, hipGetErrorString(e));
        done[dev] = true;
    }
    return LA_OK;
}

struct Plan {
    int RT, KS, XS, NS;       // NS = LDS stages
    int PRE;                  // chunks requested before the loop (0 = all stages)
    int KC;                   // keys per chunk
    int n_row_blocks;
    int n_prefix_chunks, n_chunks;
    size_t partial_bytes_per_wg;
};

// Bytes of one workgroup's partial (Cfg::PART_WG_BYTES): per wave its slices as bf16 and (m, l).
size_t partial_wg_bytes(int D, int RT, int KS)
{
    const int DB = D / 32, SPW = KS > 1 ? DB / KS : DB;
    return (size_t)RT * KS * ((size_t)SPW * 16 * 64 * 2 + 64 * 8);
}

// Most LDS stages that fit beside the workgroup's Q rows.
int max_stages(int D, int RT)
{
    if (D != 128) return 4;
    return RT <= 2 ? 4 : 3;
}

bool plan_supported(int D, int RT, int KS, int NS, int KC)
{
    if (KC == 32) return D == 128 && RT == 2 && KS == 2 && NS == 9;
    if (KC != 64) return false;
    if (KS == 4) return D == 128 && RT == 2 && NS == 4;
    if (RT == 4 && KS == 2) return D == 128 && NS == 4;
    if (NS != 2 && NS != max_stages(D, RT)) return false;
    if (D == 128)
        return (RT == 1 && KS == 2) || (RT == 2 && KS == 2) || (RT == 4 && KS == 1) || (RT == 2 && KS == 1);
    return (RT == 1 && KS == 2) || (RT == 2 && KS == 2) || (RT == 4 && KS == 1);
}

// Plans compiled for a paged cache: the ones the heuristic below picks.
bool paged_plan_supported(int D, int RT, int KS, int NS, int KC)
{
    if (KC != 64 || NS != 4) return false;
    if (D == 128) return (RT == 2 && KS == 4) || (RT == 4 && KS == 2) || (RT == 1 && KS == 2) || (RT == 2 && KS == 2);
    return (RT == 1 && KS == 2) || (RT == 2 && KS == 2);
}

// Plans compiled for a row subset: as for a paged cache, without the 128-row plan (the ids need
// 4 KB of LDS that it does not leave).
bool rowset_plan_supported(int D, int RT, int KS, int NS, int KC)
{
    return paged_plan_supported(D, RT, KS, NS, KC) && RT != 4;
}

Plan make_plan(const Overrides& ov, int P, int T, int group, int kv_heads, int D, bool paged = false, bool rowset = false,
               bool rope = false)
{
    Plan pl;
    const int R = T * group;
    const int tiles = (R + 31) / 32;
    pl.KC = 64;
    // Workgroups of eight waves, two per SIMD, so that one wave's MFMAs overlap the other's
    // softmax arithmetic: 64 rows whose four waves per tile split the keys (measured best from the
    // 7B shape up to grouped-query shapes with a few hundred rows per KV head), or 128 rows with two
    // key-split waves per tile when there are many rows and a long prefix (more reuse of each
    // chunk in LDS).  Head dimension 64 and single-tile problems keep four-wave workgroups.
    if (tiles <= 1) { pl.RT = 1; pl.KS = 2; }
    else if (D != 128) { pl.RT = 2; pl.KS = 2; }
    else if (tiles >= 16 && (P + T) / pl.KC >= 64 && !rowset && !rope) { pl.RT = 4; pl.KS = 2; }  // (no LDS left for tables)
    else { pl.RT = 2; pl.KS = 4; }
    pl.XS = 0;
    pl.NS = 0;
    pl.PRE = 0;
    // testing hook: a decomposition forced by hand, "RT,KS,XS,NS,KC[,PRE]" (XS = 0, PRE = 0: heuristic)
    if (ov.has_plan) {
        const int b = ov.plan[0], c = ov.plan[1], d = ov.plan[2], e = ov.plan[3], f = ov.plan[4], g = ov.plan[5];
        if (plan_supported(D, b, c, e, f) && (!paged || paged_plan_supported(D, b, c, e, f)) &&
            (!rowset || rowset_plan_supported(D, b, c, e, f))) {
            pl.RT = b; pl.KS = c; pl.XS = d; pl.NS = e; pl.KC = f;
            pl.PRE = g;
        }
    }
    if (pl.NS == 0) pl.NS = (pl.KS == 4 || (pl.RT == 4 && pl.KS == 2)) ? 4 : max_stages(D, pl.RT);
    pl.n_prefix_chunks = (P + pl.KC - 1) / pl.KC;
    pl.n_chunks = pl.n_prefix_chunks + (T + pl.KC - 1) / pl.KC;
    const int rows_wg = pl.RT * 32;
    pl.n_row_blocks = (R + rows_wg - 1) / rows_wg;
    if (pl.XS <= 0) {
        // One workgroup per compute unit and never more than 256 in all: a workgroup owns most
        // of a compute unit's LDS, so a second round would only start when the first has ended.
        const int units = kv_heads * pl.n_row_blocks;
        int xs = 256 / units;
        if (xs > pl.n_chunks / 2) xs = pl.n_chunks / 2;
        pl.XS = xs < 1 ? 1 : xs;
    }
    if (pl.XS > pl.n_chunks) pl.XS = pl.n_chunks;
    if (pl.XS > 64) pl.XS = 64;
    pl.partial_bytes_per_wg = partial_wg_bytes(D, pl.RT, pl.KS);
    return pl;
}

template <int D, int RT, int KS, int NSTAGE, int KC = 64, bool PAGED = false, bool ROWSET = false, int KVB = 2, bool ROPE = false>
la_status launch_cfg(const AttnParams& prm, hipStream_t stream)
{
    using C = Cfg<D, RT, KS, KC, NSTAGE, KVB>;
    constexpr int kLds = C::LDS_BYTES + (ROWSET ? C::ROWIDS_BYTES : 0) + (ROPE ? C::ROPE_MAX_BYTES : 0);
    static_assert(kLds <= 160 * 1024, "LDS of a compute unit");
    if (ROPE && 2 * prm.rope_block > C::ROPE_MAX_BYTES)
        return fail(LA_EUNSUPPORTED, "la_step_attention_rope: %d positions of cosines and sines do not fit beside this "
                                     "decomposition (%d bytes of LDS left): rotate q with la_step_rope instead",
                    prm.rope_rows, C::ROPE_MAX_BYTES);
    auto kern = step_attention_kernel<D, RT, KS, KC, NSTAGE, PAGED, ROWSET, KVB, ROPE>;
    static bool attr_set[16] = {false};
    const la_status st = set_lds_attribute_once(reinterpret_cast<const void*>(kern), kLds, attr_set);
    if (st != LA_OK) return st;
    const unsigned grid = (unsigned)prm.wg_per_xcd * 8u;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), kLds, stream, prm);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_step_attention launch: %s", hipGetErrorString(e));
    return LA_OK;
}

}  // namespace

size_t step_attention_workspace_bytes(int P, int W, int N, int G, int heads, int kv_heads, int head_dim)
{
    const int T = 1 + (W + G) * (N - 1);
    const Plan pl = make_plan(current_overrides(), P, T, heads / kv_heads, kv_heads, head_dim);
    if (pl.XS <= 1) return 0;
    return (size_t)kv_heads * pl.n_row_blocks * pl.XS * pl.partial_bytes_per_wg;
}

namespace {

// Everything of a launch's parameters that follows from the arguments and the plan (no workspace).
la_status build_params(AttnParams& prm, const Overrides& ov, const Plan& pl, const void* q, const void* k_cache, const void* v_cache,
                       long long capacity, const int* block_table, int page_size, int n_pages, const int* row_ids,
                       int T, const void* step_k, const void* step_v, int P, int W, int N, int G, int heads,
                       int kv_heads, int head_dim, void* out)
{
    const int group = heads / kv_heads;
    prm.q = (const __bf16*)q;
    prm.k_cache = (const __bf16*)k_cache;
    prm.v_cache = (const __bf16*)v_cache;
    prm.step_k = (const __bf16*)step_k;
    prm.step_v = (const __bf16*)step_v;
    prm.out = (__bf16*)out;
    prm.rope_rows = prm.rope_block = prm.rope_flags = 0;
    prm.partials = nullptr;
    prm.tickets = nullptr;
    prm.P = P; prm.W = W; prm.N = N; prm.G = G; prm.T = T;
    if (block_table && (pl.n_prefix_chunks >= (1 << 21) || page_size % pl.KC != 0))
        return fail(LA_EUNSUPPORTED, "la_step_attention_paged: prefix of %d keys / page of %d not supported", P, page_size);
    prm.cache_rows = block_table ? page_size : capacity;
    prm.block_table = block_table;
    prm.row_ids = row_ids;
    prm.page_bytes = (long long)kv_heads * page_size * head_dim * 2;
    prm.page_chunks = block_table ? page_size / pl.KC : 1;
    prm.n_pages = n_pages;
    prm.table_last = block_table ? (P + page_size - 1) / page_size - 1 : 0;
    if (prm.table_last < 0) prm.table_last = 0;
    prm.inv_page_chunks = 1.0f / (float)prm.page_chunks;
    prm.heads = heads; prm.kv_heads = kv_heads; prm.group = group;
    prm.R = T * group;
    prm.n_prefix_chunks = pl.n_prefix_chunks;
    prm.n_chunks = pl.n_chunks;
    prm.n_row_blocks = pl.n_row_blocks;
    prm.XS = pl.XS;
    const long long total = (long long)kv_heads * pl.n_row_blocks * pl.XS;
    if (total >= (1 << 21)) return fail(LA_EUNSUPPORTED, "la_step_attention: too many workgroups");
    prm.total_wg = (int)total;
    prm.wg_per_xcd = (int)((total + 7) / 8);
    prm.scale_log2 = 1.4426950408889634f / sqrtf((float)head_dim);
    prm.inv_XS = 1.0f / (float)pl.XS;
    prm.inv_row_blocks = 1.0f / (float)pl.n_row_blocks;
    prm.inv_group = 1.0f / (float)group;
    prm.inv_W = 1.0f / (float)(W > 0 ? W : 1);
    prm.inv_n1 = 1.0f / (float)(N - 1);
    prm.chunks_lo = pl.n_chunks / pl.XS;
    prm.chunks_rem = pl.n_chunks % pl.XS;
    // Chunks requested before the loop: the first iteration's and one more.  Requesting every
    // stage up front delays the first chunk (each request costs issue time); fewer leave the
    // second iteration waiting.
    const int kb = pl.KC / 32, cpi = pl.KS > kb ? pl.KS / kb : 1;  // chunks per iteration
    prm.pre = (pl.PRE >= cpi && pl.PRE <= pl.NS) ? pl.PRE : (cpi + 1 < pl.NS ? cpi + 1 : pl.NS);
    // Long walks with one chunk per iteration (the 128-row plan): the start-up cost is amortised
    // and a full ring keeps three chunks in flight instead of two (measured 6-8 % at 50 chunks
    // per workgroup, a loss at 8).
    if (pl.PRE == 0 && cpi == 1 && prm.chunks_lo >= 16) prm.pre = pl.NS;
    // Short walks with two chunks per iteration (the 7B configuration: 4 or 5 chunks per workgroup):
    // only the first iteration's chunks up front.  Every request that stands in front of them
    // delays the first MFMA of every workgroup on the chip, and with so few iterations nothing
    // amortises that (11.8 against 12.1 us in alternating runs; no difference from 11 chunks on).
    if (pl.PRE == 0 && cpi == 2 && prm.chunks_lo <= 6) prm.pre = cpi;
    // testing hook: exercise the path taken when a split group is not on one XCD
    prm.force_recompute = ov.force_recompute ? 1 : 0;
    return LA_OK;
}

}  // namespace

namespace {

// Which of the two kernels a plain step (packed or in-place bf16 cache, whole step) takes.  The
// row-tile kernel, measured against the staged one: ahead (10 to 28 %) while the keys fit a dozen
// chunks and its workgroups one round of the compute units, behind beyond either.
bool picks_rowtile(const Overrides& ov, int P, int T, int group, int kv_heads, int head_dim)
{
    if (ov.has_plan || !rowtile_supported(head_dim, group, T)) return false;
    if (ov.rowtile >= 0) return ov.rowtile == 1;
    const int tiles = (T * group + 31) / 32;
    const int n_chunks = (P + 63) / 64 + (T + 63) / 64;
    return n_chunks <= 12 && (long long)kv_heads * tiles * 2 <= 256;
}

}  // namespace

int step_attention_kernel_choice(int P, int W, int N, int G, int heads, int kv_heads, int head_dim)
{
    const int T = 1 + (W + G) * (N - 1);
    return picks_rowtile(current_overrides(), P, T, heads / kv_heads, kv_heads, head_dim) ? 1 : 0;
}

la_status launch_step_attention(const void* q, const void* k_cache, const void* v_cache,
                                long long capacity, const int* block_table, int page_size, int n_pages,
                                const int* row_ids, int n_rows, const void* step_k, const void* step_v, int P,
                                int W, int N, int G, int heads, int kv_heads, int head_dim, void* out,
                                hipStream_t stream, const FixedWorkspace* fixed, const float* k_scale,
                                const float* v_scale, const RopeTables* rope)
{
    const int T = row_ids ? n_rows : 1 + (W + G) * (N - 1);
    const int group = heads / kv_heads;
    if ((long long)T * group >= (1 << 21) || (long long)T * heads * head_dim * 2 >= (1ll << 31) ||
        (long long)kv_heads * head_dim * 2 >= (1 << 24))
        return fail(LA_EUNSUPPORTED, "la_step_attention: step too large (T=%d, heads=%d)", T, heads);
    const Overrides ov = current_overrides();
    if (!block_table && !row_ids && !k_scale && picks_rowtile(ov, P, T, group, kv_heads, head_dim)) {
        // (the rotating form of the row-tile kernel stages fewer positions than the staged kernel's:
        // a wider step stays with the staged kernel)
        const int far = W > 0 ? (W + N - 2 > N - 1 ? W + N - 2 : N - 1) : (G > 0 ? N - 1 : 0);
        if (!rope || far + 1 <= rowtile_rope_positions())
            return launch_step_attention_rowtile(q, k_cache, v_cache, capacity, step_k, step_v, P, W, N, G, heads,
                                                 kv_heads, out, stream, rope);
    }
    const Plan pl = make_plan(ov, P, T, group, kv_heads, head_dim, block_table != nullptr, row_ids != nullptr,
                              rope != nullptr);
    AttnParams prm;
    const la_status st = build_params(prm, ov, pl, q, k_cache, v_cache, capacity, block_table, page_size, n_pages, row_ids,
                                      T, step_k, step_v, P, W, N, G, heads, kv_heads, head_dim, out);
    if (st != LA_OK) return st;
    const long long total = prm.total_wg;
    const bool quantised = k_scale != nullptr;
    if (quantised) {
        // 8-bit keys and values: rows of head_dim bytes (cache_rows counts rows, so it stands)
        const bool compiled = pl.KC == 64 && pl.NS == 4 &&
                              (head_dim == 128 ? ((pl.RT == 2 && pl.KS == 4) || (pl.RT == 4 && pl.KS == 2) ||
                                                  (pl.RT == 1 && pl.KS == 2) || (pl.RT == 2 && pl.KS == 2))
                                               : ((pl.RT == 1 && pl.KS == 2) || (pl.RT == 2 && pl.KS == 2)));
        if (block_table || row_ids || !compiled)
            return fail(LA_EUNSUPPORTED, "la_step_attention_fp8kv: no kernel for head_dim=%d plan (%d,%d,%d,%d)",
                        head_dim, pl.RT, pl.KS, pl.NS, pl.KC);
        prm.k_scale = k_scale;  // (in place of the block table and the row ids, which this variant does not have)
        prm.v_scale = v_scale;
    }

    if (pl.XS > 1) {
        const size_t ticket_bytes = (size_t)kv_heads * pl.n_row_blocks * pl.RT * pl.KS * sizeof(unsigned) * kTicketStride;
        const size_t bytes = (size_t)total * pl.partial_bytes_per_wg;
        if (fixed) {
            // a caller that cannot allocate: the blocks are given and cannot grow
            if (ticket_bytes > fixed->ticket_bytes || bytes > fixed->partial_bytes)
                return fail(LA_EUNSUPPORTED,
                            "la_step_attention_noalloc: the step needs %zu + %zu bytes of scratch memory, the fixed "
                            "block holds %zu + %zu", ticket_bytes, bytes, fixed->ticket_bytes, fixed->partial_bytes);
            prm.tickets = (unsigned*)fixed->tickets;
            prm.partials = fixed->partials;
            // the block is shared by every call on this device and keeps what the last one left:
            // the tickets must start at zero (a fill kernel, not a memset, so that the call can
            // be recorded into a graph)
            const int n_words = (int)(ticket_bytes / sizeof(unsigned));
            hipLaunchKernelGGL(clear_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, stream, prm.tickets, n_words);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return fail(LA_EHIP, "la_step_attention_noalloc: clearing the tickets: %s", hipGetErrorString(e));
        } else {
            prm.tickets = (unsigned*)zeroed_workspace(ticket_bytes, stream);
            if (!prm.tickets) return last_failure();
            prm.partials = scratch_workspace(bytes, stream);
            if (!prm.partials) return last_failure();
        }
    }

    if (row_ids) {
        if (block_table || n_rows > 1024 || !rowset_plan_supported(head_dim, pl.RT, pl.KS, pl.NS, pl.KC))
            return fail(LA_EUNSUPPORTED, "la_step_attention_rows: no kernel for head_dim=%d plan (%d,%d,%d), %d rows",
                        head_dim, pl.RT, pl.KS, pl.NS, n_rows);
        if (head_dim == 128) {
            if (pl.KS == 4) return launch_cfg<128, 2, 4, 4, 64, false, true>(prm, stream);
            if (pl.RT == 1) return launch_cfg<128, 1, 2, 4, 64, false, true>(prm, stream);
            return launch_cfg<128, 2, 2, 4, 64, false, true>(prm, stream);
        }
        if (pl.RT == 1) return launch_cfg<64, 1, 2, 4, 64, false, true>(prm, stream);
        return launch_cfg<64, 2, 2, 4, 64, false, true>(prm, stream);
    }
    if (block_table) {
        if (!paged_plan_supported(head_dim, pl.RT, pl.KS, pl.NS, pl.KC))
            return fail(LA_EUNSUPPORTED, "la_step_attention_paged: no kernel for head_dim=%d plan (%d,%d,%d)",
                        head_dim, pl.RT, pl.KS, pl.NS);
        if (head_dim == 128) {
            if (pl.KS == 4) return launch_cfg<128, 2, 4, 4, 64, true>(prm, stream);
            if (pl.RT == 4) return launch_cfg<128, 4, 2, 4, 64, true>(prm, stream);
            if (pl.RT == 1) return launch_cfg<128, 1, 2, 4, 64, true>(prm, stream);
            return launch_cfg<128, 2, 2, 4, 64, true>(prm, stream);
        }
        if (pl.RT == 1) return launch_cfg<64, 1, 2, 4, 64, true>(prm, stream);
        return launch_cfg<64, 2, 2, 4, 64, true>(prm, stream);
    }
    if (rope) {
        // the furthest position of the step: the newest window level's last column, or a candidate's last token
        const int far = W > 0 ? (W + N - 2 > N - 1 ? W + N - 2 : N - 1) : (G > 0 ? N - 1 : 0);
        prm.rope_rows = far + 1;
        prm.rope_block = (prm.rope_rows * head_dim * 2 + 1023) / 1024 * 1024;
        prm.rope_flags = (rope->interleaved ? 1 : 0) | (rope->rotate_keys ? 2 : 0);
        const bool compiled = pl.KC == 64 && pl.NS == 4 &&
                              (head_dim == 128 ? ((pl.RT == 2 && pl.KS == 4) || (pl.RT == 1 && pl.KS == 2) ||
                                                  (pl.RT == 2 && pl.KS == 2))
                                               : ((pl.RT == 1 && pl.KS == 2) || (pl.RT == 2 && pl.KS == 2)));
        if (block_table || row_ids || quantised || !compiled)
            return fail(LA_EUNSUPPORTED, "la_step_attention_rope: no kernel for head_dim=%d plan (%d,%d,%d,%d)",
                        head_dim, pl.RT, pl.KS, pl.NS, pl.KC);
        prm.rope_cos = rope->cos + (size_t)P * (head_dim / 2);
        prm.rope_sin = rope->sin + (size_t)P * (head_dim / 2);
        if (head_dim == 128) {
            if (pl.KS == 4) return launch_cfg<128, 2, 4, 4, 64, false, false, 2, true>(prm, stream);
            if (pl.RT == 1) return launch_cfg<128, 1, 2, 4, 64, false, false, 2, true>(prm, stream);
            return launch_cfg<128, 2, 2, 4, 64, false, false, 2, true>(prm, stream);
        }
        if (pl.RT == 1) return launch_cfg<64, 1, 2, 4, 64, false, false, 2, true>(prm, stream);
        return launch_cfg<64, 2, 2, 4, 64, false, false, 2, true>(prm, stream);
    }
    if (quantised) {
        if (head_dim == 128) {
            if (pl.KS == 4) return launch_cfg<128, 2, 4, 4, 64, false, false, 1>(prm, stream);
            if (pl.RT == 4) return launch_cfg<128, 4, 2, 4, 64, false, false, 1>(prm, stream);
            if (pl.RT == 1) return launch_cfg<128, 1, 2, 4, 64, false, false, 1>(prm, stream);
            return launch_cfg<128, 2, 2, 4, 64, false, false, 1>(prm, stream);
        }
        if (pl.RT == 1) return launch_cfg<64, 1, 2, 4, 64, false, false, 1>(prm, stream);
        return launch_cfg<64, 2, 2, 4, 64, false, false, 1>(prm, stream);
    }
    if (pl.KC == 32) return launch_cfg<128, 2, 2, 9, 32>(prm, stream);
    if (pl.KS == 4) return launch_cfg<128, 2, 4, 4>(prm, stream);
    if (pl.RT == 4 && pl.KS == 2) return launch_cfg<128, 4, 2, 4>(prm, stream);
#define LA_DISPATCH(D_, RT_, KS_, NSMAX_)                                        \
    if (head_dim == D_ && pl.RT == RT_ && pl.KS == KS_) {                       \
        if (pl.NS == 2) return launch_cfg<D_, RT_, KS_, 2>(prm, stream);        \
        return launch_cfg<D_, RT_, KS_, NSMAX_>(prm, stream);                   \
    }
    LA_DISPATCH(128, 1, 2, 4)
    LA_DISPATCH(128, 2, 2, 4)
    LA_DISPATCH(128, 2, 1, 4)
    LA_DISPATCH(128, 4, 1, 3)
    LA_DISPATCH(64, 1, 2, 4)
    LA_DISPATCH(64, 2, 2, 4)
    LA_DISPATCH(64, 4, 1, 4)
#undef LA_DISPATCH
    return fail(LA_EUNSUPPORTED, "la_step_attention: no kernel for head_dim=%d plan (%d,%d)",
                head_dim, pl.RT, pl.KS);
}

// ---- several steps in one launch

namespace {

template <int D, int RT, int KS, int NSTAGE, bool PAGED = false>
la_status launch_batch_cfg(const BatchParams& bp, unsigned grid, hipStream_t stream)
{
    using C = Cfg<D, RT, KS, 64, NSTAGE>;
    auto kern = step_attention_batch_kernel<D, RT, KS, 64, NSTAGE, PAGED>;
    static bool attr_set[16] = {false};
    const la_status st = set_lds_attribute_once(reinterpret_cast<const void*>(kern), C::LDS_BYTES, attr_set);
    if (st != LA_OK) return st;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS_BYTES, stream, bp);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_step_attention_batch launch: %s", hipGetErrorString(e));
    return LA_OK;
}

}  // namespace

static_assert(sizeof(BatchParams) <= 4000, "the batch travels as a kernel argument");

la_status launch_step_attention_batch(const BatchSeq* seqs, int n_seqs, int page_size, int n_pages, int W, int N,
                                      int G, int heads, int kv_heads, int head_dim, hipStream_t stream)
{
    const bool paged = page_size > 0;
    const int T = 1 + (W + G) * (N - 1);
    const int group = heads / kv_heads;
    if ((long long)T * group >= (1 << 21) || (long long)T * heads * head_dim * 2 >= (1ll << 31) ||
        (long long)kv_heads * head_dim * 2 >= (1 << 24))
        return fail(LA_EUNSUPPORTED, "la_step_attention_batch: step too large (T=%d, heads=%d)", T, heads);
    const Overrides ov = current_overrides();
    // longest first: workgroups are handed out in id order
    int order[1024];
    if (n_seqs > 1024) return fail(LA_EUNSUPPORTED, "la_step_attention_batch: at most 1024 steps per call");
    for (int i = 0; i < n_seqs; ++i) order[i] = i;
    for (int i = 1; i < n_seqs; ++i)
        for (int j = i; j > 0 && seqs[order[j]].P > seqs[order[j - 1]].P; --j) {
            const int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t;
        }
    for (int first = 0; first < n_seqs; first += kMaxBatch) {
        const int n = n_seqs - first < kMaxBatch ? n_seqs - first : kMaxBatch;
        if (n == 1) {  // nothing to share a launch with: the one-step path and its own decomposition
            const BatchSeq& d = seqs[order[first]];
            const la_status st = launch_step_attention(d.q, d.k_cache, d.v_cache, d.P, d.P > 0 ? d.block_table : nullptr,
                                                       page_size, n_pages, nullptr, 0, d.step_k, d.step_v, d.P, W, N, G,
                                                       heads, kv_heads, head_dim, d.out, stream);
            if (st != LA_OK) return st;
            continue;
        }
        // One decomposition (row tiles, key-split waves) for the whole launch; the key ranges are
        // cut so that every workgroup gets about the same number of chunks, with enough
        // workgroups for two rounds over the 256 compute units.
        Plan pl[kMaxBatch];
        for (int i = 0; i < n; ++i) pl[i] = make_plan(Overrides(), seqs[order[first + i]].P, T, group, kv_heads, head_dim);
        long long work = 0;
        // 128-row workgroups (a chunk of K/V staged once for four row tiles: half the traffic into
        // LDS per flop) as soon as the batch fills three quarters of the GPU with them; otherwise
        // 64-row workgroups, twice as many.  (Measured: eight 7B-shaped steps 33 vs 40 us.)
        int RT = 2, KS = 4;
        if (head_dim == 128) {
            const int tiles = (T * group + 31) / 32;
            const long long units128 = (long long)n * kv_heads * ((tiles + 3) / 4);
            if (tiles >= 3 && units128 >= 192) { RT = 4; KS = 2; }
        } else {
            KS = 2;
        }
        if (head_dim == 128 && ov.batch_rows == 4) { RT = 4; KS = 2; }  // testing hook
        if (head_dim == 128 && ov.batch_rows == 2) { RT = 2; KS = 4; }
        const int rows_wg = RT * 32;
        const int n_row_blocks = (T * group + rows_wg - 1) / rows_wg;
        for (int i = 0; i < n; ++i) work += (long long)kv_heads * n_row_blocks * pl[i].n_chunks;
        // One round of workgroups when the steps are alike (a second round only waits for the
        // first); half a round more when their lengths differ, to even out the ends (measured).
        bool alike = true;
        for (int i = 1; i < n; ++i) alike = alike && pl[i].n_chunks == pl[0].n_chunks;
        const long long wgs = alike ? 256 : 384;
        long long target = (work + wgs - 1) / wgs;   // chunks per workgroup
        if (target < 4) target = 4;
        BatchParams bp;
        bp.slots.n = n;
        size_t partial_bytes = 0, ticket_count = 0;
        int slot = 0;
        for (int i = 0; i < n; ++i) {
            const BatchSeq& d = seqs[order[first + i]];
            Plan& q = pl[i];
            q.RT = RT; q.KS = KS; q.NS = 4; q.KC = 64; q.PRE = 0;
            q.n_row_blocks = n_row_blocks;
            q.partial_bytes_per_wg = partial_wg_bytes(head_dim, RT, KS);
            int xs = (int)((q.n_chunks + target - 1) / target);
            if (xs > q.n_chunks / 2) xs = q.n_chunks / 2;
            if (xs > 64) xs = 64;
            q.XS = xs < 1 ? 1 : xs;
            const la_status st = build_params(bp.seq[i], ov, q, d.q, d.k_cache, d.v_cache, d.P,
                                              d.P > 0 ? d.block_table : nullptr, page_size, n_pages, nullptr, T,
                                              d.step_k, d.step_v, d.P, W, N, G, heads, kv_heads, head_dim, d.out);
            if (st != LA_OK) return st;
            bp.slots.slot0[i] = slot;
            slot += bp.seq[i].wg_per_xcd;
            if (q.XS > 1) {
                partial_bytes += (size_t)bp.seq[i].total_wg * q.partial_bytes_per_wg;
                ticket_count += (size_t)kv_heads * n_row_blocks * RT * KS * kTicketStride;
            }
        }
        for (int i = n; i <= kMaxBatch; ++i) bp.slots.slot0[i] = slot;
        if (partial_bytes) {
            unsigned* tickets = (unsigned*)zeroed_workspace(ticket_count * sizeof(unsigned), stream);
            unsigned char* partials = (unsigned char*)scratch_workspace(partial_bytes, stream);
            if (!tickets || !partials) return last_failure();
            for (int i = 0; i < n; ++i) {
                if (pl[i].XS <= 1) continue;
                bp.seq[i].tickets = tickets;
                bp.seq[i].partials = partials;
                tickets += (size_t)kv_heads * n_row_blocks * RT * KS * kTicketStride;
                partials += (size_t)bp.seq[i].total_wg * pl[i].partial_bytes_per_wg;
            }
        }
        const unsigned grid = (unsigned)slot * 8u;
        la_status st;
        if (paged) {
            if (head_dim == 128 && RT == 4) st = launch_batch_cfg<128, 4, 2, 4, true>(bp, grid, stream);
            else if (head_dim == 128) st = launch_batch_cfg<128, 2, 4, 4, true>(bp, grid, stream);
            else st = launch_batch_cfg<64, 2, 2, 4, true>(bp, grid, stream);
        } else if (head_dim == 128 && RT == 4) st = launch_batch_cfg<128, 4, 2, 4>(bp, grid, stream);
        else if (head_dim == 128) st = launch_batch_cfg<128, 2, 4, 4>(bp, grid, stream);
        else st = launch_batch_cfg<64, 2, 2, 4>(bp, grid, stream);
        if (st != LA_OK) return st;
    }
    return LA_OK;
}

// ---- testing hooks

la_status set_override(const char* key, const char* value)
{
    if (!key) return fail(LA_EINVAL, "la_debug_override: null key");
    const std::string k = key;
    std::lock_guard<std::mutex> lock(g_config_mutex);
    overrides_from_env_locked();
    if (k == "attn_plan") {
        if (!parse_plan(value, g_overrides) && value && value[0])
            return fail(LA_EINVAL, "la_debug_override: attn_plan wants \"RT,KS,XS,NS,KC[,PRE]\", got \"%s\"", value);
    } else if (k == "batch_plan") {
        g_overrides.batch_rows = (value && (value[0] == '2' || value[0] == '4')) ? value[0] - '0' : 0;
    } else if (k == "attn_rowtile") {
        g_overrides.rowtile = (value && (value[0] == '0' || value[0] == '1')) ? value[0] - '0' : -1;
    } else if (k == "force_recompute") {
        g_overrides.force_recompute = value && value[0] == '1';
    } else {
        return fail(LA_EINVAL, "la_debug_override: unknown key \"%s\"", key);
    }
    return LA_OK;
}

// ---- the fixed scratch block of la_step_attention_noalloc

la_status fixed_workspace(FixedWorkspace* ws)
{
    static std::mutex mutex;
    static unsigned char* base[16] = {nullptr};  // device address of `scratch`, per device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return fail(LA_EHIP, "hipGetDevice failed");
    std::lock_guard<std::mutex> lock(mutex);
    if (!base[dev]) {
        // each device has its own copy of the array at its own address; `dev` is current here
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(LA_EHIP, "la_step_attention_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
        base[dev] = (unsigned char*)ptr;
    }
    ws->tickets = base[dev];
    ws->ticket_bytes = kFixedTicketBytes;
    ws->partials = base[dev] + kFixedTicketBytes;
    ws->partial_bytes = kFixedPartialBytes;
    return LA_OK;
}

}  // namespace la

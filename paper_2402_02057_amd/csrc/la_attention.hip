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
// Decomposition.  A workgroup owns (KV head, block of RT*RW 32-row tiles, one of XS ranges of
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
// Split combine, in the same launch.  With XS > 1 each workgroup stores its unnormalised fp32
// accumulator and (max, sum) per row, waits for the stores to reach the L2, and takes a
// ticket; the workgroup that arrives last merges all XS partials in index order (so results
// do not depend on arrival order), normalises and writes bf16.  The L2 of one XCD is
// coherent for all its compute units, but the eight L2s are not coherent with each other
// inside a kernel, and an agent-scope fence (L2 write-back + invalidate) costs tens of
// microseconds here.  So the workgroups of a split group are laid out on one XCD (workgroup
// ids go round-robin over XCDs) and the ticket also carries the XCD id each member read
// from the hardware register: if all ids agree the partials are read straight from the shared
// L2; if not, the last workgroup ignores the partials and recomputes its rows over all
// chunks from the read-only inputs.  Either way the result is exact; tickets return to zero,
// so no memset is needed between calls.
#include <stdlib.h>

#include "la_internal.h"

namespace la {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr float kNegInf = -__builtin_huge_valf();

struct AttnParams {
    const __bf16* q;
    const __bf16* k_cache;
    const __bf16* v_cache;
    const __bf16* step_k;
    const __bf16* step_v;
    __bf16* out;
    void* partials;     // XS > 1: per workgroup, fragment-layout bf16 accumulators and fp32 (m, l)
    unsigned* tickets;  // XS > 1: one counter per (KV head, row block), zero between calls
    int P, W, N, G, T;
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
    int force_recompute;  // testing: treat every group as spread over several XCDs
#ifdef LA_DEV_KNOBS
    int dev_mode;         // timing experiments only (results are wrong): see LA_DEV_MODE
    long long* dev_trace; // 8 wall-clock stamps per workgroup
#endif
};

// Which step keys a step row may see, as index ranges (see the header comment).
struct RowVis {
    int t;      // step index of the row
    int e0;     // keys 0..e0 are visible
    int s1;     // keys t, t-s1, t-2*s1, ... (cnt of them) are visible
    int cnt;
};

// floor(a / d) for 0 <= a < 2^21 given inv = 1.0f / d: (a + 0.5) / d is at least 0.5 / d away
// from an integer, more than the rounding error of the two float operations.
__device__ __forceinline__ int div_small(int a, float inv)
{
    return (int)(((float)a + 0.5f) * inv);
}

__device__ __forceinline__ RowVis row_visibility(int t, int W, int N, float inv_W, float inv_n1)
{
    RowVis v;
    v.t = t;
    const int n_look = W * (N - 1);
    if (t == 0) {
        v.e0 = 0; v.s1 = 1; v.cnt = 1;
    } else if (t <= n_look) {
        const int x = t - 1;
        const int l = div_small(x, inv_W), j = x - l * W;
        v.e0 = 1 + j; v.s1 = W; v.cnt = l + 1;
    } else {
        const int x = t - 1 - n_look;
        const int k = x - div_small(x, inv_n1) * (N - 1);
        v.e0 = 0; v.s1 = 1; v.cnt = k + 1;
    }
    return v;
}

// Bit b set iff step key (key0 + b) is visible to the row.
__device__ __forceinline__ unsigned step_block_word(const RowVis& v, int key0)
{
    unsigned w = 0;
    const int n0 = v.e0 - key0 + 1;  // keys key0 .. e0
    if (n0 > 0) w = n0 >= 32 ? 0xFFFFFFFFu : ((1u << n0) - 1u);
    int c = v.t;
    for (int k = 0; k < v.cnt; ++k, c -= v.s1) {
        const unsigned d = (unsigned)(c - key0);
        if (d < 32u) w |= 1u << d;
    }
    return w;
}

// Three-way maximum in one instruction; unlike fmaxf the compiler adds no NaN-quieting moves
// around it (scores are MFMA results or -inf, never signalling NaNs).
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// max of a value with the one held by the lane 32 away (the other 16 keys of the same row).
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of its
// second: fed the same value twice it returns (lower half everywhere, upper half everywhere).
__device__ __forceinline__ float max_across_halves(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most `later` * LPW of this wave's loads are still in flight (later < NS).
template <int LPW, int NS>
__device__ __forceinline__ void wait_chunks(int later)
{
    static_assert(LPW * (NS - 1) < 64, "vmcnt is a 6-bit counter");
    switch (later) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<(NS > 1 ? 1 : 0) * LPW>(); break;
    case 2: wait_vmcnt<(NS > 2 ? 2 : 0) * LPW>(); break;
    case 3: wait_vmcnt<(NS > 3 ? 3 : 0) * LPW>(); break;
    case 4: wait_vmcnt<(NS > 4 ? 4 : 0) * LPW>(); break;
    case 5: wait_vmcnt<(NS > 5 ? 5 : 0) * LPW>(); break;
    case 6: wait_vmcnt<(NS > 6 ? 6 : 0) * LPW>(); break;
    case 7: wait_vmcnt<(NS > 7 ? 7 : 0) * LPW>(); break;
    default: wait_vmcnt<(NS > 8 ? 8 : 0) * LPW>(); break;
    }
}

// One direct-to-LDS load: every lane fetches 16 bytes from its own global address, the wave's
// 1 KB lands at LDS byte address `lds_base` + lane * 16 (M0 carries the base).  Written as
// assembly so that the compiler's wait-count bookkeeping does not know of these loads: it would
// otherwise make every later LDS read wait for ALL of them, including the chunks being
// prefetched.  Completion is tracked by hand: s_waitcnt vmcnt(n) + workgroup barrier.
// The address is a wave-uniform 64-bit base in scalar registers plus a 32-bit per-lane byte
// offset: no 64-bit vector arithmetic per load.
__device__ __forceinline__ void dma16_base(const void* base, unsigned lane_off, unsigned lds_base)
{
    // the base is the same in every lane; say so, or the operand may be given vector registers
    const unsigned long long b = reinterpret_cast<unsigned long long>(base);
    const unsigned long long lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    const unsigned long long hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off), "s"((hi << 32) | lo), "s"(lds_base)
                 : "memory");
}

__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}

// 16-byte piece `lc` of row `row` lives at piece position lc ^ swizzle(row) of that row.
template <int D>
__device__ __forceinline__ int swizzle(int row)
{
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    return (row >> 1) & 7;
}

template <int D, int RW, int RT, int KS, int KC, int NSTAGE>
struct Cfg {
    static constexpr int NW = RT * KS;
    static constexpr int NT = NW * 64;
    static constexpr int RBYTES = D * 2;
    static constexpr int NCH = D / 8;                     // 16-byte pieces per row
    static constexpr int KB = KC / 32;                    // 32-key blocks per chunk
    // Key-split waves of a row tile: up to KB of them share a chunk (one or more blocks each);
    // beyond that, groups of KB waves take consecutive chunks of the same iteration.
    static constexpr int CPI = KS > KB ? KS / KB : 1;     // chunks consumed per iteration
    static constexpr int KBW = KS >= KB ? 1 : KB / KS;    // blocks per wave per chunk
    static constexpr int KV_BYTES = KC * RBYTES;          // one of K or V of a chunk
    static constexpr int STAGE_BYTES = 2 * KV_BYTES;
    static constexpr int WLOADS = STAGE_BYTES / 1024;     // 64-lane x 16-byte loads per chunk
    static constexpr int LPW = WLOADS / NW;               // loads per wave per chunk
    static constexpr int TILES = RT * RW;                 // 32-row tiles per workgroup
    static constexpr int ROWS = TILES * 32;
    static constexpr int DB = D / 32;                     // 32-wide blocks of head_dim
    static constexpr int FRAG_FLOATS = DB * 16 * 64;      // one tile's accumulators
    static constexpr int TILE_FLOATS = FRAG_FLOATS + 128; // + m and l per lane
    // a split's partial in global memory: per tile the accumulators as bf16 in fragment order
    // ([8 values][lane], 16 bytes per lane and access) followed by (m, l) per lane in fp32
    static constexpr int PART_ACC_BYTES = DB * 16 * 64 * 2;
    static constexpr int PART_TILE_BYTES = PART_ACC_BYTES + 64 * 8;
    static constexpr int PART_WG_BYTES = TILES * PART_TILE_BYTES;
    static constexpr int OUT_PITCH = RBYTES + 16;         // LDS pitch of the output transpose
    static constexpr int Q_BYTES = ROWS * RBYTES;         // the workgroup's query rows
    static constexpr int Q_OFFSET = NSTAGE * STAGE_BYTES; // they sit behind the stage ring
    static constexpr int QLPW = Q_BYTES / 1024 / NW;      // Q loads per wave
    static constexpr int LDS_MAIN = NSTAGE * STAGE_BYTES + Q_BYTES;
    static constexpr int LDS_MERGE = (KS / 2) * RT * RW * TILE_FLOATS * 4;
    static constexpr int LDS_OUT = ROWS * OUT_PITCH;
    static constexpr int LDS_BYTES =
        LDS_MAIN > LDS_MERGE ? (LDS_MAIN > LDS_OUT ? LDS_MAIN : LDS_OUT)
                             : (LDS_MERGE > LDS_OUT ? LDS_MERGE : LDS_OUT);
    static_assert(KS >= KB ? KS % KB == 0 : KB % KS == 0, "key-split waves and blocks must divide");
    static_assert(NSTAGE >= CPI, "an iteration's chunks must fit the ring");
    static_assert(WLOADS % NW == 0, "chunk loads must divide among the waves");
    static_assert((Q_BYTES / 1024) % NW == 0, "Q loads must divide among the waves");
    static_assert(NSTAGE <= 9, "wait_chunks covers up to 8 younger chunks");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of a compute unit");
};

#ifdef LA_DEV_KNOBS
#define LA_STAMP(k) do { if (p.dev_trace && (threadIdx.x & 63) == 0) p.dev_trace[((size_t)blockIdx.x * 8 + (threadIdx.x >> 6)) * 24 + (k)] = wall_clock64(); } while (0)
#define LA_CYC(k) do { if (p.dev_trace && (threadIdx.x & 63) == 0 && it == 1) p.dev_trace[((size_t)(4096 + blockIdx.x) * 8 + (threadIdx.x >> 6)) * 24 + (k)] = __builtin_readcyclecounter(); } while (0)
#else
#define LA_STAMP(k) do { } while (0)
#define LA_CYC(k) do { } while (0)
#endif

// Id of the XCD (accelerator die, with its own L2) this wave runs on.
__device__ __forceinline__ unsigned xcc_id()
{
    unsigned v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return v & 0xfu;
}

// Copy the workgroup's finished rows (bf16, pitch C::OUT_PITCH in LDS) to `out`, 16 bytes a lane.
template <class C, int D = C::RBYTES / 2>
__device__ __forceinline__ void write_rows_from_lds(const AttnParams& p, const unsigned char* lds,
                                                    int rb, int kvh, int tid)
{
    const int rows_here = min(C::ROWS, p.R - rb * C::ROWS);
    for (int piece = tid; piece < rows_here * C::NCH; piece += C::NT) {
        const int r = piece / C::NCH, ch = piece % C::NCH;
        const int rr = rb * C::ROWS + r;
        const int t = div_small(rr, p.inv_group), hh = rr - t * p.group;
        const f32x4 v = *reinterpret_cast<const f32x4*>(lds + r * C::OUT_PITCH + ch * 16);
        *reinterpret_cast<f32x4*>(p.out + ((size_t)t * p.heads + (size_t)kvh * p.group + hh) * D + ch * 8) = v;
    }
}

template <int D, int RW, int RT, int KS, int KC, int NSTAGE>
__global__ __launch_bounds__(RT* KS * 64) void step_attention_kernel(const AttnParams p)
{
    using C = Cfg<D, RW, RT, KS, KC, NSTAGE>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // Consecutive workgroup ids go round-robin over the 8 XCDs (each with its own L2); put
    // the workgroups that stream the same KV head on one XCD.
    LA_STAMP(0);
    int logical = (int)(blockIdx.x & 7) * p.wg_per_xcd + (int)(blockIdx.x >> 3);
#ifdef LA_DEV_KNOBS
    if (p.dev_mode >= 16) logical = (int)blockIdx.x;  // experiment: no XCD grouping (wrong combine!)
#endif
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
    const int rt = wave / KS;   // row tile group of this wave
    const int ks = wave % KS;   // which key blocks of a chunk it takes
    const int hi = lane >> 5;   // upper half-wave
    const int l32 = lane & 31;

    const unsigned lds_base = lds_address(lds);
    const int row_base = rb * C::ROWS + rt * (RW * 32);  // first row of this wave (in R space)
    const bool wave_active = row_base < p.R;            // else: only helps loading

    // ---- chunk range of this split
    int c_begin = xs * p.chunks_lo + min(xs, p.chunks_rem);
    int c_end = c_begin + p.chunks_lo + (xs < p.chunks_rem ? 1 : 0);
    bool direct = p.XS == 1;  // this pass covers every key of the rows: write `out` directly

    // Per-lane part of a load's address.  A wave-load covers RPW = 64 / NCH consecutive rows of
    // 16-byte pieces; with row = wl*RPW + lane_row the swizzle splits into a lane part and a part that
    // depends only on the (wave-uniform) load index wl, so the byte offset of a lane is
    // lane_off ^ (uni(wl) << 4) and the rest of the address is uniform.
    const int lane_row = lane / C::NCH;
    const int lane_lc0 = (lane % C::NCH) ^ (D == 128 ? (lane_row << 2) : (lane_row >> 1));
    const unsigned lane_off = (unsigned)(lane_row * C::RBYTES + (lane_lc0 << 4));

    // Issue the direct-to-LDS loads of chunk `c` into stage `st`: a wave-uniform 64-bit base
    // plus a 32-bit lane offset per load.
    auto issue_chunk = [&](int c, int st) {
        const bool is_step = c >= p.n_prefix_chunks;
        const int key0 = (is_step ? c - p.n_prefix_chunks : c) * KC;
        const int limit = is_step ? p.T : p.P;
        const int last_row = min(KC, limit - key0) - 1;  // >= 0
        const unsigned stage_lds = lds_base + st * C::STAGE_BYTES;
        // rows of the prefix cache are contiguous; step keys are strided by kv_heads
        const unsigned stride_b = (unsigned)(is_step ? p.kv_heads * C::RBYTES : C::RBYTES);
        const size_t first = is_step ? ((size_t)key0 * p.kv_heads + kvh) * D
                                     : ((size_t)kvh * p.P + key0) * D;
        const unsigned char* kbase = reinterpret_cast<const unsigned char*>((is_step ? p.step_k : p.k_cache) + first);
        const unsigned char* vbase = reinterpret_cast<const unsigned char*>((is_step ? p.step_v : p.v_cache) + first);
        if (!is_step && last_row == KC - 1) {
            // a full chunk of the prefix cache: K and V are contiguous KV_BYTES regions
#pragma unroll
            for (int i = 0; i < C::LPW; ++i) {
                const int wl = wave + i * C::NW;                  // wave-load index in the chunk
                const bool is_v = wl >= C::WLOADS / 2;
                const int wl2 = is_v ? wl - C::WLOADS / 2 : wl;   // index within K or V
                const unsigned uni = D == 128 ? (unsigned)(wl2 & 3) : (unsigned)((wl2 & 1) << 2);
                dma16_base((is_v ? vbase : kbase) + wl2 * 1024, lane_off ^ (uni << 4),
                           __builtin_amdgcn_readfirstlane(stage_lds + wl * 1024));
            }
        } else {
            // ragged end or strided step keys: rows past the end repeat the last one
            // (the host checks that the row stride is below 2^24 bytes)
#pragma unroll
            for (int i = 0; i < C::LPW; ++i) {
                const int wl = wave + i * C::NW;
                const bool is_v = wl >= C::WLOADS / 2;
                const int wl2 = is_v ? wl - C::WLOADS / 2 : wl;
                const unsigned uni = D == 128 ? (unsigned)(wl2 & 3) : (unsigned)((wl2 & 1) << 2);
                const int srow = min(wl2 * (64 / C::NCH) + lane_row, last_row);
                const unsigned off = __umul24((unsigned)srow, stride_b) + (((unsigned)lane_lc0 ^ uni) << 4);
                dma16_base(is_v ? vbase : kbase, off, __builtin_amdgcn_readfirstlane(stage_lds + wl * 1024));
            }
        }
    };

    // Request Q and the first chunks before anything else: the stream from HBM is the critical
    // path.  The workgroup's query rows go to LDS (same swizzle as K) and are the oldest loads
    // in flight, so the first chunk's wait covers them.  Rows past the end repeat the last row.
#ifdef LA_DEV_KNOBS
    if (!(p.dev_mode & 32))
#endif
    {
#pragma unroll
        for (int i = 0; i < C::QLPW; ++i) {
            const int wl = wave + i * C::NW;
            const int piece = wl * 64 + lane;
            const int row = piece / C::NCH, pc = piece % C::NCH;
            const int lc = pc ^ swizzle<D>(row);
            const int rr = min(rb * C::ROWS + row, p.R - 1);
            const int t = div_small(rr, p.inv_group), hh = rr - t * p.group;
            // (the host checks that q spans less than 2^31 bytes)
            const unsigned off = (unsigned)(((t * p.heads + kvh * p.group + hh) * D + lc * 8) * 2);
            dma16_base(p.q, off, __builtin_amdgcn_readfirstlane(lds_base + C::Q_OFFSET + wl * 1024));
        }
    }
#pragma unroll
    for (int s = 0; s < NSTAGE; ++s)
        if (s < c_end - c_begin) issue_chunk(c_begin + s, s);
    LA_STAMP(1);

    // which step keys each of this lane's rows may see
    RowVis vis[RW];
#pragma unroll
    for (int rw = 0; rw < RW; ++rw) {
        const int rr = min(row_base + rw * 32 + l32, p.R - 1);
        vis[rw] = row_visibility(div_small(rr, p.inv_group), p.W, p.N, p.inv_W, p.inv_n1);
    }
    bf16x8 qreg[RW][D / 16];  // B operand of S^T = K Q^T: row l32, d = k16*16 + hi*8 .. +8

    f32x16 o[RW][C::DB];
    float m_run[RW], l_run[RW];
    // after the ticket: 0 not last, 1 last and co-located, 2 recompute.  It lives where the Q rows
    // were (they are in registers by then), so that the stage ring can use every other byte.
    volatile unsigned* s_role = reinterpret_cast<volatile unsigned*>(lds + C::Q_OFFSET);

    for (int pass = 0;; ++pass) {
#pragma unroll
        for (int rw = 0; rw < RW; ++rw) {
            m_run[rw] = kNegInf;
            l_run[rw] = 0.0f;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[rw][db][i] = 0.0f;
        }
        const int n_my = c_end - c_begin;
        if (pass > 0) {
#pragma unroll
            for (int s = 0; s < NSTAGE; ++s)
                if (s < n_my) issue_chunk(c_begin + s, s);
        }

        const int n_iter = (n_my + C::CPI - 1) / C::CPI;
        for (int it = 0; it < n_iter; ++it) {
            // Iteration `it` consumes chunks it*CPI .. it*CPI+CPI-1.  Every stage is requested up
            // front; the stages an iteration frees are refilled at the start of the next one.
            // Wait for this wave's loads of the chunks needed now; younger ones stay in flight.
            const int c_hi = min(n_my, (it + 1) * C::CPI) - 1;
            const int issued = min(n_my, NSTAGE + (it > 0 ? (it - 1) * C::CPI : 0));
            wait_chunks<C::LPW, NSTAGE>(issued - 1 - c_hi);  // 0 .. NSTAGE-1 younger chunks
            LA_CYC(7);
            __syncthreads();  // these chunks are complete in LDS; everyone is done with the last ones
            LA_CYC(6);
            if (it < 8) LA_STAMP(8 + 2 * it);
            if (it == 0 && pass == 0) {
                // Q has landed with the first chunk: move this wave's rows to registers
#pragma unroll
                for (int rw = 0; rw < RW; ++rw) {
                    const int qrow = (rt * RW + rw) * 32 + l32;
                    const unsigned char* qr = lds + C::Q_OFFSET + qrow * C::RBYTES;
                    const int qsw = swizzle<D>(qrow);
#pragma unroll
                    for (int k16 = 0; k16 < D / 16; ++k16)
                        qreg[rw][k16] = *reinterpret_cast<const bf16x8*>(qr + (((k16 * 2 + hi) ^ qsw) << 4));
                }
            }
            if (it >= 1) {
#pragma unroll
                for (int j = 0; j < C::CPI; ++j) {
                    const int cn = (it - 1) * C::CPI + NSTAGE + j;
                    if (cn < n_my) issue_chunk(c_begin + cn, cn % NSTAGE);
                }
            }
            const int cl = it * C::CPI + (KS > C::KB ? ks / C::KB : 0);  // this wave's chunk
            if (cl >= n_my) continue;
            if (!wave_active) continue;
#ifdef LA_DEV_KNOBS
            if ((p.dev_mode & 15) == 2) continue;  // loads only
#endif

            const int c = c_begin + cl;
            const bool is_step = c >= p.n_prefix_chunks;
            const int chunk_key0 = (is_step ? c - p.n_prefix_chunks : c) * KC;
            const int limit = is_step ? p.T : p.P;
            const unsigned char* kst = lds + (cl % NSTAGE) * C::STAGE_BYTES;
            const unsigned char* vst = kst + C::KV_BYTES;

#pragma unroll
            for (int kbw = 0; kbw < C::KBW; ++kbw) {
                const int kb = KS >= C::KB ? ks % C::KB : ks + kbw * KS;
                const int key0 = chunk_key0 + kb * 32;
                if (key0 >= limit) continue;  // block entirely past the end (wave-uniform)

                // ---- operands: all K pieces of the block, and the V pieces of its first 16 keys,
                //      are requested from LDS before the first MFMA (LDS answers in order)
                const int krow = kb * 32 + l32;
                const unsigned char* kr = kst + krow * C::RBYTES;
                const int ksw = swizzle<D>(krow);
                bf16x8 kf[D / 16];
#pragma unroll
                for (int k16 = 0; k16 < D / 16; ++k16)
                    kf[k16] = *reinterpret_cast<const bf16x8*>(kr + (((k16 * 2 + hi) ^ ksw) << 4));
                // V^T operand: k-slot e of half `hi` of 16-key step kk is key
                // kb*32 + kk*16 + (e/4)*8 + hi*4 + e%4 (the layout S^T leaves P in).  A 16-lane
                // block reads 4 keys x 16 columns; the transposing read hands lane n column n.
                const int b16 = lane >> 4, i16 = lane & 15;
                const int jj = i16 >> 2, q4 = i16 & 3;
                bf16x8 vf[2][C::DB];
                auto read_v = [&](int kk) {
                    const int vrow0 = kb * 32 + kk * 16 + hi * 4 + jj;  // e = 0..3
                    const int vrow1 = vrow0 + 8;                        // e = 4..7
                    const int sw0 = swizzle<D>(vrow0), sw1 = swizzle<D>(vrow1);
#pragma unroll
                    for (int db = 0; db < C::DB; ++db) {
                        const int col = db * 32 + (b16 & 1) * 16 + q4 * 4;
                        const int lc = col >> 3, within = (col & 7) * 2;
                        const unsigned char* a0 = vst + vrow0 * C::RBYTES + ((lc ^ sw0) << 4) + within;
                        const unsigned char* a1 = vst + vrow1 * C::RBYTES + ((lc ^ sw1) << 4) + within;
                        union { struct { short4v a, b; } s; bf16x8 v; } u;
                        u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4v __attribute__((address_space(3)))*)a0);
                        u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4v __attribute__((address_space(3)))*)a1);
                        vf[kk][db] = u.v;
                    }
                };
                LA_CYC(0);
                read_v(0);
                __builtin_amdgcn_sched_barrier(0);
                LA_CYC(1);

                // ---- S^T block: 32 keys x 32 rows per tile
                f32x16 s[RW];
#pragma unroll
                for (int rw = 0; rw < RW; ++rw)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[rw][i] = 0.0f;
#pragma unroll
                for (int k16 = 0; k16 < D / 16; ++k16)
#pragma unroll
                    for (int rw = 0; rw < RW; ++rw)
                        s[rw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[k16], qreg[rw][k16], s[rw], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                LA_CYC(2);
                read_v(1);  // in flight during the softmax arithmetic

                // ---- mask, running max, exponentials
                const bool full = !is_step && (key0 + 32 <= limit);  // wave-uniform
                bf16x8 pf[RW][2];
#pragma unroll
                for (int rw = 0; rw < RW; ++rw) {
                    if (!full) {
                        unsigned word;
                        if (is_step) {
                            word = step_block_word(vis[rw], key0);
                        } else {
                            const int n = limit - key0;  // 1..31
                            word = (1u << n) - 1u;
                        }
                        word >>= hi * 4;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int bit = (i >> 2) * 8 + (i & 3);  // hi*4 already shifted out
                            if (!((word >> bit) & 1u)) s[rw][i] = kNegInf;
                        }
                    }
                    float mx = max3(s[rw][0], s[rw][1], s[rw][2]);
#pragma unroll
                    for (int i = 3; i < 15; i += 2) mx = max3(mx, s[rw][i], s[rw][i + 1]);
                    mx = max_across_halves(fmaxf(mx, s[rw][15]));
                    LA_CYC(3);
                    // Scores stay unscaled; exp(x/sqrt(d)) = exp2(x * scale_log2).  The reference
                    // m_run only moves when the block maximum exceeds it by more than 2^8 in the
                    // exponent (or no key was seen yet): softmax is invariant to the reference, and
                    // skipping small moves saves rescaling the accumulators nearly every time.
                    const bool move = (mx - m_run[rw]) * p.scale_log2 > 8.0f || m_run[rw] == kNegInf;
                    const float m_new = move ? mx : m_run[rw];
                    const float m_use = (m_new == kNegInf) ? 0.0f : m_new;
                    const float neg_mc = -m_use * p.scale_log2;
                    if (__builtin_amdgcn_ballot_w64(move) != 0ull) {
                        const float alpha = fast_exp2(__builtin_fmaf(m_run[rw], p.scale_log2, neg_mc));
                        l_run[rw] *= alpha;
#pragma unroll
                        for (int db = 0; db < C::DB; ++db)
#pragma unroll
                            for (int i = 0; i < 16; ++i) o[rw][db][i] *= alpha;
                    }
                    m_run[rw] = m_new;
                    float psum0 = 0.0f, psum1 = 0.0f;
                    float pv[16];
#pragma unroll
                    for (int i = 0; i < 16; i += 2) {
                        pv[i] = fast_exp2(__builtin_fmaf(s[rw][i], p.scale_log2, neg_mc));
                        pv[i + 1] = fast_exp2(__builtin_fmaf(s[rw][i + 1], p.scale_log2, neg_mc));
                        psum0 += pv[i];
                        psum1 += pv[i + 1];
                    }
                    l_run[rw] += psum0 + psum1;
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                        for (int e = 0; e < 8; ++e) pf[rw][kk][e] = (__bf16)pv[kk * 8 + e];
                }
                __builtin_amdgcn_sched_barrier(0);
                LA_CYC(4);

                // ---- O^T += V^T P^T
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int db = 0; db < C::DB; ++db)
#pragma unroll
                        for (int rw = 0; rw < RW; ++rw)
                            o[rw][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][db], pf[rw][kk], o[rw][db], 0, 0, 0);
            }
            LA_CYC(5);
            if (it < 8) LA_STAMP(9 + 2 * it);
        }

        LA_STAMP(3);
#ifdef LA_DEV_KNOBS
        if ((p.dev_mode & 15) == 1 || (p.dev_mode & 15) == 2) {  // stop after the main loop
            if (l_run[0] == 123.456f) p.out[tid] = (__bf16)o[0][0][0];
            return;
        }
#endif
        // the two half-waves of a row hold the sums over their own keys
#pragma unroll
        for (int rw = 0; rw < RW; ++rw) l_run[rw] += __shfl_xor(l_run[rw], 32, 64);

        __syncthreads();  // all stages consumed: LDS is reused below

        // ---- merge the KS waves of a row tile through LDS, pairwise: at each step the waves
        //      whose key index has the step's bit set hand their state to the wave `step` below
        //      (fragment layout: [4 regs][lane], 16 bytes per lane and access)
        if (KS > 1) {
            float* mg = reinterpret_cast<float*>(lds);
#pragma unroll
            for (int step = 1; step < KS; step <<= 1) {
                const bool sender = (ks & (2 * step - 1)) == step;
                const bool receiver = (ks & (2 * step - 1)) == 0;
                // slot of the pair within this step: one per (receiver, tile)
                float* slot = mg + (((ks >> 1) / step * RT + rt) * RW) * C::TILE_FLOATS;
                if (sender && wave_active) {
#pragma unroll
                    for (int rw = 0; rw < RW; ++rw) {
                        float* dst = slot + rw * C::TILE_FLOATS;
#pragma unroll
                        for (int db = 0; db < C::DB; ++db)
#pragma unroll
                            for (int i4 = 0; i4 < 4; ++i4) {
                                f32x4 v = {o[rw][db][i4 * 4], o[rw][db][i4 * 4 + 1], o[rw][db][i4 * 4 + 2],
                                           o[rw][db][i4 * 4 + 3]};
                                *reinterpret_cast<f32x4*>(dst + ((db * 4 + i4) * 64 + lane) * 4) = v;
                            }
                        *reinterpret_cast<f32x2*>(dst + C::FRAG_FLOATS + lane * 2) = f32x2{m_run[rw], l_run[rw]};
                    }
                }
                __syncthreads();
                if (receiver && wave_active) {
#pragma unroll
                    for (int rw = 0; rw < RW; ++rw) {
                        const float* src = slot + rw * C::TILE_FLOATS;
                        const f32x2 ml2 = *reinterpret_cast<const f32x2*>(src + C::FRAG_FLOATS + lane * 2);
                        const float m2 = ml2[0], l2 = ml2[1];
                        const float m_new = fmaxf(m_run[rw], m2);
                        const float m_use = (m_new == kNegInf) ? 0.0f : m_new;
                        const float a1 = fast_exp2((m_run[rw] - m_use) * p.scale_log2);
                        const float a2 = fast_exp2((m2 - m_use) * p.scale_log2);
                        l_run[rw] = l_run[rw] * a1 + l2 * a2;
                        m_run[rw] = m_new;
#pragma unroll
                        for (int db = 0; db < C::DB; ++db)
#pragma unroll
                            for (int i4 = 0; i4 < 4; ++i4) {
                                const f32x4 v = *reinterpret_cast<const f32x4*>(src + ((db * 4 + i4) * 64 + lane) * 4);
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    o[rw][db][i4 * 4 + e] = o[rw][db][i4 * 4 + e] * a1 + v[e] * a2;
                            }
                    }
                }
                __syncthreads();
            }
        }
        LA_STAMP(4);
        if (direct) break;

        // ---- split combine: store this split's partial, then take a ticket
        unsigned char* group_base = reinterpret_cast<unsigned char*>(p.partials) +
                                    (size_t)((kvh * p.n_row_blocks + rb) * p.XS) * C::PART_WG_BYTES;
        if (ks == 0 && wave_active) {
#pragma unroll
            for (int rw = 0; rw < RW; ++rw) {
                unsigned char* dst = group_base + (size_t)xs * C::PART_WG_BYTES +
                                     (size_t)(rt * RW + rw) * C::PART_TILE_BYTES;
#pragma unroll
                for (int db = 0; db < C::DB; ++db)
#pragma unroll
                    for (int i8 = 0; i8 < 2; ++i8) {
                        bf16x8 v;
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (__bf16)o[rw][db][i8 * 8 + e];
                        *reinterpret_cast<bf16x8*>(dst + ((db * 2 + i8) * 64 + lane) * 16) = v;
                    }
                *reinterpret_cast<f32x2*>(dst + C::PART_ACC_BYTES + lane * 8) = f32x2{m_run[rw], l_run[rw]};
            }
        }
        // Stores are acknowledged by the L2 of this XCD: wait for them, then publish.
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        LA_STAMP(5);
        if (tid == 0) {
            // One atomic carries the arrival count and, to tell whether every member of the group
            // ran on the same XCD (and so shares one L2), the sum and the sum of squares of the
            // members' XCD ids: XS * sum(x^2) == (sum x)^2 holds iff all ids are equal.
            const unsigned x = xcc_id();
            const unsigned mine = 1u | (x << 8) | ((x * x) << 18);
            unsigned* ticket = p.tickets + (kvh * p.n_row_blocks + rb);
            const unsigned total = atomicAdd(ticket, mine) + mine;
            const unsigned cnt = total & 0xffu, sum = (total >> 8) & 0x3ffu, sq = total >> 18;
            unsigned role = 0;
            if (cnt == (unsigned)p.XS) {
                *ticket = 0u;  // everyone has arrived; clean for the next call
                role = (sq * (unsigned)p.XS == sum * sum && !p.force_recompute) ? 1u : 2u;
            }
            *s_role = role;
        }
        __syncthreads();
        const unsigned role = __builtin_amdgcn_readfirstlane(*s_role);  // same in every lane
        LA_STAMP(6);
        if (role == 0) return;
#ifdef LA_DEV_KNOBS
        if (p.dev_mode == 4) return;  // everything but the final merge
#endif
        if (role == 1) {
            // ---- last to arrive, all partials sit in the L2 this XCD shares: merge them in
            //      index order.  Work unit: one (tile, 32-column block); a wave takes two units
            //      at a time and requests all their partials before merging any, so that the
            //      usual case (at most 4 splits) costs one trip to the L2.
            constexpr int NSUB = C::TILES * C::DB;
            constexpr int NU = (RW == 1 && NSUB > C::NW) ? 2 : 1;  // units in flight per wave
            constexpr int MB = RW == 1 ? 4 : 2;                     // splits requested at a time
            for (int st0 = wave; st0 < NSUB; st0 += NU * C::NW) {
                float m_acc[NU], l_acc[NU];
                float acc[NU][16];
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    m_acc[u] = kNegInf;
                    l_acc[u] = 0.0f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[u][i] = 0.0f;
                }
                for (int s0 = 0; s0 < p.XS; s0 += MB) {
                    // request everything of this batch, then merge: one trip to the L2
                    f32x2 ml[NU][MB];
                    bf16x8 v[NU][MB][2];
#pragma unroll
                    for (int u = 0; u < NU; ++u) {
                        const int st = min(st0 + u * C::NW, NSUB - 1);
                        const int tile = st / C::DB, db = st - tile * C::DB;
                        const unsigned char* src0 = group_base + (size_t)tile * C::PART_TILE_BYTES;
#pragma unroll
                        for (int w = 0; w < MB; ++w) {
                            const int s2 = min(s0 + w, p.XS - 1);
                            const unsigned char* src = src0 + (size_t)s2 * C::PART_WG_BYTES;
                            ml[u][w] = *reinterpret_cast<const f32x2*>(src + C::PART_ACC_BYTES + lane * 8);
#pragma unroll
                            for (int i8 = 0; i8 < 2; ++i8)
                                v[u][w][i8] = *reinterpret_cast<const bf16x8*>(src + ((db * 2 + i8) * 64 + lane) * 16);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < NU; ++u) {
                        // batch maximum, then one weight per split: acc = acc * a0 + sum_w v_w * a_w
                        float mb = m_acc[u];
#pragma unroll
                        for (int w = 0; w < MB; ++w)
                            if (s0 + w < p.XS) mb = fmaxf(mb, ml[u][w][0]);
                        const float m_use = (mb == kNegInf) ? 0.0f : mb;
                        const float a0 = fast_exp2((m_acc[u] - m_use) * p.scale_log2);
                        l_acc[u] *= a0;
                        if (s0 > 0) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc[u][i] *= a0;
                        }
                        m_acc[u] = mb;
#pragma unroll
                        for (int w = 0; w < MB; ++w) {
                            const float aw = s0 + w < p.XS ? fast_exp2((ml[u][w][0] - m_use) * p.scale_log2) : 0.0f;
                            l_acc[u] = __builtin_fmaf(ml[u][w][1], aw, l_acc[u]);
#pragma unroll
                            for (int i8 = 0; i8 < 2; ++i8)
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    acc[u][i8 * 8 + e] = __builtin_fmaf((float)v[u][w][i8][e], aw, acc[u][i8 * 8 + e]);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int st = st0 + u * C::NW;
                    if (st >= NSUB) break;
                    const int tile = st / C::DB, db = st - tile * C::DB;
                    const float inv = 1.0f / l_acc[u];
                    unsigned char* row_ptr = lds + (tile * 32 + l32) * C::OUT_PITCH;
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        bf16x4 ov;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(acc[u][i4 * 4 + e] * inv);
                        *reinterpret_cast<bf16x4*>(row_ptr + (db * 32 + i4 * 8 + hi * 4) * 2) = ov;
                    }
                }
            }
            LA_STAMP(20);
            __syncthreads();
            LA_STAMP(21);
            write_rows_from_lds<C>(p, lds, rb, kvh, tid);
            LA_STAMP(7);
            return;
        }
        // ---- role 2: the group was spread over several XCDs, whose L2s are not coherent with
        //      each other inside a kernel.  Inputs are read-only and always coherent, so the last
        //      workgroup simply recomputes its rows over every chunk and writes them directly.
        c_begin = 0;
        c_end = p.n_chunks;
        direct = true;
    }

    // ---- normalise, transpose through LDS, write bf16 rows with 16-byte stores
    if (ks == 0 && wave_active) {
#pragma unroll
        for (int rw = 0; rw < RW; ++rw) {
            const float inv = 1.0f / l_run[rw];  // >= 1 visible key per row, so l > 0
            unsigned char* row_ptr = lds + ((rt * RW + rw) * 32 + l32) * C::OUT_PITCH;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[rw][db][i4 * 4 + e] * inv);
                    const int dcol = db * 32 + i4 * 8 + hi * 4;
                    *reinterpret_cast<bf16x4*>(row_ptr + dcol * 2) = v;
                }
        }
    }
    __syncthreads();
    write_rows_from_lds<C>(p, lds, rb, kvh, tid);
}

// ---------------------------------------------------------------------------------------
// host side

struct Plan {
    int RW, RT, KS, XS, NS;   // NS = LDS stages
    int KC;                   // keys per chunk
    int n_row_blocks;
    int n_prefix_chunks, n_chunks;
    size_t partial_bytes_per_wg;
};


// Most LDS stages that fit beside the workgroup's Q rows.
int max_stages(int D, int RW, int RT, int KC)
{
    const int tiles = RW * RT;
    if (D != 128) return 4;
    return tiles <= 2 ? 4 : (tiles <= 4 ? 3 : 2);
}

bool plan_supported(int D, int RW, int RT, int KS, int NS, int KC)
{
    if (KC == 32) return D == 128 && RW == 1 && RT == 2 && KS == 2 && NS == 9;
    if (KC != 64) return false;
    if (KS == 4) return D == 128 && RW == 1 && RT == 2 && NS == 4;
    if (RT == 4 && KS == 2) return D == 128 && RW == 1 && NS == 4;
    if (NS != 2 && NS != max_stages(D, RW, RT, KC)) return false;
    if (D == 128)
        return (RW == 1 && ((RT == 1 && KS == 2) || (RT == 2 && KS == 2) || (RT == 4 && KS == 1) ||
                            (RT == 2 && KS == 1))) ||
               (RW == 2 && ((RT == 2 && KS == 2) || (RT == 4 && KS == 1)));
    return RW == 1 && ((RT == 1 && KS == 2) || (RT == 2 && KS == 2) || (RT == 4 && KS == 1));
}

Plan make_plan(int P, int T, int group, int kv_heads, int D)
{
    Plan pl;
    const int R = T * group;
    const int tiles = (R + 31) / 32;
    pl.KC = 64;
    // Few rows per KV head (memory-bound): 64-row workgroups whose wave pairs split the keys.
    // Many rows (grouped-query models, wide windows): 128-row workgroups, one tile per wave.
    // (64-row waves, RW = 2, are compiled and tested but were slower in every measurement.)
    if (tiles <= 1) { pl.RW = 1; pl.RT = 1; pl.KS = 2; }
    else if (tiles <= 4 || D != 128) { pl.RW = 1; pl.RT = 2; pl.KS = 2; }
    else { pl.RW = 1; pl.RT = 4; pl.KS = 1; }
    pl.XS = 0;
    pl.NS = 0;
    // developer override: LA_ATTN_PLAN="RW,RT,KS,XS,NS,KC" (XS = 0 keeps the heuristic)
    if (const char* env = getenv("LA_ATTN_PLAN")) {
        int a = 0, b = 0, c = 0, d = 0, e = 0, f = 0;
        if (sscanf(env, "%d,%d,%d,%d,%d,%d", &a, &b, &c, &d, &e, &f) == 6 &&
            plan_supported(D, a, b, c, e, f)) {
            pl.RW = a; pl.RT = b; pl.KS = c; pl.XS = d; pl.NS = e; pl.KC = f;
        }
    }
    if (pl.NS == 0) pl.NS = max_stages(D, pl.RW, pl.RT, pl.KC);
    pl.n_prefix_chunks = (P + pl.KC - 1) / pl.KC;
    pl.n_chunks = pl.n_prefix_chunks + (T + pl.KC - 1) / pl.KC;
    const int rows_wg = pl.RT * pl.RW * 32;
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
    pl.partial_bytes_per_wg = (size_t)pl.RT * pl.RW * ((size_t)(D / 32) * 16 * 64 * 2 + 64 * 8);
    return pl;
}

template <int D, int RW, int RT, int KS, int NSTAGE, int KC = 64>
la_status launch_cfg(const AttnParams& prm, hipStream_t stream)
{
    using C = Cfg<D, RW, RT, KS, KC, NSTAGE>;
    auto kern = step_attention_kernel<D, RW, RT, KS, KC, NSTAGE>;
    static bool attr_set[16] = {false};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return fail(LA_EHIP, "hipGetDevice failed");
    if (!attr_set[dev]) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return fail(LA_EHIP, "hipFuncSetAttribute(%d bytes LDS): %s", C::LDS_BYTES, hipGetErrorString(e));
        attr_set[dev] = true;
    }
    const unsigned grid = (unsigned)prm.wg_per_xcd * 8u;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS_BYTES, stream, prm);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_step_attention launch: %s", hipGetErrorString(e));
    return LA_OK;
}

}  // namespace

size_t step_attention_workspace_bytes(int P, int W, int N, int G, int heads, int kv_heads, int head_dim)
{
    const int T = 1 + (W + G) * (N - 1);
    const Plan pl = make_plan(P, T, heads / kv_heads, kv_heads, head_dim);
    if (pl.XS <= 1) return 0;
    return (size_t)kv_heads * pl.n_row_blocks * pl.XS * pl.partial_bytes_per_wg;
}

la_status launch_step_attention(const void* q, const void* k_cache, const void* v_cache,
                                const void* step_k, const void* step_v, int P, int W, int N, int G,
                                int heads, int kv_heads, int head_dim, void* out, hipStream_t stream)
{
    const int T = 1 + (W + G) * (N - 1);
    const int group = heads / kv_heads;
    if ((long long)T * group >= (1 << 21) || (long long)T * heads * head_dim * 2 >= (1ll << 31) ||
        (long long)kv_heads * head_dim * 2 >= (1 << 24))
        return fail(LA_EUNSUPPORTED, "la_step_attention: step too large (T=%d, heads=%d)", T, heads);
    const Plan pl = make_plan(P, T, group, kv_heads, head_dim);

    AttnParams prm;
    prm.q = (const __bf16*)q;
    prm.k_cache = (const __bf16*)k_cache;
    prm.v_cache = (const __bf16*)v_cache;
    prm.step_k = (const __bf16*)step_k;
    prm.step_v = (const __bf16*)step_v;
    prm.out = (__bf16*)out;
    prm.partials = nullptr;
    prm.tickets = nullptr;
    prm.P = P; prm.W = W; prm.N = N; prm.G = G; prm.T = T;
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
    // testing hook: exercise the path taken when a split group is not on one XCD
    const char* fr = getenv("LA_FORCE_RECOMPUTE");
    prm.force_recompute = (fr && fr[0] == '1') ? 1 : 0;
#ifdef LA_DEV_KNOBS
    const char* dm = getenv("LA_DEV_MODE");
    prm.dev_mode = dm ? atoi(dm) : 0;
    const char* tp = getenv("LA_DEV_TRACE_PTR");
    prm.dev_trace = tp ? (long long*)strtoull(tp, nullptr, 16) : nullptr;
#endif

    if (pl.XS > 1) {
        const size_t ticket_bytes = (size_t)kv_heads * pl.n_row_blocks * sizeof(unsigned);
        prm.tickets = (unsigned*)zeroed_workspace(ticket_bytes, stream);
        if (!prm.tickets) return LA_ENOMEM;
        const size_t bytes = (size_t)total * pl.partial_bytes_per_wg;
        prm.partials = scratch_workspace(bytes);
        if (!prm.partials) return LA_ENOMEM;
    }

    if (pl.KC == 32) return launch_cfg<128, 1, 2, 2, 9, 32>(prm, stream);
    if (pl.KS == 4) return launch_cfg<128, 1, 2, 4, 4>(prm, stream);
    if (pl.RT == 4 && pl.KS == 2) return launch_cfg<128, 1, 4, 2, 4>(prm, stream);
#define LA_DISPATCH(D_, RW_, RT_, KS_, NSMAX_)                                       \
    if (head_dim == D_ && pl.RW == RW_ && pl.RT == RT_ && pl.KS == KS_) {           \
        if (pl.NS == 2) return launch_cfg<D_, RW_, RT_, KS_, 2>(prm, stream);       \
        return launch_cfg<D_, RW_, RT_, KS_, NSMAX_>(prm, stream);                  \
    }
    LA_DISPATCH(128, 1, 1, 2, 4)
    LA_DISPATCH(128, 1, 2, 2, 4)
    LA_DISPATCH(128, 1, 2, 1, 4)
    LA_DISPATCH(128, 1, 4, 1, 3)
    LA_DISPATCH(128, 2, 2, 2, 3)
    LA_DISPATCH(128, 2, 4, 1, 2)
    LA_DISPATCH(64, 1, 1, 2, 4)
    LA_DISPATCH(64, 1, 2, 2, 4)
    LA_DISPATCH(64, 1, 4, 1, 4)
#undef LA_DISPATCH
    return fail(LA_EUNSUPPORTED, "la_step_attention: no kernel for head_dim=%d plan (%d,%d,%d)",
                head_dim, pl.RW, pl.RT, pl.KS);
}

}  // namespace la

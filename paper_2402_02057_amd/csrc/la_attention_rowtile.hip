// Lookahead-step attention (Sec. 3.3 mask, Sec. 2 attention), the decomposition WITHOUT partial
// results between workgroups: a workgroup owns one tile of 32 query rows of a KV head and one half
// of the value columns, and walks ALL keys of that head (prefix cache, then the step's own keys
// under the mask).  Both halves compute the same scores and softmax weights (that arithmetic is
// cheap where this kernel is used: few rows per KV head) and each multiplies them with its half of
// V, so a finished row block goes straight to `out`: no partials in global memory, no ticket, no
// last-arriver combine, whose chain of round trips to the L2 costs a third of the launch at the
// shapes with one query head per KV head.  The price is that every workgroup of a KV head streams
// all of K (and half of V) from the L2, which serves the copies of one line to the workgroups of a
// head at several times the rate of distinct lines.
//
// Eight waves: four compute (one per SIMD; wave w takes 32-key block w of the iteration's 128 keys)
// and four that do nothing but request chunks.  A request stalls its wave while the compute unit's
// memory pipeline is full; on a wave of its own that stall costs nothing.  The ring holds six
// chunks of 64 keys (K 16 KB + half of V 8 KB each): two being read, four in flight.
//
// Where it is used: the launch costs about 2.5 us until the first chunks have landed, 0.75 us per
// 128 keys with up to 128 workgroups (the compute unit's intake plus a part of the block) and
// 0.95 us with 256 (what the L2s deliver to all compute units at once, every workgroup of a head
// pulling all of K; the arithmetic is hidden then), and 1.5 us to merge and write.  Measured and
// dropped: six computing waves with three chunks in flight, a loop that overlaps the next
// block's MFMAs with the exponentials, 16-row waves, two waves per SIMD half an iteration apart,
// two tiles per workgroup.  That compares with 8 us and more of
// fixed cost for the staged kernel with its split groups: ahead up to a dozen chunks (prefix
// + step <= 768 keys) if its workgroups, 2 per row tile and KV head, fit one round of the compute
// units, behind beyond that (the 7B configuration, 1145 keys: 12.1 against 11.3 us).
//
// Same arithmetic per block as the staged kernel (la_attention.hip): S^T = K Q^T and
// O^T += V^T P^T with v_mfma_f32_32x32x16_bf16, softmax weights in bf16 with the row sum over the
// rounded values, lazy moves of the running reference, mask words from indices.  The four waves'
// states are merged through LDS in fp32, in key order.
//
// Rotating form (ROPE): the query rows, and on request the step keys, arrive as the projection
// left them and are turned in LDS at the positions of Fig. 2(b), with the arithmetic of
// la_step_rope; the table rows of those positions are staged behind Q, in the room of the ring's
// sixth stage.
#include <math.h>

#include <mutex>

#include "la_internal.h"
#include "la_attention_common.h"
#include "la_rope_common.h"

#ifdef LA_DEV_HOOKS_ROWTILE
#include LA_DEV_HOOKS_ROWTILE  // developer builds only: timing stamps, never part of the product build
#else
#define LA_STAMP(k) do { } while (0)
#endif

namespace la {
namespace {

struct RowTileParams {
    const __bf16* q;
    const __bf16* k_cache;
    const __bf16* v_cache;
    const __bf16* step_k;
    const __bf16* step_v;
    __bf16* out;
    long long cache_rows;  // rows between the caches of consecutive KV heads (>= P)
    int P, W, N, T;
    int heads, kv_heads, group;
    int R;                 // T * group query rows per KV head
    int n_tiles;           // 32-row tiles per KV head
    int n_prefix_chunks, n_chunks;
    int total_wg, wg_per_xcd;
    float scale_log2, inv_group, inv_W, inv_n1, inv_tiles;
    // rotating variant: the rows of the model's tables from the prefix length on ([rope_rows][D/2]
    // fp32 each), staged in LDS; bit 0 of the flags: pairing (x[2i], x[2i+1]); bit 1: the step keys
    // arrive unrotated as well
    const float* rope_cos;
    const float* rope_sin;
    int rope_rows, rope_block, rope_flags;
};

constexpr int D = 128;
constexpr int KC = 64;                    // keys per chunk
constexpr int NWC = 4, NWP = 4;           // computing and requesting waves
constexpr int CPI = NWC / 2;              // chunks per iteration: a 32-key block per computing wave
constexpr int K_BYTES = KC * D * 2;       // 16 KB
constexpr int VH_BYTES = KC * D;          // half of the value columns: 8 KB
constexpr int STAGE_BYTES = K_BYTES + VH_BYTES;
constexpr int Q_BYTES = 32 * D * 2;
// The ring: six chunks, or five in the rotating variant, which needs the room for the table rows of
// the step's positions (up to 64 positions of 256 + 256 bytes behind Q).
template <bool ROPE>
struct Ring {
    static constexpr int NSTAGE = ROPE ? 5 : 6;
    static constexpr int Q_OFFSET = NSTAGE * STAGE_BYTES;
    static constexpr int ROPE_OFFSET = Q_OFFSET + Q_BYTES;
    static constexpr int ROPE_MAX_BYTES = ROPE ? 160 * 1024 - ROPE_OFFSET : 0;  // both tables
    static constexpr int LDS_BYTES = ROPE_OFFSET + ROPE_MAX_BYTES;
};
constexpr int ROPE_POS_BYTES = D * 2;     // one position of one table (D/2 fp32)
constexpr int K_LOADS = K_BYTES / 1024 / NWP;   // per requesting wave and chunk: 4
constexpr int V_LOADS = VH_BYTES / 1024 / NWP;  // 2
constexpr int LPW = K_LOADS + V_LOADS;
// merge of the four waves' states: per wave two 32 x 32 slices in fp32 and (m, l) per lane
constexpr int MERGE_WAVE_BYTES = 2 * 16 * 64 * 4 + 64 * 8;
static_assert(Ring<false>::LDS_BYTES <= 160 * 1024 && Ring<true>::LDS_BYTES <= 160 * 1024, "LDS of a compute unit");
static_assert(Ring<true>::NSTAGE >= 2 * CPI, "an iteration's chunks are requested while the last iteration's are read");
static_assert(LPW * (Ring<false>::NSTAGE - CPI) < 64, "vmcnt is a 6-bit counter");
static_assert(NWC * MERGE_WAVE_BYTES <= Ring<true>::NSTAGE * STAGE_BYTES, "the merge reuses the ring");

// Rows of the value half are 128 bytes, two to a sweep of the banks: the transposing read takes 64
// bytes of each of rows r .. r+3 per half-wave; rows two apart start at the same bank, so every
// other pair of rows has the halves of its pieces exchanged.
__device__ __forceinline__ int vh_swizzle(int row) { return (row & 2) << 1; }

// (two waves per SIMD are all there will be: the compiler need not save registers for more)
template <bool ROPE>
__global__ __launch_bounds__((NWC + NWP) * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void step_attention_rowtile_kernel(const RowTileParams)
{
    constexpr int NSTAGE = Ring<ROPE>::NSTAGE, Q_OFFSET = Ring<ROPE>::Q_OFFSET, ROPE_OFFSET = Ring<ROPE>::ROPE_OFFSET;
    const RowTileParams& p = warmed_arguments<RowTileParams>();
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    LA_STAMP(0);
    const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
    const int logical = xcd * p.wg_per_xcd + slot;
    if (logical >= p.total_wg) return;
    const int unit = logical >> 1, vpart = logical & 1;  // (KV head, row tile), half of the value columns
    const int kvh = __builtin_amdgcn_readfirstlane(div_small(unit, p.inv_tiles));
    const int tile = unit - kvh * p.n_tiles;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hi = lane >> 5, l32 = lane & 31;
    const unsigned lds_base = lds_address(lds);
    const int n_chunks = p.n_chunks, n_prefix_chunks = p.n_prefix_chunks;
    const int n_iter = (n_chunks + CPI - 1) / CPI;

    f32x16 o[2];
    float m_run = kNegInf, l_run = 0.0f;
    const float sl2 = p.scale_log2;

    // ---- rotating variant: what every thread of the workgroup does behind an iteration's barrier.
    //      Eight pairs of one 16-bit row in LDS (16-byte pieces swizzled with `sw`) are turned in place
    //      by the staged table rows of position digit `digit`, with the arithmetic of la_step_rope.
    auto rotate_unit = [&](unsigned char* row, int sw, int c, int digit) {
        constexpr int UPR = D / 16;  // units of eight pairs per row
        const bool inter = (p.rope_flags & 1) != 0;
        bf16x8* va = reinterpret_cast<bf16x8*>(row + (((inter ? 2 * c : c) ^ sw) << 4));
        bf16x8* vb = reinterpret_cast<bf16x8*>(row + (((inter ? 2 * c + 1 : c + UPR) ^ sw) << 4));
        const float* cs = reinterpret_cast<const float*>(lds + ROPE_OFFSET + digit * ROPE_POS_BYTES) + c * 8;
        const float* sn = reinterpret_cast<const float*>(lds + ROPE_OFFSET + p.rope_block + digit * ROPE_POS_BYTES) + c * 8;
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
    // Behind the barrier of iteration `it`: in the first one the tile's query rows, and in any one
    // the K rows of those of its chunks that hold step keys (if the keys arrive unrotated), followed
    // by one more barrier.  Whether there is anything to do is the same for every wave.
    auto rotate_after_barrier = [&](int it) {
        if constexpr (ROPE) {
            const int first = it * CPI;
            const bool keys = (p.rope_flags & 2) != 0 && min(first + CPI, n_chunks) > n_prefix_chunks;
            if (it != 0 && !keys) return;
            if (it == 0) {
                for (int u = tid; u < 32 * (D / 16); u += (NWC + NWP) * 64) {
                    const int r = u / (D / 16), c = u - r * (D / 16);
                    const int rr = min(tile * 32 + r, p.R - 1);
                    const int digit = min(step_row_digit(div_small(rr, p.inv_group), p.W, p.N, p.inv_W, p.inv_n1), p.rope_rows - 1);
                    rotate_unit(lds + Q_OFFSET + r * (D * 2), swizzle<D>(r), c, digit);
                }
            }
            if (keys) {
                for (int j = 0; j < CPI; ++j) {
                    const int c_abs = first + j;
                    if (c_abs < n_chunks && c_abs >= n_prefix_chunks) {
                        unsigned char* stage = lds + (c_abs % NSTAGE) * STAGE_BYTES;
                        const int t0 = (c_abs - n_prefix_chunks) * KC;
                        for (int u = tid; u < KC * (D / 16); u += (NWC + NWP) * 64) {
                            const int r = u / (D / 16), c = u - r * (D / 16);
                            const int digit = min(step_row_digit(min(t0 + r, p.T - 1), p.W, p.N, p.inv_W, p.inv_n1), p.rope_rows - 1);
                            rotate_unit(stage + r * (D * 2), swizzle<D>(r), c, digit);
                        }
                    }
                }
            }
            __syncthreads();
        }
    };

    if (wave >= NWC) {
        // ---------------- requesting waves
        const int lw = wave - NWC;
        const unsigned char* const kc_head = reinterpret_cast<const unsigned char*>(p.k_cache) + (size_t)kvh * (size_t)p.cache_rows * (D * 2);
        const unsigned char* const vc_head = reinterpret_cast<const unsigned char*>(p.v_cache) + (size_t)kvh * (size_t)p.cache_rows * (D * 2);
        const unsigned char* const sk_head = reinterpret_cast<const unsigned char*>(p.step_k) + (size_t)kvh * (D * 2);
        const unsigned char* const sv_head = reinterpret_cast<const unsigned char*>(p.step_v) + (size_t)kvh * (D * 2);
        const unsigned step_stride = (unsigned)(p.kv_heads * D * 2);
        // K: a wave-load is 4 rows of 16 pieces; V half: 8 rows of 8 pieces.  LDS side linear, the
        // swizzle on the global side.
        int k_row[K_LOADS], v_row[V_LOADS];
        unsigned k_piece[K_LOADS], v_piece[V_LOADS];
#pragma unroll
        for (int j = 0; j < K_LOADS; ++j) {
            k_row[j] = (lw + j * NWP) * 4 + (lane >> 4);
            k_piece[j] = (unsigned)(((lane & 15) ^ swizzle<D>(k_row[j])) << 4);
        }
#pragma unroll
        for (int j = 0; j < V_LOADS; ++j) {
            v_row[j] = (lw + j * NWP) * 8 + (lane >> 3);
            v_piece[j] = (unsigned)(vpart * D + (((lane & 7) ^ vh_swizzle(v_row[j])) << 4));
        }
        auto issue_chunk = [&](int c) {
            const bool is_step = c >= n_prefix_chunks;
            const int key0 = (c - (is_step ? n_prefix_chunks : 0)) * KC;
            const unsigned stride = is_step ? step_stride : (unsigned)(D * 2);
            const unsigned char* kb = (is_step ? sk_head : kc_head) + (size_t)key0 * stride;
            const unsigned char* vb = (is_step ? sv_head : vc_head) + (size_t)key0 * stride;
            const int last_row = min(KC, (is_step ? p.T : p.P) - key0) - 1;  // rows past the end repeat the last one
            const unsigned dst = lds_base + (unsigned)((c % NSTAGE) * STAGE_BYTES) + (unsigned)lw * 1024u;
#pragma unroll
            for (int j = 0; j < K_LOADS; ++j)
                dma16_base(kb, __umul24((unsigned)min(k_row[j], last_row), stride) + k_piece[j], dst + j * NWP * 1024);
#pragma unroll
            for (int j = 0; j < V_LOADS; ++j)
                dma16_base(vb, __umul24((unsigned)min(v_row[j], last_row), stride) + v_piece[j],
                           dst + K_BYTES + j * NWP * 1024);
        };
        auto issue_q = [&]() {
#pragma unroll
            for (int i = 0; i < Q_BYTES / 1024 / NWP; ++i) {
                const int wl = lw + i * NWP;
                const int row = wl * 4 + (lane >> 4);
                const int lc = (lane & 15) ^ swizzle<D>(row);
                const int rr = min(tile * 32 + row, p.R - 1);
                const int t = div_small(rr, p.inv_group), hh = rr - t * p.group;
                const unsigned off = (unsigned)(((t * p.heads + kvh * p.group + hh) * D + lc * 8) * 2);
                dma16_base(p.q, off, lds_base + Q_OFFSET + wl * 1024);
            }
        };
        if constexpr (ROPE) {
            // the table rows of the step's positions first (they are needed with Q): two linear blocks,
            // 1 KB per wave-load, lanes past the end repeat the last 16 bytes
            const int per_table = p.rope_block >> 10;
            const unsigned last = (unsigned)(p.rope_rows * ROPE_POS_BYTES - 16);
            for (int i = lw; i < 2 * per_table; i += NWP) {
                const bool is_sin = i >= per_table;
                const int j = is_sin ? i - per_table : i;
                dma16_base(is_sin ? p.rope_sin : p.rope_cos, min((unsigned)(j * 1024 + lane * 16), last),
                           lds_base + ROPE_OFFSET + (is_sin ? p.rope_block : 0) + j * 1024);
            }
        }
        int issued = 0;
        // Four chunks before the first barrier (the first iteration's two, Q, two more), the ring's
        // other stages right behind it: a requesting wave cannot reach the barrier while its requests
        // wait to be accepted, so a full ring up front holds the first iteration back (7.1 -> 6.6 us
        // at the 7B heads on 256 keys, 12.7 -> 12.1 on 1024; three or four measure alike, two is slower).
        const int upfront = min(n_chunks, 4);
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s) {
            if (s == CPI) issue_q();  // Q is needed with the first iteration's chunks
            if (s < upfront) issue_chunk(s);
        }
        issued = upfront;
        LA_STAMP(1);
        for (int it = 0, done = 0; it < n_iter; ++it, done += CPI) {
            // this iteration's chunks (and Q, requested before chunk CPI) have landed; younger ones stay in flight
            wait_young<LPW, NSTAGE - CPI>(issued - min(n_chunks, done + CPI));
            __syncthreads();
            // the stages read in the last iteration are free: the ring has room up to chunk done + NSTAGE - 1
            const int room = min(n_chunks, done + NSTAGE);
            while (issued < room) issue_chunk(issued++);
            rotate_after_barrier(it);
        }
        wait_vmcnt<0>();
        __syncthreads();  // (the computing waves are through with the ring)
        __syncthreads();  // (their states are in LDS)
        return;
    }

    // ---------------- computing waves
    const int ks = wave;                      // block of the iteration's 128 keys
    const int my_chunk = ks >> 1, kb = ks & 1;
    const int row0 = tile * 32;               // first row of the tile (in R space)
    const int t_lane = div_small(min(row0 + l32, p.R - 1), p.inv_group);
    const RowVis vis = row_visibility(t_lane, p.W, p.N, p.inv_W, p.inv_n1);
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.0f;

    // LDS read offsets of this lane relative to the start of a stage
    unsigned k_off[D / 16], v_off[2][2];
    {
        const int krow = kb * 32 + l32;
        const int ksw = swizzle<D>(krow);
#pragma unroll
        for (int j = 0; j < D / 16; ++j) k_off[j] = (unsigned)(krow * (D * 2) + (((j * 2 + hi) ^ ksw) << 4));
        // V^T operand: k-slot e of half `hi` of 16-key step kk is key kb*32 + kk*16 + (e/4)*8 + hi*4 + e%4;
        // a 16-lane block reads 4 keys x 16 columns, the transposing read hands lane n column n
        const int b16 = lane >> 4, i16 = lane & 15;
        const int jj = i16 >> 2, q4 = i16 & 3;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int vrow = kb * 32 + hi * 4 + jj + r * 8;
            const int sw = vh_swizzle(vrow);  // (the same for vrow + 16)
#pragma unroll
            for (int db = 0; db < 2; ++db) {
                const int col = db * 32 + (b16 & 1) * 16 + q4 * 4;  // within the half
                const int lc = col >> 3, within = (col & 7) * 2;
                v_off[r][db] = (unsigned)(K_BYTES + vrow * D + ((lc ^ sw) << 4) + within);
            }
        }
    }

    const int n_P = p.P, n_T = p.T;
    bf16x8 qreg[D / 16];
    for (int it = 0, done = 0; it < n_iter; ++it, done += CPI) {
        __syncthreads();  // this iteration's chunks have landed; everyone is done with the last ones
        if (it < 4) LA_STAMP(8 + 2 * it);
        rotate_after_barrier(it);
        if (it == 0) {
            const unsigned char* qr = lds + Q_OFFSET + l32 * (D * 2);
            const int qsw = swizzle<D>(l32);
#pragma unroll
            for (int k16 = 0; k16 < D / 16; ++k16)
                qreg[k16] = *reinterpret_cast<const bf16x8*>(qr + (((k16 * 2 + hi) ^ qsw) << 4));
        }
        const int c = done + my_chunk;
        if (c < n_chunks) {
            const bool is_step = c >= n_prefix_chunks;
            const int key0 = (c - (is_step ? n_prefix_chunks : 0)) * KC + kb * 32;
            const int limit = is_step ? n_T : n_P;
            if (key0 < limit) {
                // ---- which of this lane's 16 keys of the block its row may see (bit (i/4)*8 + i%4 for
                //      score register i); a step block that no row of the tile sees at all is skipped
                const bool full = !is_step && (key0 + 32 <= limit);
                unsigned word = 0xFFFFFFFFu;
                bool skip = false;
                if (!full) {
                    if (is_step) word = step_block_word(vis, key0);
                    else word = (1u << (limit - key0)) - 1u;  // 1..31 keys left
                    word = (word >> (hi * 4)) & 0x0F0F0F0Fu;
                    skip = is_step && __builtin_amdgcn_ballot_w64(word != 0u) == 0ull;
                }
                if (!skip) {
                    const unsigned char* blk = lds + (unsigned)((c % NSTAGE) * STAGE_BYTES);
                    bf16x8 kf[D / 16];
#pragma unroll
                    for (int k16 = 0; k16 < D / 16; ++k16) kf[k16] = *reinterpret_cast<const bf16x8*>(blk + k_off[k16]);
                    bf16x8 vf[2][2];
                    auto read_v = [&](int kk) {
#pragma unroll
                        for (int db = 0; db < 2; ++db) {
                            union { struct { short4v a, b; } s; bf16x8 v; } u;
                            u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (short4v __attribute__((address_space(3)))*)(blk + v_off[0][db] + kk * 16 * D));
                            u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (short4v __attribute__((address_space(3)))*)(blk + v_off[1][db] + kk * 16 * D));
                            vf[kk][db] = u.v;
                        }
                    };
                    read_v(0);
                    // (all of K in registers before the first MFMA: left alone, the compiler reads piece
                    // by piece into the same registers and every MFMA waits for a round trip to LDS)
                    asm volatile("" ::"v"(kf[0]), "v"(kf[1]), "v"(kf[2]), "v"(kf[3]), "v"(kf[4]), "v"(kf[5]), "v"(kf[6]), "v"(kf[7]));
                    // ---- S^T block: 32 keys x 32 rows
                    f32x16 s;
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[i] = 0.0f;
#pragma unroll
                    for (int k16 = 0; k16 < D / 16; ++k16)
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[k16], qreg[k16], s, 0, 0, 0);
                    read_v(1);  // in flight during the softmax arithmetic
                    // ---- mask, running maximum, exponentials (as in the staged kernel)
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
                    const bool move = (mx - m_run) * sl2 > 8.0f || m_run == kNegInf;
                    const float m_new = move ? mx : m_run;
                    const float m_use = (m_new == kNegInf) ? 0.0f : m_new;  // the row has seen no key at all
                    const float neg_mc = -m_use * sl2;
                    if (__builtin_amdgcn_ballot_w64(move) != 0ull) {
                        const float alpha = fast_exp2(__builtin_fmaf(m_run, sl2, neg_mc));
                        l_run *= alpha;
#pragma unroll
                        for (int db = 0; db < 2; ++db)
#pragma unroll
                            for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
                    }
                    m_run = m_new;
                    // P in bf16, as the PV product uses it; the row sum adds up those same rounded values
                    bf16x8 pf[2];
#pragma unroll
                    for (int i = 0; i < 16; ++i) pf[i >> 3][i & 7] = (__bf16)fast_exp2(__builtin_fmaf(s[i], sl2, neg_mc));
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
                    // ---- O^T += V^T P^T (this workgroup's half of the columns)
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                        for (int db = 0; db < 2; ++db)
                            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][db], pf[kk], o[db], 0, 0, 0);
                }
            }
        }
        if (it < 4) LA_STAMP(9 + 2 * it);
    }
    LA_STAMP(3);
    l_run += __shfl_xor(l_run, 32, 64);  // the two half-waves of a row hold the sums over their own keys

    // ---- merge the four waves: every wave leaves its two slices and (m, l); after the barrier wave w
    //      sums registers (w/2)*8 .. +7 of slice w%2 over the four states, in key order, and writes
    //      those columns of its rows
    __syncthreads();  // everyone is through with the ring
    {
        unsigned char* dst = lds + wave * MERGE_WAVE_BYTES;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4)
                *reinterpret_cast<f32x4*>(dst + ((db * 4 + i4) * 64 + lane) * 16) =
                    f32x4{o[db][i4 * 4], o[db][i4 * 4 + 1], o[db][i4 * 4 + 2], o[db][i4 * 4 + 3]};
        *reinterpret_cast<f32x2*>(dst + 2 * 16 * 64 * 4 + lane * 8) = f32x2{m_run, l_run};
    }
    LA_STAMP(2);
    __syncthreads();
    LA_STAMP(19);
    constexpr int QW = 2;  // four-register groups of a slice per wave
    const int my_db = wave & 1, my_part = wave >> 1;
    f32x2 ml[NWC];
    f32x4 v[NWC][QW];
#pragma unroll
    for (int k = 0; k < NWC; ++k) {
        const unsigned char* src = lds + k * MERGE_WAVE_BYTES;
        ml[k] = *reinterpret_cast<const f32x2*>(src + 2 * 16 * 64 * 4 + lane * 8);
#pragma unroll
        for (int h = 0; h < QW; ++h)
            v[k][h] = *reinterpret_cast<const f32x4*>(src + ((my_db * 4 + my_part * QW + h) * 64 + lane) * 16);
    }
    float m_all = ml[0][0];
#pragma unroll
    for (int k = 1; k < NWC; ++k) m_all = fmaxf(m_all, ml[k][0]);
    const float m_use = (m_all == kNegInf) ? 0.0f : m_all;
    float a[NWC], l = 0.0f;
#pragma unroll
    for (int k = 0; k < NWC; ++k) {
        a[k] = fast_exp2((ml[k][0] - m_use) * sl2);
        l = __builtin_fmaf(ml[k][1], a[k], l);
    }
    LA_STAMP(4);
    const int rr = row0 + l32;
    if (rr < p.R) {
        const float inv = 1.0f / l;  // (>= 1 visible key per row, so l > 0)
        const int t = div_small(rr, p.inv_group), hh = rr - t * p.group;
        __bf16* row = p.out + ((size_t)t * p.heads + (size_t)kvh * p.group + hh) * D + vpart * (D / 2) + my_db * 32 + hi * 4;
#pragma unroll
        for (int h = 0; h < QW; ++h) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float acc = v[0][h][e] * a[0];
#pragma unroll
                for (int k = 1; k < NWC; ++k) acc = __builtin_fmaf(v[k][h][e], a[k], acc);
                w[e] = (__bf16)(acc * inv);
            }
            *reinterpret_cast<bf16x4*>(row + (my_part * QW + h) * 8) = w;
        }
    }
    LA_STAMP(7);
}

}  // namespace

bool rowtile_supported(int head_dim, int group, int T)
{
    return head_dim == D && (long long)T * group < (1 << 21);
}

// Positions whose table rows fit behind the rotating variant's ring.
int rowtile_rope_positions() { return Ring<true>::ROPE_MAX_BYTES / (2 * ROPE_POS_BYTES); }

namespace {

template <bool ROPE>
la_status launch_rowtile(const RowTileParams& p, hipStream_t stream)
{
    constexpr int kLds = Ring<ROPE>::LDS_BYTES;
    auto kern = step_attention_rowtile_kernel<ROPE>;
    static bool attr_set[16] = {false};
    static std::mutex mutex;
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return fail(LA_EHIP, "hipGetDevice failed");
        std::lock_guard<std::mutex> lock(mutex);
        if (!attr_set[dev]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
            if (e != hipSuccess) return fail(LA_EHIP, "hipFuncSetAttribute(%d bytes LDS): %s", kLds, hipGetErrorString(e));
            attr_set[dev] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)p.wg_per_xcd * 8u), dim3((NWC + NWP) * 64), kLds, stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_step_attention launch: %s", hipGetErrorString(e));
    return LA_OK;
}

}  // namespace

// `rope` != nullptr: q (and with rope->rotate_keys the step keys) arrive unrotated; the caller has
// checked that the tables cover the step's positions and that those fit (rowtile_rope_positions).
la_status launch_step_attention_rowtile(const void* q, const void* k_cache, const void* v_cache, long long capacity,
                                        const void* step_k, const void* step_v, int P, int W, int N, int G, int heads,
                                        int kv_heads, void* out, hipStream_t stream, const RopeTables* rope)
{
    RowTileParams p;
    p.q = (const __bf16*)q;
    p.k_cache = (const __bf16*)k_cache;
    p.v_cache = (const __bf16*)v_cache;
    p.step_k = (const __bf16*)step_k;
    p.step_v = (const __bf16*)step_v;
    p.out = (__bf16*)out;
    p.cache_rows = capacity;
    p.P = P; p.W = W; p.N = N;
    p.T = 1 + (W + G) * (N - 1);
    p.heads = heads; p.kv_heads = kv_heads; p.group = heads / kv_heads;
    p.R = p.T * p.group;
    p.n_tiles = (p.R + 31) / 32;
    p.n_prefix_chunks = (P + KC - 1) / KC;
    p.n_chunks = p.n_prefix_chunks + (p.T + KC - 1) / KC;
    p.total_wg = kv_heads * p.n_tiles * 2;
    p.wg_per_xcd = (p.total_wg + 7) / 8;
    p.scale_log2 = 1.4426950408889634f / sqrtf((float)D);
    p.inv_group = 1.0f / (float)p.group;
    p.inv_W = W > 0 ? 1.0f / (float)W : 1.0f;
    p.inv_n1 = 1.0f / (float)(N - 1);
    p.inv_tiles = 1.0f / (float)p.n_tiles;
    p.rope_cos = p.rope_sin = nullptr;
    p.rope_rows = p.rope_block = p.rope_flags = 0;
    if (!rope) return launch_rowtile<false>(p, stream);
    // the furthest position of the step: the newest window level's last column, or a candidate's last token
    const int far = W > 0 ? (W + N - 2 > N - 1 ? W + N - 2 : N - 1) : (G > 0 ? N - 1 : 0);
    p.rope_rows = far + 1;
    p.rope_block = (p.rope_rows * ROPE_POS_BYTES + 1023) / 1024 * 1024;
    if (2 * p.rope_block > Ring<true>::ROPE_MAX_BYTES)
        return fail(LA_EUNSUPPORTED, "la_step_attention_rope: %d positions do not fit beside the ring", p.rope_rows);
    p.rope_flags = (rope->interleaved ? 1 : 0) | (rope->rotate_keys ? 2 : 0);
    p.rope_cos = rope->cos + (size_t)P * (D / 2);
    p.rope_sin = rope->sin + (size_t)P * (D / 2);
    return launch_rowtile<true>(p, stream);
}

}  // namespace la

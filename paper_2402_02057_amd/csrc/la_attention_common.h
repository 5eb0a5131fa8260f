// Device-side helpers shared by the lookahead-step attention kernels (la_attention.hip: the
// staged kernel, whose workgroups split the keys of a row block and combine partial results;
// la_attention_rowtile.hip: the kernel whose workgroups walk all keys for one row tile).  Nothing
// here is part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>

namespace la {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegInf = -__builtin_huge_valf();

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

// The maxima above and below are written as assembly, which the compiler's hazard bookkeeping does
// not look into: a vector instruction must not read the result registers of a matrix instruction
// for up to 19 cycles after it was issued (it would see the accumulator before the last pass; seen
// here as a reference maximum that changed from run to run).  Where such a maximum may directly
// follow the MFMA that produces its operands, these idle cycles stand in for the wait the compiler
// would have inserted.
template <class V>
__device__ __forceinline__ void settle_mfma_result(V& acc)
{
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 2" : "+v"(acc));
}

__device__ __forceinline__ float max2(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// max of a value with the one held by the lane 32 away (the other 16 keys of the same row).
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of its
// second: fed the same value twice it returns (lower half everywhere, upper half everywhere).
__device__ __forceinline__ float max_across_halves(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return max2(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most y * LPW of this wave's loads are still in flight, 0 <= y <= Y.  The
// steady-state value (the largest) costs one comparison.
template <int LPW, int Y>
__device__ __forceinline__ void wait_young(int y)
{
    static_assert(LPW * Y < 64, "vmcnt is a 6-bit counter");
    if constexpr (Y > 0) {
        if (y < Y) {
            wait_young<LPW, Y - 1>(y);
            return;
        }
    }
    wait_vmcnt<Y * LPW>();
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


// The same with 4 bytes per lane (256 bytes per wave).
__device__ __forceinline__ void dma4_base(const void* base, unsigned lane_off, unsigned lds_base)
{
    const unsigned long long b = reinterpret_cast<unsigned long long>(base);
    const unsigned long long lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
    const unsigned long long hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(lane_off), "s"((hi << 32) | lo), "s"(lds_base)
                 : "memory");
}

__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}

// 16-byte piece `lc` of row `row` lives at piece position lc ^ row_swizzle(row) of that row, for
// rows of RB bytes (256: 16 pieces, 128: 8 pieces, 64: 4 pieces).  Chosen so that the lanes of a
// 16-byte read down a column of pieces (16 consecutive rows), and of a transposing read (rows
// h*4 .. h*4+3 and 8 + h*4 .. +3), hit distinct banks.
template <int RB>
__device__ __forceinline__ int row_swizzle(int row)
{
    static_assert(RB == 256 || RB == 128 || RB == 64, "row sizes in use");
    if (RB == 256) return ((row & 3) << 2) | ((row >> 2) & 3);
    if (RB == 128) return (row >> 1) & 7;
    return (row >> 2) & 3;
}
// (rows of D bf16 elements)
template <int D>
__device__ __forceinline__ int swizzle(int row)
{
    return row_swizzle<D * 2>(row);
}

// Position of step row t relative to the current token (the digit on the token in Fig. 2(b)):
// 0 for the current token, 1 + level + column for a lookahead token, 1 + index for a candidate token.
__device__ __forceinline__ int step_row_digit(int t, int W, int N, float inv_W, float inv_n1)
{
    if (t == 0) return 0;
    const int n_look = W * (N - 1);
    if (t <= n_look) return 1 + (t - 1) - div_small(t - 1, inv_W) * (W - 1);  // 1 + l + j with t - 1 = l*W + j
    const int x = t - 1 - n_look;
    return 1 + x - div_small(x, inv_n1) * (N - 1);
}

// Eight 8-bit floats (E4M3, finite-only; `lo` holds the first four, lowest byte first) as bf16:
// every such value is a bf16 number, so the conversion (scale 1) is exact.
__device__ __forceinline__ bf16x8 fp8x8_to_bf16(unsigned lo, unsigned hi)
{
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
    const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
    const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
    return bf16x8{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

// Id of the XCD (accelerator die, with its own L2) this wave runs on.
__device__ __forceinline__ unsigned xcc_id()
{
    unsigned v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return v & 0xfu;
}

// Kernel arguments are read through the scalar cache, which every launch finds empty; the compiler
// loads a field shortly before its first use, so the way to the first request to memory led
// through several such misses one after the other.  Here every 64-byte line of the arguments is
// touched at once - one miss - and the pointer the kernel then reads its arguments through is an
// output of that statement, so that no such read can be moved ahead of it.  Plain scalar loads,
// waited for on the spot.  `offset`: where in the argument segment the T sits (the kernel's own
// parameter only gives the segment its layout).
template <class T>
__device__ __forceinline__ const T& warmed_arguments(unsigned offset = 0)
{
    typedef const char __attribute__((address_space(4))) * kernarg_ptr;
    kernarg_ptr k = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr() + offset;
    constexpr unsigned bytes = (unsigned)sizeof(T);
    static_assert(bytes <= 256, "four lines per statement");
    unsigned d0, d1, d2, d3;
    asm volatile(
        "s_load_dword %0, %4, 0x0\n\t"
        "s_load_dword %1, %4, %5\n\t"
        "s_load_dword %2, %4, %6\n\t"
        "s_load_dword %3, %4, %7\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(d0), "=&s"(d1), "=&s"(d2), "=&s"(d3), "+s"(k)
        : "s"(bytes > 64 ? 64u : 0u), "s"(bytes > 128 ? 128u : 0u), "s"(bytes > 192 ? 192u : bytes - 4u)
        : "memory");
    return *(const T*)k;
}

}  // namespace
}  // namespace la

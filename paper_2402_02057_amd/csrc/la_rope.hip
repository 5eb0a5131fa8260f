// Rotary position embedding of a step's queries and keys at the positions the step's tokens hold
// (the digits of Fig. 2(b): current token 0, lookahead token of level l and column j at 1 + l + j,
// candidate token k at 1 + k; Sec. 3.1 and 3.3), in place and in one launch for both tensors (or
// for the keys alone).
//
// One workgroup per step row.  A work item is eight pairs of one head: two 16-byte vectors of the
// row (pieces c and c + d/16 when pair i is (x[i], x[i + d/2]); pieces 2c and 2c + 1 when it is
// (x[2i], x[2i + 1])) and eight cosines and sines of the row's position.  Arithmetic in fp32,
// one rounding to bf16.  The pass is bound by its launch: 2 MB at the 7B shape.
#include "la_internal.h"
#include "la_rope_common.h"

namespace la {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct RopeParams {
    __bf16* q;
    __bf16* step_k;
    const float* cos;
    const float* sin;
    int P, W, n1, G, heads, kv_heads, head_dim, interleaved;
};

// Relative position of step row r (row order of include/la.h).
__device__ __forceinline__ int row_position(int r, int W, int n1)
{
    if (r == 0) return 0;
    const int look = W * n1;
    if (r <= look) {
        const int l = (r - 1) / W, j = (r - 1) - l * W;
        return 1 + l + j;
    }
    return 1 + (r - 1 - look) % n1;
}

__global__ __launch_bounds__(256) void step_rope_kernel(RopeParams p)
{
    const int r = blockIdx.x;
    const int half = p.head_dim / 2;
    const int items_per_head = p.head_dim / 16;
    const int t = p.P + row_position(r, p.W, p.n1);
    const float* cs = p.cos + (size_t)t * half;
    const float* sn = p.sin + (size_t)t * half;
    const int n_items = (p.heads + p.kv_heads) * items_per_head;
    for (int x = threadIdx.x; x < n_items; x += blockDim.x) {
        const int h = x / items_per_head, c = x - h * items_per_head;
        __bf16* row = h < p.heads ? p.q + ((size_t)r * p.heads + h) * p.head_dim
                                  : p.step_k + ((size_t)r * p.kv_heads + (h - p.heads)) * p.head_dim;
        bf16x8* va = reinterpret_cast<bf16x8*>(row) + (p.interleaved ? 2 * c : c);
        bf16x8* vb = reinterpret_cast<bf16x8*>(row) + (p.interleaved ? 2 * c + 1 : c + items_per_head);
        const bf16x8 xa = *va, xb = *vb;
        const float4 c0 = *reinterpret_cast<const float4*>(cs + c * 8), c1 = *reinterpret_cast<const float4*>(cs + c * 8 + 4);
        const float4 s0 = *reinterpret_cast<const float4*>(sn + c * 8), s1 = *reinterpret_cast<const float4*>(sn + c * 8 + 4);
        const float co[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        const float si[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        bf16x8 ya, yb;
        rope_eight_pairs(xa, xb, co, si, p.interleaved != 0, ya, yb);
        *va = ya;
        *vb = yb;
    }
}

}  // namespace

la_status launch_step_rope(void* q, void* step_k, const float* cos, const float* sin, int P, int W, int N, int G,
                           int heads, int kv_heads, int head_dim, int interleaved, hipStream_t stream)
{
    RopeParams p;
    p.q = (__bf16*)q;
    p.step_k = (__bf16*)step_k;
    p.cos = cos;
    p.sin = sin;
    p.P = P; p.W = W; p.n1 = N - 1; p.G = G;
    p.heads = q ? heads : 0;  // no q: the keys alone (the attention kernel can rotate its queries itself)
    p.kv_heads = kv_heads; p.head_dim = head_dim; p.interleaved = interleaved;
    const int T = 1 + (W + G) * (N - 1);
    hipLaunchKernelGGL(step_rope_kernel, dim3((unsigned)T), dim3(256), 0, stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_EHIP, "la_step_rope launch: %s", hipGetErrorString(e));
    return LA_OK;
}

}  // namespace la

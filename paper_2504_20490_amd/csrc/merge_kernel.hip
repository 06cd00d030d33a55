// Merge of two partial attention results of the same rows over disjoint key sets (one step of the ring of
// context-parallel attention): LSE = ln(exp(LSE_a) + exp(LSE_b)), O = exp(LSE_a - LSE) O_a + exp(LSE_b - LSE) O_b.
// A partial result whose LSE is -inf (no visible key) is the neutral element.  Pure HBM stream: every thread
// moves 16 bytes of each operand.
#include "attn_device.hpp"
#include "kernels.hpp"

namespace hspmd {

template <int D>
__global__ __launch_bounds__(kThreads) void merge_kernel(MergeParams p) {
    constexpr int LANES = D / 4;                 // threads per (token, head) row, 4 floats each
    constexpr int ROWS = kThreads / LANES;
    const int64_t n_rows = p.total_tokens * p.q_heads;
    const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LANES;
    const int c = threadIdx.x % LANES;
    const int hd = p.head_dim;   // floats per row in memory, <= D
    if (row >= n_rows || c * 4 >= hd) return;
    const int64_t t = row / p.q_heads, h = row % p.q_heads;
    const float la = p.lse_a[h * p.total_tokens + t], lb = p.lse_b[h * p.total_tokens + t];
    const float m = fmaxf(la, lb);
    float wa = 0.f, wb = 0.f, lse = -INFINITY;
    if (m != -INFINITY) {
        const float ea = __expf(la - m), eb = __expf(lb - m);   // exp(-inf) = 0
        const float z = ea + eb;                                 // >= 1
        wa = ea / z;
        wb = eb / z;
        lse = m + __logf(z);
    }
    const f32x4 a = *reinterpret_cast<const f32x4*>(p.o_a + row * hd + c * 4);
    const f32x4 b = *reinterpret_cast<const f32x4*>(p.o_b + row * hd + c * 4);
    f32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = wa * a[j] + wb * b[j];
    *reinterpret_cast<f32x4*>(p.o_out + row * hd + c * 4) = o;
    if (p.o_out_bf16) {
        u32x2 w;
        w[0] = pack_bf16(o[0], o[1]);
        w[1] = pack_bf16(o[2], o[3]);
        *reinterpret_cast<u32x2*>(p.o_out_bf16 + row * hd + c * 4) = w;
    }
    if (c == 0) p.lse_out[h * p.total_tokens + t] = lse;
}

hipError_t launch_merge(const MergeParams& p, hipStream_t stream) {
    const int64_t n_rows = p.total_tokens * p.q_heads;
    if (n_rows == 0) return hipSuccess;
    const int rows_per_block = kThreads / (tile_width(p.head_dim) / 4);
    const dim3 grid((unsigned)((n_rows + rows_per_block - 1) / rows_per_block)), threads(kThreads);
    if (tile_width(p.head_dim) == 128) {
        hipLaunchKernelGGL(merge_kernel<128>, grid, threads, 0, stream, p);
    } else {
        hipLaunchKernelGGL(merge_kernel<64>, grid, threads, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

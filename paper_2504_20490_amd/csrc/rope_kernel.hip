// Rotary position embedding of the q and k of a pack (model configuration table of the paper: position encoding
// RoPE), and the table of cos / sin values that this kernel and the backward epilogues read.
//
// Pairing: column i with column i + head_dim/2 ("rotate-half"); a token at position p of its sequence turns the
// pair by p * theta_i, theta_i = base^(-2i/head_dim).  HBM-bound: every q and k element is read once and written
// once; the table row of a position is shared by all heads and stays in L2.
#include "attn_device.hpp"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

namespace {

constexpr int kRopeThreads = 256;

// table[p][i] = (cos(p theta_i), sin(p theta_i)), evaluated in fp64 and rounded once
__global__ __launch_bounds__(kRopeThreads) void rope_table_kernel(float* table, int64_t entries, int half, int head_dim,
                                                                  double base) {
    const int64_t e = (int64_t)blockIdx.x * kRopeThreads + threadIdx.x;
    if (e >= entries) return;
    const int64_t pos = e / half;
    const int i = (int)(e % half);
    const double theta = pow(base, -2.0 * (double)i / (double)head_dim);
    double s, c;
    sincos((double)pos * theta, &s, &c);
    *reinterpret_cast<float2*>(table + 2 * e) = make_float2((float)c, (float)s);
}

// VEC consecutive columns of the low half and their partners of the high half, one token, one head
template <int VEC>
__device__ __forceinline__ void rotate_piece(const uint16_t* src, uint16_t* dst, int half, const float* cs, float sin_sign) {
    using Raw = typename std::conditional<VEC == 8, u32x4, u32x2>::type;
    const Raw lo = *reinterpret_cast<const Raw*>(src);
    const Raw hi = *reinterpret_cast<const Raw*>(src + half);
    f32x4 t[VEC / 2];
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j) t[j] = *reinterpret_cast<const f32x4*>(cs + 4 * j);   // (cos, sin) of two columns
    Raw out_lo, out_hi;
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j) {
        float y_lo[2], y_hi[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            // bf16 -> fp32 is a shift into the high half of the word
            const float a = __uint_as_float(e == 0 ? lo[j] << 16 : lo[j] & 0xffff0000u);
            const float b = __uint_as_float(e == 0 ? hi[j] << 16 : hi[j] & 0xffff0000u);
            const float c = t[j][2 * e], s = t[j][2 * e + 1] * sin_sign;
            y_lo[e] = a * c - b * s;
            y_hi[e] = b * c + a * s;
        }
        out_lo[j] = pack_bf16(y_lo[0], y_lo[1]);
        out_hi[j] = pack_bf16(y_hi[0], y_hi[1]);
    }
    *reinterpret_cast<Raw*>(dst) = out_lo;
    *reinterpret_cast<Raw*>(dst + half) = out_hi;
}

// e / n and e % n for 0 <= e < 2^22 and 0 < n through a float reciprocal (the +0.5 keeps the quotient at least
// 0.5 / n away from an integer, far more than the rounding error of the product)
__device__ __forceinline__ void divmod(int e, int n, float inv_n, int& quot, int& rem) {
    quot = (int)(((float)e + 0.5f) * inv_n);
    rem = e - quot * n;
}

// rows r_begin .. r_end-1 (counted from token0, which sits at position pos0 of its sequence) of a [tokens, heads,
// head_dim] tensor, all heads: consecutive lanes walk along the contiguous token rows (16 or 8 bytes of the low
// half of a head and as many of its high half per lane).  In place is fine: a thread reads what it writes.
template <int VEC>
__device__ __forceinline__ void rotate_rows(const uint16_t* src, uint16_t* dst, int64_t stride, int64_t out_stride,
                                            int64_t token0, int pos0, int r_begin, int r_end, int heads, int hd,
                                            const float* table, float sin_sign) {
    const int half = hd / 2, pieces = half / VEC;   // pieces per head
    const int per_row = heads * pieces;
    const float inv_per_row = 1.f / (float)per_row, inv_pieces = 1.f / (float)pieces;
    for (int e = threadIdx.x; e < (r_end - r_begin) * per_row; e += kRopeThreads) {
        int r, x, head, piece;
        divmod(e, per_row, inv_per_row, r, x);
        divmod(x, pieces, inv_pieces, head, piece);
        r += r_begin;
        const int c = piece * VEC;
        rotate_piece<VEC>(src + (token0 + r) * stride + head * hd + c, dst + (token0 + r) * out_stride + head * hd + c, half,
                          table + ((int64_t)(pos0 + r) * half + c) * 2, sin_sign);
    }
}

// Packed plans: one workgroup per item of the forward list.  The items (tile, head) of one tile exist once per q
// head, so the workgroup of head h takes the h-th share of the tile's rows and rotates ALL heads of those rows,
// of q and of k.
template <int VEC>
__global__ __launch_bounds__(kRopeThreads) void rope_qk_kernel(RopeParams p) {
    const hspmd_work_item item = p.items[blockIdx.x];
    if (item.tile < 0) return;   // padding slot
    const int row0 = item.tile * kFwdQTile;
    const int rows = min(kFwdQTile, item.seq_len - row0);
    const int r_begin = rows * item.head / p.q_heads, r_end = rows * (item.head + 1) / p.q_heads;
    const int64_t token0 = (int64_t)item.token_start + row0;
    rotate_rows<VEC>(p.q, p.q_out, p.q_stride, p.q_out_stride, token0, row0, r_begin, r_end, p.q_heads, p.head_dim, p.table,
                     p.sin_sign);
    rotate_rows<VEC>(p.k, p.k_out, p.kv_stride, p.kv_out_stride, token0, row0, r_begin, r_end, p.q_heads / p.group,
                     p.head_dim, p.table, p.sin_sign);
}

// Block plans: the query chunks are walked through the forward list (items (q tile, q head)), the key chunks through
// the dK/dV list (items (k tile, kv head)); positions are those of the chunks inside their sequences.
template <int VEC, bool KEYS>
__global__ __launch_bounds__(kRopeThreads) void rope_block_kernel(RopeParams p) {
    const hspmd_block_item item = p.block_items[blockIdx.x];
    if (item.tile < 0) return;   // padding slot
    const int tile_rows = KEYS ? kDkvKTile : kFwdQTile;
    const int heads = KEYS ? p.q_heads / p.group : p.q_heads;
    const int len = KEYS ? item.k_len : item.q_len;
    const int row0 = item.tile * tile_rows;
    const int rows = min(tile_rows, len - row0);
    if (rows <= 0) return;
    const int r_begin = rows * item.head / heads, r_end = rows * (item.head + 1) / heads;
    if constexpr (KEYS)
        rotate_rows<VEC>(p.k, p.k_out, p.kv_stride, p.kv_out_stride, (int64_t)item.k_start + row0,
                         item.q_pos - item.offset + row0, r_begin, r_end, heads, p.head_dim, p.table, p.sin_sign);
    else
        rotate_rows<VEC>(p.q, p.q_out, p.q_stride, p.q_out_stride, (int64_t)item.q_start + row0, item.q_pos + row0, r_begin,
                         r_end, heads, p.head_dim, p.table, p.sin_sign);
}

}  // namespace

hipError_t launch_rope_table(float* table, int32_t positions, int32_t head_dim, double base, hipStream_t stream) {
    const int64_t entries = (int64_t)positions * (head_dim / 2);
    if (entries == 0) return hipSuccess;
    const dim3 grid((unsigned)((entries + kRopeThreads - 1) / kRopeThreads)), threads(kRopeThreads);
    hipLaunchKernelGGL(rope_table_kernel, grid, threads, 0, stream, table, entries, head_dim / 2, head_dim, base);
    return hipGetLastError();
}

hipError_t launch_rope_qk(const RopeParams& p, int64_t num_items, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), threads(kRopeThreads);
    // 16-byte pieces when half a head is a whole number of them, 8-byte pieces otherwise (head_dim is a multiple of 8)
    if ((p.head_dim / 2) % 8 == 0) hipLaunchKernelGGL(rope_qk_kernel<8>, grid, threads, 0, stream, p);
    else hipLaunchKernelGGL(rope_qk_kernel<4>, grid, threads, 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_rope_block(const RopeParams& p, int64_t num_items, bool keys, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), threads(kRopeThreads);
    const bool wide = (p.head_dim / 2) % 8 == 0;
    if (keys) {
        if (wide) hipLaunchKernelGGL((rope_block_kernel<8, true>), grid, threads, 0, stream, p);
        else hipLaunchKernelGGL((rope_block_kernel<4, true>), grid, threads, 0, stream, p);
    } else {
        if (wide) hipLaunchKernelGGL((rope_block_kernel<8, false>), grid, threads, 0, stream, p);
        else hipLaunchKernelGGL((rope_block_kernel<4, false>), grid, threads, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

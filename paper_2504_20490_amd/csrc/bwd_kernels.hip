// Backward kernels.  Both passes recompute P = exp(S - LSE) from the forward's logsumexp.
//
//   D pass    : D[h, t] = sum_c dO[t,h,c] * O[t,h,c]; also LSE * log2(e) and a +inf constant that
//               the dK/dV pass copies into LDS for rows past a sequence's end      (HBM stream)
//   dQ pass   : one workgroup per (sequence, 128-row q tile, q head); loops over 64-key tiles of
//               the causal prefix; per wave (32 queries along MFMA columns):
//                 S^T = K Q^T, dP^T = V dO^T, dS^T = P^T (dP^T - D), dQ^T += K^T dS^T
//   dK/dV pass: bwd_dkv_kernel.hip
// In every product the operand that changes per step comes from a row-major LDS tile, read
// either along its rows or with the transpose read; the wave's own rows stay in registers.
#include <type_traits>

#include "attn_device.hpp"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

// ---------------------------------------------------------------------------------- D pass
template <int D>
__global__ __launch_bounds__(kThreads) void bwd_dsum_kernel(BwdParams p) {
    constexpr int LANES = D / 8;                 // lanes per (token, head) row, 16 B each
    constexpr int ROWS = kThreads / LANES;
    const int64_t n_rows = p.total_tokens * p.q_heads;
    const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LANES;
    const int c = threadIdx.x % LANES;
    float s = 0.f;
    if (row < n_rows) {
        union { u32x4 u; bf16x8 v; } a, b;
        a.u = *reinterpret_cast<const u32x4*>(p.o + row * D + c * 8);
        b.u = *reinterpret_cast<const u32x4*>(p.d_o + row * D + c * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) s += (float)a.v[i] * (float)b.v[i];
    }
#pragma unroll
    for (int off = LANES / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row < n_rows && c == 0) {
        const int64_t t = row / p.q_heads, h = row % p.q_heads;
        p.dsum[h * p.total_tokens + t] = s;
        p.lse2[h * p.total_tokens + t] = p.lse[h * p.total_tokens + t] * kLog2e;
    }
    if (blockIdx.x == 0 && threadIdx.x < 16) p.inf_pad[threadIdx.x] = INFINITY;
}

// --------------------------------------------------------------------------------- dQ pass
template <int D>
__global__ __launch_bounds__(kThreads, 2) void bwd_dq_kernel(BwdParams p) {
    constexpr int BQ = kFwdQTile, BK = kFwdKTile;
    constexpr int KK = D / 16, DB = D / 32;
    constexpr int kTileBytes = BK * D * 2;
    __shared__ __attribute__((aligned(1024))) char lds[2 * 2 * kTileBytes];   // {K, V} x 2 stages

    const hspmd_work_item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = item.seq_len, h = item.head, hk = h / p.group;
    const int q_row0 = item.tile * BQ;
    const int wave_row0 = q_row0 + wave * 32;
    const int my_row = wave_row0 + (lane & 31);
    const int hh = lane >> 5;
    const bool valid = my_row < L;

    const uint16_t* qbase = p.q + (int64_t)item.token_start * p.q_stride + (int64_t)h * D;
    const uint16_t* dobase = p.d_o + ((int64_t)item.token_start * p.q_heads + h) * D;
    const uint16_t* kbase = p.k + (int64_t)item.token_start * p.kv_stride + (int64_t)hk * D;
    const uint16_t* vbase = p.v + (int64_t)item.token_start * p.kv_stride + (int64_t)hk * D;

    const int kv_end = min(L, q_row0 + BQ);
    const int n_tiles = (kv_end + BK - 1) / BK;

    TileCopy<D, BK> kvcopy;   // K and V share stride and geometry
    kvcopy.init(p.kv_stride, wave, lane);
    kvcopy.issue(lds, kbase, p.kv_stride, 0, L, wave, lane);
    kvcopy.issue(lds + kTileBytes, vbase, p.kv_stride, 0, L, wave, lane);

    bf16x8 qf[KK], dof[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        union { u32x4 u; bf16x8 v; } a, b;
        a.u = u32x4{0u, 0u, 0u, 0u};
        b.u = u32x4{0u, 0u, 0u, 0u};
        if (valid) {
            a.u = *reinterpret_cast<const u32x4*>(qbase + (int64_t)my_row * p.q_stride + kk * 16 + hh * 8);
            b.u = *reinterpret_cast<const u32x4*>(dobase + (int64_t)my_row * p.q_heads * D + kk * 16 + hh * 8);
        }
        qf[kk] = a.v;
        dof[kk] = b.v;
    }
    const int64_t stat = (int64_t)h * p.total_tokens + item.token_start + my_row;
    const float lse2 = valid ? p.lse2[stat] : INFINITY;   // rows past the end get P = 0
    const float dsum = valid ? p.dsum[stat] : 0.f;
    const float c = p.scale_log2;

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

    // One key tile.  MASK = false: every key of the tile precedes every row of this q tile (no compare, no
    // skipped block); MASK = true: the tile touches the diagonal.
    auto step = [&](int kt, auto masked) {
        constexpr bool kMask = decltype(masked)::value;
        wait_tile_loads();
        __syncthreads();   // tile kt has landed; every wave is done with the other stage
        const char* ktile = lds + (kt & 1) * (2 * kTileBytes);
        const char* vtile = ktile + kTileBytes;
        if (kt + 1 < n_tiles) {
            char* next = lds + ((kt + 1) & 1) * (2 * kTileBytes);
            kvcopy.issue(next, kbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
            kvcopy.issue(next + kTileBytes, vbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
        }
        const int key0 = kt * BK;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int kb = key0 + jb * 32;
            if (!kMask || kb <= wave_row0 + 31) {           // otherwise every key of the block is masked for this wave
                f32x16 s, dp;
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
                {
                    bf16x8 kf[KK];
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) kf[kk] = read_rowmajor_frag<D>(ktile, jb, kk, lane);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) s = mfma(kf[kk], qf[kk], s);
                }
                {
                    bf16x8 vf[KK];
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) vf[kk] = read_rowmajor_frag<D>(vtile, jb, kk, lane);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) dp = mfma(vf[kk], dof[kk], dp);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float pr = fast_exp2(fmaf(s[i], c, -lse2));
                    if (kMask && kb + acc_row(i, lane) > my_row) pr = 0.f;
                    s[i] = pr * (dp[i] - dsum);   // dS^T
                }
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const bf16x8 dsf = frag_to_bf16(s, tt);
                    bf16x8 ktf[DB];
#pragma unroll
                    for (int db = 0; db < DB; ++db) ktf[db] = read_transposed_frag<D>(ktile, db, jb * 2 + tt, lane);
#pragma unroll
                    for (int db = 0; db < DB; ++db) acc[db] = mfma(ktf[db], dsf, acc[db]);
                }
            }
        }
    };
    // two loops instead of a test per tile: the tiles wholly below the diagonal, then the (at most two) on it
    const int n_interior = min(n_tiles, 2 * item.tile);
    int kt = 0;
    for (; kt < n_interior; ++kt) step(kt, std::false_type{});
    for (; kt < n_tiles; ++kt) step(kt, std::true_type{});

    if (valid) {
        const int64_t row_elem = ((int64_t)(item.token_start + my_row) * p.q_heads + h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4)
                store_grad4(p.dq, row_elem + db * 32 + i4 * 8 + hh * 4, p.grad_f32 != 0,
                            acc[db][4 * i4 + 0] * p.scale, acc[db][4 * i4 + 1] * p.scale,
                            acc[db][4 * i4 + 2] * p.scale, acc[db][4 * i4 + 3] * p.scale);
    }
}

// ------------------------------------------------------------------------------- launchers
hipError_t launch_bwd_dsum(const BwdParams& p, int head_dim, hipStream_t stream) {
    const int64_t n_rows = p.total_tokens * p.q_heads;
    if (n_rows == 0) return hipSuccess;
    const int rows_per_block = kThreads / (head_dim / 8);
    const dim3 grid((unsigned)((n_rows + rows_per_block - 1) / rows_per_block)), block(kThreads);
    if (head_dim == 128) {
        hipLaunchKernelGGL(bwd_dsum_kernel<128>, grid, block, 0, stream, p);
    } else {
        hipLaunchKernelGGL(bwd_dsum_kernel<64>, grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_bwd_dq(const BwdParams& p, int head_dim, int64_t num_items, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kThreads);
    if (head_dim == 128) {
        hipLaunchKernelGGL(bwd_dq_kernel<128>, grid, block, 0, stream, p);
    } else {
        hipLaunchKernelGGL(bwd_dq_kernel<64>, grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

// Backward kernels.  Both passes recompute P = exp(S - LSE) from the forward's logsumexp.
//
//   D pass    : D[h, t] = sum_c dO[t,h,c] * O[t,h,c]                       (HBM stream)
//   dQ pass   : one workgroup per (sequence, 128-row q tile, q head); loops over 64-key tiles of
//               the causal prefix; per wave (32 queries along MFMA columns):
//                 S^T = K Q^T, dP^T = V dO^T, dS^T = P^T (dP^T - D), dQ^T += K^T dS^T
//   dK/dV pass: one workgroup per (sequence, 128-key tile, kv head); loops over the query heads of
//               the KV group and over 64-row q tiles at or below the diagonal; per wave (32 keys
//               along MFMA columns):
//                 S = Q K^T, dP = dO V^T, dS = P (dP - D), dV^T += dO^T P, dK^T += Q^T dS
//               The group loop runs inside the workgroup, so dK/dV need no atomics.
// In every product the operand that changes per step comes from a row-major LDS tile, read
// either along its rows or with the transpose read; the wave's own rows stay in registers.
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
    }
}

// writes 4 consecutive gradient elements of one row (bf16 or fp32)
__device__ __forceinline__ void store_grad4(void* base, int64_t elem, bool f32, float a, float b, float c, float d) {
    if (f32) {
        *reinterpret_cast<f32x4*>(static_cast<float*>(base) + elem) = f32x4{a, b, c, d};
    } else {
        u32x2 w;
        w[0] = pack_bf16(a, b);
        w[1] = pack_bf16(c, d);
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(base) + elem) = w;
    }
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

    tile_load_async<D, BK>(lds, kbase, p.kv_stride, 0, L, wave, lane);
    tile_load_async<D, BK>(lds + kTileBytes, vbase, p.kv_stride, 0, L, wave, lane);

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
    const float lse2 = valid ? p.lse[stat] * kLog2e : INFINITY;   // rows past the end get P = 0
    const float dsum = valid ? p.dsum[stat] : 0.f;
    const float c = p.scale_log2;

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

    for (int kt = 0; kt < n_tiles; ++kt) {
        wait_tile_loads();
        __syncthreads();   // tile kt has landed; every wave is done with the other stage
        const char* ktile = lds + (kt & 1) * (2 * kTileBytes);
        const char* vtile = ktile + kTileBytes;
        if (kt + 1 < n_tiles) {
            char* next = lds + ((kt + 1) & 1) * (2 * kTileBytes);
            tile_load_async<D, BK>(next, kbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
            tile_load_async<D, BK>(next + kTileBytes, vbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
        }
        const int key0 = kt * BK;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int kb = key0 + jb * 32;
            if (kb <= wave_row0 + 31) {           // otherwise every key of the block is masked for this wave
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
                const bool diag = kb + 31 > wave_row0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float pr = fast_exp2(fmaf(s[i], c, -lse2));
                    if (diag && kb + acc_row(i, lane) > my_row) pr = 0.f;
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
    }

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

// ------------------------------------------------------------------------------ dK/dV pass
template <int D>
__global__ __launch_bounds__(kThreads, 1) void bwd_dkv_kernel(BwdParams p) {
    constexpr int BKV = kDkvKTile, BQ = kDkvQTile;
    constexpr int KK = D / 16, DB = D / 32;
    constexpr int kTileBytes = BQ * D * 2;
    constexpr int kStatBytes = 1024;                           // lse2[BQ], dsum[BQ] (fp32), padded
    constexpr int kStageBytes = 2 * kTileBytes + kStatBytes;   // Q, dO, statistics
    __shared__ __attribute__((aligned(1024))) char lds[2 * kStageBytes];

    const hspmd_work_item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = item.seq_len, g = item.head;
    const int key0 = item.tile * BKV;
    const int wave_key0 = key0 + wave * 32;
    const int my_key = wave_key0 + (lane & 31);
    const int hh = lane >> 5;
    const bool valid = my_key < L;

    const uint16_t* kbase = p.k + (int64_t)item.token_start * p.kv_stride + (int64_t)g * D;
    const uint16_t* vbase = p.v + (int64_t)item.token_start * p.kv_stride + (int64_t)g * D;

    // steps: for each head of the group, q tiles first_qt .. n_qt-1 (rows at or below the diagonal)
    const int first_qt = key0 / BQ;
    const int n_qt = (L + BQ - 1) / BQ;
    const int per_head = n_qt - first_qt;
    const int n_steps = per_head * p.group;

    float st_lse = 0.f, st_dsum = 0.f;   // threads 0..BQ-1 carry one row's statistics of the next step
    auto load_step = [&](int step, char* stage) {
        const int hq = g * p.group + step / per_head;
        const int row0 = (first_qt + step % per_head) * BQ;
        const uint16_t* qb = p.q + (int64_t)item.token_start * p.q_stride + (int64_t)hq * D;
        const uint16_t* dob = p.d_o + ((int64_t)item.token_start * p.q_heads + hq) * D;
        tile_load_async<D, BQ>(stage, qb, p.q_stride, row0, L, wave, lane);
        tile_load_async<D, BQ>(stage + kTileBytes, dob, (int64_t)p.q_heads * D, row0, L, wave, lane);
        if (tid < BQ) {
            const int r = row0 + tid;
            const int64_t stat = (int64_t)hq * p.total_tokens + item.token_start + r;
            st_lse = r < L ? p.lse[stat] * kLog2e : INFINITY;   // rows past the end: P = exp2(-inf) = 0
            st_dsum = r < L ? p.dsum[stat] : 0.f;
        }
    };
    auto store_stats = [&](char* stage) {
        if (tid < BQ) {
            reinterpret_cast<float*>(stage + 2 * kTileBytes)[tid] = st_lse;
            reinterpret_cast<float*>(stage + 2 * kTileBytes + BQ * 4)[tid] = st_dsum;
        }
    };

    if (n_steps > 0) {
        load_step(0, lds);
        store_stats(lds);
    }

    bf16x8 kf[KK], vf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        union { u32x4 u; bf16x8 v; } a, b;
        a.u = u32x4{0u, 0u, 0u, 0u};
        b.u = u32x4{0u, 0u, 0u, 0u};
        if (valid) {
            a.u = *reinterpret_cast<const u32x4*>(kbase + (int64_t)my_key * p.kv_stride + kk * 16 + hh * 8);
            b.u = *reinterpret_cast<const u32x4*>(vbase + (int64_t)my_key * p.kv_stride + kk * 16 + hh * 8);
        }
        kf[kk] = a.v;
        vf[kk] = b.v;
    }
    const float c = p.scale_log2;

    f32x16 dk[DB], dv[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk[db][i] = 0.f; dv[db][i] = 0.f; }

    for (int step = 0; step < n_steps; ++step) {
        wait_tile_loads();
        __syncthreads();   // this step's tiles and statistics are in LDS; the other stage is free
        const char* stage = lds + (step & 1) * kStageBytes;
        const char* qtile = stage;
        const char* dotile = stage + kTileBytes;
        const float* lse_s = reinterpret_cast<const float*>(stage + 2 * kTileBytes);
        const float* dsum_s = lse_s + BQ;
        const bool more = step + 1 < n_steps;
        char* next = lds + ((step + 1) & 1) * kStageBytes;
        if (more) load_step(step + 1, next);
        const int row0 = (first_qt + step % per_head) * BQ;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int qb0 = row0 + rb * 32;
            if (qb0 + 31 >= wave_key0) {          // otherwise every query of the block precedes every key
                f32x16 s, dp;
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
                {
                    bf16x8 qf[KK];
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) qf[kk] = read_rowmajor_frag<D>(qtile, rb, kk, lane);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) s = mfma(qf[kk], kf[kk], s);
                }
                {
                    bf16x8 dof[KK];
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) dof[kk] = read_rowmajor_frag<D>(dotile, rb, kk, lane);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) dp = mfma(dof[kk], vf[kk], dp);
                }
                const bool diag = qb0 < wave_key0 + 31;
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int rloc = rb * 32 + i4 * 8 + hh * 4;
                    const f32x4 lse4 = *reinterpret_cast<const f32x4*>(lse_s + rloc);
                    const f32x4 ds4 = *reinterpret_cast<const f32x4*>(dsum_s + rloc);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = i4 * 4 + e;
                        float pr = fast_exp2(fmaf(s[i], c, -lse4[e]));
                        if (diag && row0 + rloc + e < my_key) pr = 0.f;
                        s[i] = pr;                         // P
                        dp[i] = pr * (dp[i] - ds4[e]);     // dS
                    }
                }
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const bf16x8 pf = frag_to_bf16(s, tt);
                    const bf16x8 dsf = frag_to_bf16(dp, tt);
                    bf16x8 dotf[DB], qtf[DB];
#pragma unroll
                    for (int db = 0; db < DB; ++db) dotf[db] = read_transposed_frag<D>(dotile, db, rb * 2 + tt, lane);
#pragma unroll
                    for (int db = 0; db < DB; ++db) qtf[db] = read_transposed_frag<D>(qtile, db, rb * 2 + tt, lane);
#pragma unroll
                    for (int db = 0; db < DB; ++db) dv[db] = mfma(dotf[db], pf, dv[db]);
#pragma unroll
                    for (int db = 0; db < DB; ++db) dk[db] = mfma(qtf[db], dsf, dk[db]);
                }
            }
        }
        if (more) store_stats(next);
    }

    if (valid) {
        const int64_t row_elem = ((int64_t)(item.token_start + my_key) * p.kv_heads + g) * D;
        const bool f32 = p.grad_f32 != 0;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int64_t e = row_elem + db * 32 + i4 * 8 + hh * 4;
                store_grad4(p.dk, e, f32, dk[db][4 * i4 + 0] * p.scale, dk[db][4 * i4 + 1] * p.scale,
                            dk[db][4 * i4 + 2] * p.scale, dk[db][4 * i4 + 3] * p.scale);
                store_grad4(p.dv, e, f32, dv[db][4 * i4 + 0], dv[db][4 * i4 + 1], dv[db][4 * i4 + 2], dv[db][4 * i4 + 3]);
            }
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

hipError_t launch_bwd_dkv(const BwdParams& p, int head_dim, int64_t num_items, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kThreads);
    if (head_dim == 128) {
        hipLaunchKernelGGL(bwd_dkv_kernel<128>, grid, block, 0, stream, p);
    } else {
        hipLaunchKernelGGL(bwd_dkv_kernel<64>, grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

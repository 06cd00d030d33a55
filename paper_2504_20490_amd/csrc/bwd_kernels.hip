// Backward kernels.  Both passes recompute P = exp(S - LSE) from the forward's logsumexp.
//
//   D pass    : -D[h, t] = -sum_c dO[t,h,c] * O[t,h,c]; also -LSE / scale (the logsumexp in units of raw
//               scores) and a -inf constant that the dK/dV pass copies into LDS for rows past a
//               sequence's end.  Both statistics are stored negated because the dK/dV pass feeds
//               them to the MFMA as the initial accumulator: S - LSE/scale and dP - D come out of
//               the matrix core                                                     (HBM stream)
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
    const int hd = p.head_dim;   // elements per row in memory, <= D
    float s = 0.f;
    if (row < n_rows && c * 8 < hd) {
        union { u32x4 u; bf16x8 v; } a, b;
        a.u = *reinterpret_cast<const u32x4*>(p.o + row * hd + c * 8);
        b.u = *reinterpret_cast<const u32x4*>(p.d_o + row * hd + c * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) s += (float)a.v[i] * (float)b.v[i];
    }
#pragma unroll
    for (int off = LANES / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row < n_rows && c == 0) {
        const int64_t t = row / p.q_heads, h = row % p.q_heads;
        p.negd[h * p.total_tokens + t] = -s;
        // a row without any visible key (lse = -inf; possible only for partial results) takes no part: P = 0
        const float l = p.lse[h * p.total_tokens + t];
        p.nlse[h * p.total_tokens + t] = l == -INFINITY ? -INFINITY : -l / p.scale;
    }
    if (blockIdx.x == 0 && threadIdx.x < 16) p.ninf_pad[threadIdx.x] = -INFINITY;
}

// --------------------------------------------------------------------------------- dQ pass
// KD: 16-column steps of the contractions over head_dim (S^T = K Q^T, dP^T = V dO^T) that hold data: D / 16, or fewer
// when head_dim ends before the tile width (the steps beyond it would multiply the zero padding of the Q / dO fragments)
template <int D, bool BLOCK, int KD = D / 16>
__global__ __launch_bounds__(kThreads, 2) void bwd_dq_kernel(BwdParams p) {
    static_assert(KD >= 1 && KD <= D / 16, "k-steps inside the tile width");
    constexpr int BQ = kFwdQTile, BK = kFwdKTile;
    constexpr int KK = KD, DB = D / 32;
    constexpr int kTileBytes = BK * D * 2;
    __shared__ __attribute__((aligned(1024))) char lds[2 * 2 * kTileBytes];   // {K, V} x 2 stages

    // packed variant: this pass also produces the row statistics (see below); the constants that go with them
    if (!BLOCK && blockIdx.x == 0 && threadIdx.x < 16) p.ninf_pad[threadIdx.x] = -INFINITY;
    const ItemGeom item = load_item<BLOCK>(p.items, p.block_items, blockIdx.x);
    if (item.tile < 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Lq = item.q_len, L = item.k_len, off = item.offset;   // L: keys of the chunk (= rows when !BLOCK)
    const int h = item.head, hk = h / p.group;
    const int q_row0 = item.tile * BQ;
    const int wave_row0 = q_row0 + wave * 32;
    const int my_row = wave_row0 + (lane & 31);
    const int hh = lane >> 5;
    const bool valid = my_row < Lq;
    // last key this lane's row may see (index into the chunk), and the same for the wave's last row
    const int my_limit = BLOCK ? min(my_row + off, L - 1) : my_row;
    const int wave_limit = BLOCK ? min(wave_row0 + 31 + off, L - 1) : wave_row0 + 31;

    const int hd = p.head_dim;   // elements per head in memory, <= D (columns hd .. D-1 exist only in LDS and registers)
    const uint16_t* qbase = p.q + (int64_t)item.q_start * p.q_stride + (int64_t)h * hd;
    const uint16_t* dobase = p.d_o + ((int64_t)item.q_start * p.q_heads + h) * hd;
    const uint16_t* kbase = p.k + (int64_t)item.k_start * p.kv_stride + (int64_t)hk * hd;
    const uint16_t* vbase = p.v + (int64_t)item.k_start * p.kv_stride + (int64_t)hk * hd;

    // key j is visible to row r iff j <= r + off: the tile's last row sees keys 0 .. kv_end-1
    const int kv_end = max(0, min(L, min(Lq, q_row0 + BQ) + off));
    const int n_tiles = (kv_end + BK - 1) / BK;
    if (BLOCK && n_tiles == 0) {
        // nothing visible: this block's share of dQ is zero
        if (valid && !p.dq_accumulate) {
            float* row = static_cast<float*>(p.dq) + ((int64_t)(item.q_start + my_row) * p.q_heads + h) * hd;
#pragma unroll
            for (int c4 = 0; c4 < D / 8; ++c4)
                if (hh * (D / 2) + c4 * 4 < hd)
                    *reinterpret_cast<f32x4*>(row + hh * (D / 2) + c4 * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        return;
    }

    TileCopy<D, BK> kvcopy;   // K and V share stride and geometry
    kvcopy.init(p.kv_stride, wave, lane, hd);
    const uint32_t lds0 = lds_address(lds);   // copy destinations are LDS byte addresses
    kvcopy.issue(lds0, kbase, p.kv_stride, 0, L, wave, lane);
    kvcopy.issue(lds0 + kTileBytes, vbase, p.kv_stride, 0, L, wave, lane);

    // Q and dO rows of this lane.  The packed variant owns every (row, head) exactly once in this pass, so it
    // also computes the row statistic D = <dO, O> here (no separate pass over O and dO) and leaves -D and
    // -LSE / scale in the workspace for the dK/dV pass that follows on the stream; the block variant reads
    // what bwd_dsum_kernel wrote (the statistics of the merged rows are shared by all blocks of a row).
    bf16x8 qf[KK], dof[KK];
    float d_part = 0.f;
    float stat_a, stat_b = 0.f;   // the row's saved statistics, requested together with its Q / dO / O
    {
        // All loads first, from addresses that exist for every lane (a lane past the end of the chunk reads the tile's
        // first row, a column chunk past head_dim reads the head's last one), the selection afterwards: loads under a
        // per-lane condition end up in one conditional block per step, each waiting for its own data before the
        // next block's loads are issued: eight memory round trips in a row at the start of every item.
        const int lrow = valid ? my_row : q_row0;
        const int64_t lstat = (int64_t)h * p.total_tokens + item.q_start + lrow;
        if constexpr (BLOCK) {
            stat_a = p.nlse[lstat];
            stat_b = p.negd[lstat];
        } else {
            stat_a = p.lse[lstat];
        }
        const uint16_t* qrow = qbase + (int64_t)lrow * p.q_stride;
        const int64_t row_elem = (int64_t)lrow * p.q_heads * hd;
        const uint16_t* dorow = dobase + row_elem;
        const uint16_t* orow = p.o + ((int64_t)item.q_start * p.q_heads + h) * hd + row_elem;
        u32x4 qa[KK], da[KK], oa[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int col = min(kk * 16 + hh * 8, hd - 8);
            qa[kk] = *reinterpret_cast<const u32x4*>(qrow + col);
            da[kk] = *reinterpret_cast<const u32x4*>(dorow + col);
            if constexpr (!BLOCK) oa[kk] = *reinterpret_cast<const u32x4*>(orow + col);
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const bool keep = valid && kk * 16 + hh * 8 < hd;
            union { u32x4 u; bf16x8 v; } a, b;
            a.u = keep ? qa[kk] : u32x4{0u, 0u, 0u, 0u};
            b.u = keep ? da[kk] : u32x4{0u, 0u, 0u, 0u};
            if constexpr (!BLOCK) {
                union { u32x4 u; bf16x8 v; } o;
                o.u = oa[kk];
#pragma unroll
                for (int i = 0; i < 8; ++i) d_part += (float)b.v[i] * (float)o.v[i];   // b = 0 where nothing is kept
            }
            qf[kk] = a.v;
            dof[kk] = b.v;
        }
    }
    const int64_t stat = (int64_t)h * p.total_tokens + item.q_start + my_row;
    const float c = p.scale_log2;
    float nlse2, negd;
    if constexpr (BLOCK) {
        nlse2 = valid ? stat_a * c : -INFINITY;   // -LSE log2(e); rows past the end get P = 0
        negd = valid ? stat_b : 0.f;
    } else {
        negd = -(d_part + partner32(d_part));            // the two half rows of lanes l and l + 32
        const float nlse = valid ? -stat_a / p.scale : -INFINITY;   // rows past the end get P = 0
        nlse2 = nlse * c;                                                // -LSE log2(e)
        if (valid && hh == 0) {
            p.negd[stat] = negd;
            p.nlse[stat] = nlse;
        }
    }

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;
    f32x16 negd_frag;
#pragma unroll
    for (int i = 0; i < 16; ++i) negd_frag[i] = negd;

    // per-lane LDS offsets of the operand fragments inside a tile
    int rm[KK], tr[DB][2];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) rm[kk] = tile_offset<D>(lane & 31, kk * 16 + hh * 8);
    {
        const int c16 = lane & 15;
        const int row = (hh << 2) + (c16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int col = db * 32 + (((lane >> 4) & 1) << 4) + ((c16 & 3) << 2);
            tr[db][0] = tile_offset<D>(row, col);
            tr[db][1] = tile_offset<D>(row + 8, col);
        }
    }

    // One 32-key block, written step by step with a scheduling barrier after each step so that operand
    // fragments are requested kAhead MFMAs before their use:
    //   2 KK steps: S^T = K Q^T then dP^T = V dO^T   (fragments along tile rows)
    //   VALU      : dS^T = exp2(S^T c - LSE log2e) (dP^T - D), with the first K^T fragments already requested
    //   2 DB steps: dQ^T += K^T dS^T                 (fragments by transpose read)
    // MASK: the block touches the diagonal.  SPREAD: step n of the first phase also issues copy instruction
    // n / (2 KK / kPerWave) of a whole tile (K in block 0, V in block 1), see `piece`.
    auto block = [&](const char* ktile, const char* vtile, int jb, int kb, auto masked, auto spread, auto&& piece) {
        constexpr bool kMask = decltype(masked)::value;
        constexpr bool kSpread = decltype(spread)::value;
        constexpr int kAhead = 4, kAheadT = 3;
        constexpr int N1 = 2 * KK, N2 = 2 * DB;
        constexpr int every = N1 / TileCopy<D, BK>::kPerWave;
        auto frag1 = [&](int n) {
            return *reinterpret_cast<const bf16x8*>((n < KK ? ktile : vtile) + rm[n % KK] + jb * 32 * D * 2);
        };
        auto frag2 = [&](int n) {
            const int off = (jb * 2 + n / DB) * 16 * D * 2;
            union { struct { s16x4 a, b; } s; bf16x8 v; } u;
            u.s.a = lds_transpose_read(ktile + tr[n % DB][0] + off);
            u.s.b = lds_transpose_read(ktile + tr[n % DB][1] + off);
            return u.v;
        };
        // dP^T starts from -D (a fragment that holds the lane's -D in every element, kept for the whole item): the
        // matrix core then delivers dP^T - D and the VALU step needs no subtraction
        f32x16 sacc, dp = negd_frag;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
        bf16x8 q1[kAhead + 1];
#pragma unroll
        for (int n = 0; n < kAhead; ++n) q1[n] = frag1(n);
#pragma unroll
        for (int n = 0; n < N1; ++n) {
            if (n + kAhead < N1) q1[(n + kAhead) % (kAhead + 1)] = frag1(n + kAhead);
            if (n < KK) sacc = mfma(q1[n % (kAhead + 1)], qf[n], sacc);
            else dp = mfma(q1[n % (kAhead + 1)], dof[n - KK], dp);
            if constexpr (kSpread) {
                if (n % every == every - 1) piece(jb, n / every);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        bf16x8 q2[kAheadT + 1];
#pragma unroll
        for (int n = 0; n < kAheadT; ++n) q2[n] = frag2(n);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float pr = fast_exp2(fmaf(sacc[i], c, nlse2));
            if (kMask && kb + acc_row(i, lane) > my_limit) pr = 0.f;
            sacc[i] = pr * dp[i];   // dS^T = P (dP^T - D)
        }
        const bf16x8 dsf[2] = {frag_to_bf16(sacc, 0), frag_to_bf16(sacc, 1)};
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < N2; ++n) {
            if (n + kAheadT < N2) q2[(n + kAheadT) % (kAheadT + 1)] = frag2(n + kAheadT);
            acc[n % DB] = mfma(q2[n % (kAheadT + 1)], dsf[n / DB], acc[n % DB]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One key tile of the general kind: copies of the next tile issued at the top, blocks that lie wholly
    // above the diagonal for this wave skipped.
    auto step = [&](int kt, auto masked) {
        constexpr bool kMask = decltype(masked)::value;
        wait_tile_loads();
        __syncthreads();   // tile kt has landed; every wave is done with the other stage
        const char* ktile = lds + (kt & 1) * (2 * kTileBytes);
        const char* vtile = ktile + kTileBytes;
        if (kt + 1 < n_tiles) {
            const uint32_t next = lds0 + ((kt + 1) & 1) * (2 * kTileBytes);
            kvcopy.issue(next, kbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
            kvcopy.issue(next + kTileBytes, vbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
        }
        auto none = [](int, int) {};
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int kb = kt * BK + jb * 32;
            if (!kMask || kb <= wave_limit) block(ktile, vtile, jb, kb, masked, std::false_type{}, none);
        }
    };
    // An unmasked tile whose successor is a whole tile: the successor's copies are issued from inside the blocks,
    // one instruction at a time (all waves' copies issued together queue up in front of the CU's address unit).
    // `parity` = kt & 1, as a run-time value or as a std::integral_constant: with a constant the stage of the tile
    // is a compile-time offset and the operand reads need no address arithmetic
    auto step_spread = [&](int kt, auto parity) {
        const int par = parity;
        wait_tile_loads();
        __syncthreads();
        const char* ktile = lds + par * (2 * kTileBytes);
        const char* vtile = ktile + kTileBytes;
        const uint32_t next = lds0 + (1 - par) * (2 * kTileBytes);
        const uint16_t* k_row = kbase + (int64_t)(kt + 1) * BK * p.kv_stride;
        const uint16_t* v_row = vbase + (int64_t)(kt + 1) * BK * p.kv_stride;
        auto piece = [&](int jb, int i) {
            if (jb == 0) kvcopy.issue_full_one_at(i, next, k_row, wave);
            else kvcopy.issue_full_one_at(i, next + kTileBytes, v_row, wave);
        };
        block(ktile, vtile, 0, kt * BK, std::false_type{}, std::true_type{}, piece);
        block(ktile, vtile, 1, kt * BK + 32, std::false_type{}, std::true_type{}, piece);
    };
    // separate loops instead of tests per tile: tiles wholly below the diagonal (with and without a whole
    // successor), then the (at most two) tiles on the diagonal
    // tiles whose every key exists and is visible to every row of this q tile (with the shift, keys past the end
    // of the chunk need the mask: the last, partial tile is never an interior one)
    const int n_interior = BLOCK ? max(0, min(min(n_tiles, (q_row0 + off + 1) / BK), L / BK)) : min(n_tiles, 2 * item.tile);
    const int n_spread = max(0, min(min(n_interior, n_tiles - 1), L / BK - 1));
    int kt = 0;
    // the long loop of a long sequence runs in pairs (even tile, odd tile) with constant stage offsets
    for (; kt + 1 < n_spread; kt += 2) {
        step_spread(kt, std::integral_constant<int, 0>{});
        step_spread(kt + 1, std::integral_constant<int, 1>{});
    }
    for (; kt < n_spread; ++kt) step_spread(kt, kt & 1);
    for (; kt < n_interior; ++kt) step(kt, std::false_type{});
    for (; kt < n_tiles; ++kt) step(kt, std::true_type{});

    if (p.rope_table != nullptr) {
        // dQ with respect to the queries before their rotary embedding; row positions inside the sequence
        __syncthreads();
        char* wave_lds = lds + wave * (32 * D * 4);
        const int64_t first_elem = ((int64_t)(item.q_start + wave_row0) * p.q_heads + h) * hd;
        const float* table_row0 = p.rope_table + (int64_t)(item.q_pos + wave_row0) * hd;
        if (BLOCK && p.dq_accumulate)
            store_tile_rope_transposed<D, true>(wave_lds, acc, p.scale, p.dq, first_elem, true, (int64_t)p.q_heads * hd,
                                                min(32, Lq - wave_row0), hd, table_row0, lane);
        else
            store_tile_rope_transposed<D, false>(wave_lds, acc, p.scale, p.dq, first_elem, p.grad_f32 != 0,
                                                 (int64_t)p.q_heads * hd, min(32, Lq - wave_row0), hd, table_row0, lane);
    } else if (p.grad_f32 != 0) {
        // whole rows per store instruction, staged through LDS (free once every wave has left the tile loop)
        __syncthreads();
        char* wave_lds = lds + wave * (32 * D * 4);
        float* first_row = static_cast<float*>(p.dq) + ((int64_t)(item.q_start + wave_row0) * p.q_heads + h) * hd;
        const int rows = min(32, Lq - wave_row0);
        if (BLOCK && p.dq_accumulate)
            store_tile_f32<D, true>(wave_lds, acc, p.scale, first_row, (int64_t)p.q_heads * hd, rows, hd, lane);
        else
            store_tile_f32<D, false>(wave_lds, acc, p.scale, first_row, (int64_t)p.q_heads * hd, rows, hd, lane);
    } else {
        __syncthreads();
        store_tile_bf16<D>(lds + wave * (32 * D * 2), acc, p.scale,
                           static_cast<uint16_t*>(p.dq) + ((int64_t)(item.q_start + wave_row0) * p.q_heads + h) * hd,
                           (int64_t)p.q_heads * hd, min(32, Lq - wave_row0), hd, lane);
    }
}

// ------------------------------------------------------------------------------- launchers
hipError_t launch_bwd_dsum(const BwdParams& p, int head_dim, hipStream_t stream) {
    const int64_t n_rows = p.total_tokens * p.q_heads;
    if (n_rows == 0) return hipSuccess;
    const int rows_per_block = kThreads / (tile_width(head_dim) / 8);
    const dim3 grid((unsigned)((n_rows + rows_per_block - 1) / rows_per_block)), block(kThreads);
    if (tile_width(head_dim) == 128) {
        hipLaunchKernelGGL(bwd_dsum_kernel<128>, grid, block, 0, stream, p);
    } else {
        hipLaunchKernelGGL(bwd_dsum_kernel<64>, grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_bwd_dq(const BwdParams& p, int head_dim, int64_t num_items, bool block, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), threads(kThreads);
    if (tile_width(head_dim) == 128) {
        if (contraction_steps(head_dim) <= 7) {
            if (block) hipLaunchKernelGGL((bwd_dq_kernel<128, true, 7>), grid, threads, 0, stream, p);
            else hipLaunchKernelGGL((bwd_dq_kernel<128, false, 7>), grid, threads, 0, stream, p);
        } else {
            if (block) hipLaunchKernelGGL((bwd_dq_kernel<128, true>), grid, threads, 0, stream, p);
            else hipLaunchKernelGGL((bwd_dq_kernel<128, false>), grid, threads, 0, stream, p);
        }
    } else {
        if (block) hipLaunchKernelGGL((bwd_dq_kernel<64, true>), grid, threads, 0, stream, p);
        else hipLaunchKernelGGL((bwd_dq_kernel<64, false>), grid, threads, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

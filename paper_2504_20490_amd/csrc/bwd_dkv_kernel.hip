// Backward dK/dV pass: one workgroup per (sequence, 128-key tile, kv head).
//
// Each of the 4 waves owns 32 keys (K and V rows stay in registers as MFMA B operands) and walks
// over the query heads of the KV group and, per head, over the 32-row query blocks at or below the
// diagonal.  Per block b:
//     G1(b): S' = Q_b K^T - LSE/scale, dP' = dO_b V^T - D    (16 MFMA, operands read along tile rows; the
//            statistics are the initial accumulator values)
//     V(b) : P = exp2(S' c), dS = P dP'                       (VALU, one lane per key)
//     G2(b): dV^T += dO_b^T P, dK^T += Q_b^T dS               (16 MFMA, operands by LDS transpose read)
// The group loop runs inside the workgroup, so dK/dV need no atomics.
//
// The kernel holds two fp32 accumulators of 32 x D per wave, which leaves room for only one wave
// per SIMD; one wave is one in-order instruction stream, so the loop is software-pipelined inside the
// wave and the instruction count per MFMA is kept low.  Iteration i is one basic block in two phases:
//     phase A: MFMA G2(i-1)  |  first half of V(i)   |  LDS reads: Q/dO rows and statistics of block i+1
//     phase B: MFMA G1(i+1)  |  second half of V(i)  |  LDS reads: Q^T/dO^T of block i (for G2(i) next time)
// so every MFMA operand is requested half an iteration (16 MFMAs) before its use and the exp/multiply work
// of one block is spread under the MFMAs of its neighbours.  S'/dP' are double buffered (block i is still
// being consumed while G1(i+1) accumulates).  Scheduling-group hints fix the interleaving.
//
// LDS: four stages of {Q tile, dO tile (64 rows each), -LSE/scale [64], -D [64]}.  While iterations
// 2t and 2t+1 work on tile t and read ahead into tile t+1, tiles t+2 and t+3 are in flight
// (global -> LDS copies; t+3 goes into the stage that tile t-1 occupied).  One barrier per tile.
#include <type_traits>

#include "attn_device.hpp"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

namespace {

// KD: 16-column steps of the contractions over head_dim (G1) that hold data: D / 16, or fewer when head_dim ends
// before the tile width (the steps beyond it would multiply the zero padding of the K / V fragments)
template <int D, int KD = D / 16>
struct DkvGeom {
    static_assert(KD >= 1 && KD <= D / 16, "k-steps inside the tile width");
    static constexpr int KK = D / 16;                      // fragments per G2 operand (2 k-steps x D / 32 row blocks)
    static constexpr int K1 = KD;                          // k-steps over head_dim of G1
    static constexpr int DB = D / 32;                      // 32-row blocks of dK^T / dV^T
    static constexpr int kTileBytes = kDkvQTile * D * 2;   // one 64-row tile
    static constexpr int kBlockBytes = 32 * D * 2;         // one 32-row block of it
    static constexpr int kStatBytes = 1024;                // -LSE/scale [64] at +0, -D [64] at +256
    static constexpr int kStageBytes = 2 * kTileBytes + kStatBytes;
    static constexpr int kStages = 4;
};

template <int D, int KD>
struct DkvState {
    using G = DkvGeom<D, KD>;
    bf16x8 kf[G::K1], vf[G::K1];           // this wave's 32 keys: K rows, V rows (B operands)
    f32x16 dk[G::DB], dv[G::DB];           // dK^T, dV^T accumulators
    f32x16 s[2], dp[2];                    // S - LSE/scale and dP - D: [i & 1] of block i, [~i & 1] of block i+1
    bf16x8 qf[G::K1], dof[G::K1];          // Q, dO rows of block i+1 (A operands of G1), live inside an iteration
    bf16x8 qtf[G::KK], dotf[G::KK];        // Q^T, dO^T of block i-1 (A operands of G2), index tt*DB + db
    bf16x8 pprev[2], dsprev[2];            // P, dS of block i-1 as bf16 B operands
};

// per-lane LDS byte addresses (stage base included) of the operand fragments
template <int D>
struct DkvAddr {
    using G = DkvGeom<D>;
    int rm[G::KK];         // row-major fragment kk of a 32-row block (Q tile; dO tile is + kTileBytes)
    int tr[G::DB][2];      // transposed fragment: column block db, 8-row part
    int st;                // statistics
};

// The global -> LDS copies of one whole 64-row tile (Q chunks, dO chunks, one statistics row), cut into
// this wave's single instructions so that an iteration can issue them one at a time between its MFMAs:
// issued back to back after the barrier, the copies of all four waves queue up in front of the CU's one
// address unit and every wave sits in its issue slot for hundreds of cycles with nothing else to run.
template <int D>
struct DkvTileLoad {
    using Copy = TileCopy<D, kDkvQTile>;
    static constexpr int kPieces = 2 * Copy::kPerWave + 1;
    const Copy* qcopy;
    const Copy* docopy;
    const uint16_t* q_row;      // first row of the tile, this head, column 0
    const uint16_t* do_row;
    const float* stat;          // -LSE/scale (even waves) or -D (odd waves) of the tile's first row
    uint32_t stage;             // LDS byte addresses
    uint32_t stat_dst;
    int wave, lane;
    template <int N>
    __device__ __forceinline__ void piece() const {
        if constexpr (N < Copy::kPerWave) {
            qcopy->template issue_full_one<N>(stage, q_row, wave);
        } else if constexpr (N < 2 * Copy::kPerWave) {
            docopy->template issue_full_one<N - Copy::kPerWave>(stage + DkvGeom<D>::kTileBytes, do_row, wave);
        } else if constexpr (N == 2 * Copy::kPerWave) {
            global_to_lds<4>(stat, (uint32_t)lane * 4u, stat_dst);
        }
    }
};

__device__ __forceinline__ bf16x8 lds_read128(const char* lds, int addr) {
    return *reinterpret_cast<const bf16x8*>(lds + addr);
}

template <int D>
__device__ __forceinline__ bf16x8 lds_read_tr(const char* lds, int a0, int a1) {
    const s16x4 lo = lds_transpose_read(lds + a0);
    const s16x4 hi = lds_transpose_read(lds + a1);
    union { struct { s16x4 a, b; } s; bf16x8 v; } u;
    u.s.a = lo;
    u.s.b = hi;
    return u.v;
}

// One pipelined iteration on block i (RB = i & 1 is its position inside its 64-row tile).
//   `cur`: addresses in the stage of block i's tile; `ahead`: addresses in the stage of block i+1's tile.
// dkey = my_key - (first row of block i) - 4 * (lane / 32): element e of an accumulator fragment is a
// masked (row < key) pair iff 8 * (e / 4) + e % 4 < dkey.
// SPREAD: the iteration also issues its share of the copies of a later tile (`load`), one instruction at a
// time at fixed places among its LDS reads (the copies are ordered against LDS accesses, the reads are tied
// to the MFMAs by the scheduling hints): pieces 0-3 in the first iteration of a tile, 4-8 in the second.
template <int D, int KD, int RB, bool MASK, bool SPREAD>
__device__ __forceinline__ void dkv_iteration(DkvState<D, KD>& st, const char* lds, const DkvAddr<D>& ahead,
                                              const DkvAddr<D>& cur, int dkey, float c, const DkvTileLoad<D>& load) {
    using G = DkvGeom<D, KD>;
    constexpr int KK = G::KK, DB = G::DB, K1 = G::K1;
    constexpr int NRB = RB ^ 1;   // block i+1 sits at the other position (of the next tile when RB == 1)
    constexpr int P0 = RB == 0 ? 0 : 4;   // first piece of this iteration

    // element e of an accumulator fragment -> packed bf16 pair index; one half = 8 elements = one B operand
    auto softmax_half = [&](int half, u32x4& pw, u32x4& dw) {
#pragma unroll
        for (int e = 8 * half; e < 8 * half + 8; e += 2) {
            float p0 = fast_exp2(st.s[RB][e] * c);
            float p1 = fast_exp2(st.s[RB][e + 1] * c);
            if (MASK && (8 * (e >> 2) + (e & 3) < dkey)) p0 = 0.f;
            if (MASK && (8 * ((e + 1) >> 2) + ((e + 1) & 3) < dkey)) p1 = 0.f;
            pw[(e >> 1) & 3] = pack_bf16(p0, p1);
            dw[(e >> 1) & 3] = pack_bf16(p0 * st.dp[RB][e], p1 * st.dp[RB][e + 1]);
        }
    };

    // ================= phase A =================
    // statistics of block i+1 straight into its accumulators: rows 8 j + 4 (lane / 32) .. + 3 in registers 4 j .. 4 j + 3
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(lds + ahead.st + NRB * 128 + i4 * 32);
        const f32x4 b = *reinterpret_cast<const f32x4*>(lds + ahead.st + NRB * 128 + i4 * 32 + 256);
#pragma unroll
        for (int j = 0; j < 4; ++j) { st.s[NRB][4 * i4 + j] = a[j]; st.dp[NRB][4 * i4 + j] = b[j]; }
    }
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
        st.qf[kk] = lds_read128(lds, ahead.rm[kk] + NRB * G::kBlockBytes);
        st.dof[kk] = lds_read128(lds, ahead.rm[kk] + NRB * G::kBlockBytes + G::kTileBytes);
        if constexpr (SPREAD) {
            if (kk == KK / 4 - 1) load.template piece<P0>();
            if (kk == 3 * KK / 4 - 1) load.template piece<P0 + 1>();
        }
    }
    // G2(i-1)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int tt = kk / DB, db = kk % DB;
        st.dv[db] = mfma(st.dotf[kk], st.pprev[tt], st.dv[db]);
        st.dk[db] = mfma(st.qtf[kk], st.dsprev[tt], st.dk[db]);
    }
    u32x4 pw0, dw0;
    softmax_half(0, pw0, dw0);
    // per MFMA: LDS reads (8 statistics + 2*KK fragments in all) and a share of the VALU work
    InterleaveHint<2 * KK, 2, (MASK ? 4 : 3), 0, 0x402>::apply();
    __builtin_amdgcn_sched_barrier(0);

    // ================= phase B =================
    union { u32x4 u; bf16x8 v; } cv;
    cv.u = pw0; st.pprev[0] = cv.v;
    cv.u = dw0; st.dsprev[0] = cv.v;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int off = (RB * 2 + tt) * 16 * D * 2;   // 16 tile rows per k-step
            st.qtf[tt * DB + db] = lds_read_tr<D>(lds, cur.tr[db][0] + off, cur.tr[db][1] + off);
            st.dotf[tt * DB + db] = lds_read_tr<D>(lds, cur.tr[db][0] + off + G::kTileBytes, cur.tr[db][1] + off + G::kTileBytes);
            if constexpr (SPREAD) {
                if (tt == 0 && db == DB - 1) load.template piece<P0 + 2>();
                if (tt == 1 && db == DB / 2 - 1) load.template piece<P0 + 3>();
                if (RB == 1 && tt == 1 && db == DB - 1) load.template piece<P0 + 4>();
            }
        }
    // G1(i+1) on top of the statistics
    // the two accumulation chains alternate: an MFMA that continues a chain does not follow its predecessor directly
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
        st.s[NRB] = mfma(st.qf[kk], st.kf[kk], st.s[NRB]);
        st.dp[NRB] = mfma(st.dof[kk], st.vf[kk], st.dp[NRB]);
    }
    u32x4 pw1, dw1;
    softmax_half(1, pw1, dw1);
    cv.u = pw1; st.pprev[1] = cv.v;
    cv.u = dw1; st.dsprev[1] = cv.v;
    // per MFMA: a share of the 4 * KK transpose reads (2 each, 3 when the phase has fewer MFMAs), VALU share
    InterleaveHint<2 * K1, (K1 == KK ? 2 : 3), (MASK ? 4 : 3), 1, 0x402>::apply();
    __builtin_amdgcn_sched_barrier(0);
}

}  // namespace

template <int D, bool BLOCK, int KD = D / 16>
__global__ __launch_bounds__(kThreads, 1) void bwd_dkv_kernel(BwdParams p) {
    using G = DkvGeom<D, KD>;
    constexpr int BKV = kDkvKTile, BQ = kDkvQTile;
    constexpr int KK = G::KK, DB = G::DB, K1 = G::K1;
    __shared__ __attribute__((aligned(1024))) char lds[G::kStages * G::kStageBytes];

    const ItemGeom item = load_item<BLOCK>(p.items, p.block_items, blockIdx.x);
    if (item.tile < 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = item.q_len, Lk = item.k_len, shift = item.offset, g = item.head;   // L: rows of the chunk
    const int key0 = item.tile * BKV;
    const int wave_key0 = key0 + wave * 32;
    const int my_key = wave_key0 + (lane & 31);
    const int hh = lane >> 5;
    const bool valid = my_key < Lk;

    const int hd = p.head_dim;   // elements per head in memory, <= D (columns hd .. D-1 exist only in LDS and registers)
    const uint16_t* kbase = p.k + (int64_t)item.k_start * p.kv_stride + (int64_t)g * hd;
    const uint16_t* vbase = p.v + (int64_t)item.k_start * p.kv_stride + (int64_t)g * hd;

    constexpr int kLoadsPerTile = 2 * (BQ * D * 2 / 1024) / 4 + 1;   // per wave: Q and dO chunks + one statistics copy
    // tiles: for each head of the group, q tiles first_qt .. n_qt-1 (rows at or below the diagonal: row r sees
    // key j iff j <= r + shift, so the tile's first key is seen by the rows from key0 - shift on)
    const int first_qt = max(0, key0 - shift) / BQ;
    const int n_qt = (L + BQ - 1) / BQ;
    const int per_head = max(0, n_qt - first_qt);
    const int n_tiles = per_head * p.group;
    if (BLOCK && per_head == 0) {
        // no row of the chunk sees these keys
        if (valid) {
            const int64_t row_elem = ((int64_t)(item.k_start + my_key) * p.kv_heads + g) * hd;
#pragma unroll
            for (int c4 = 0; c4 < D / 8; ++c4) {
                if (hh * (D / 2) + c4 * 4 >= hd) continue;
                store_grad4(p.dk, row_elem + hh * (D / 2) + c4 * 4, p.grad_f32 != 0, 0.f, 0.f, 0.f, 0.f);
                store_grad4(p.dv, row_elem + hh * (D / 2) + c4 * 4, p.grad_f32 != 0, 0.f, 0.f, 0.f, 0.f);
            }
        }
        return;
    }

    // global -> LDS copy of tile u (flattened over heads) into a stage, statistics included
    const uint32_t lds0 = lds_address(lds);   // copy destinations are LDS byte addresses
    TileCopy<D, BQ> qcopy, docopy;
    qcopy.init(p.q_stride, wave, lane, hd);
    docopy.init((int64_t)p.q_heads * hd, wave, lane, hd);
    auto load_tile = [&](int u, int stage_index) {
        const uint32_t stage = lds0 + stage_index * G::kStageBytes;
        const int hq = g * p.group + u / per_head;
        const int row0 = (n_qt - 1 - u % per_head) * BQ;   // q tiles are walked from the end of the sequence down
        const uint16_t* qb = p.q + (int64_t)item.q_start * p.q_stride + (int64_t)hq * hd;
        const uint16_t* dob = p.d_o + ((int64_t)item.q_start * p.q_heads + hq) * hd;
        // even waves: -LSE/scale of the 64 rows; odd waves: -D (waves 2, 3 repeat the copies of waves 0, 1 so that
        // every wave has the same number of loads in flight)
        const int which = wave & 1;
        const uint32_t stat_dst = stage + 2 * G::kTileBytes + which * 256;
        const int64_t stat0 = (int64_t)hq * p.total_tokens + item.q_start + row0;
        if (row0 + BQ <= L) {
            qcopy.issue_full(stage, qb, p.q_stride, row0, wave);
            docopy.issue_full(stage + G::kTileBytes, dob, (int64_t)p.q_heads * hd, row0, wave);
            global_to_lds<4>((which == 0 ? p.nlse : p.negd) + stat0, (uint32_t)lane * 4u, stat_dst);
        } else {
            // last tile of a head: rows past the end read a finite duplicate; their -LSE/scale reads -inf, so P = 0
            qcopy.issue_clamped(stage, qb, p.q_stride, row0, L, wave, lane);
            docopy.issue_clamped(stage + G::kTileBytes, dob, (int64_t)p.q_heads * hd, row0, L, wave, lane);
            const int r = row0 + lane;
            const int64_t stat = stat0 + min(lane, L - 1 - row0);
            const float* src = (which == 0) ? ((r < L) ? p.nlse + stat : p.ninf_pad) : p.negd + stat;
            global_to_lds<4>(src, stat_dst);
        }
    };

    load_tile(0, 0);
    if (n_tiles > 1) load_tile(1, 1);
    if (n_tiles > 2) load_tile(2, 2);

    DkvState<D, KD> st;
#pragma unroll
    for (int kk = 0; kk < K1; ++kk) {
        union { u32x4 u; bf16x8 v; } a, b;
        a.u = u32x4{0u, 0u, 0u, 0u};
        b.u = u32x4{0u, 0u, 0u, 0u};
        if (valid && kk * 16 + hh * 8 < hd) {
            a.u = *reinterpret_cast<const u32x4*>(kbase + (int64_t)my_key * p.kv_stride + kk * 16 + hh * 8);
            b.u = *reinterpret_cast<const u32x4*>(vbase + (int64_t)my_key * p.kv_stride + kk * 16 + hh * 8);
        }
        st.kf[kk] = a.v;
        st.vf[kk] = b.v;
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) { st.dk[db][i] = 0.f; st.dv[db][i] = 0.f; }
    const float c = p.scale_log2;

    // per-lane fragment offsets inside a stage
    DkvAddr<D> off;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) off.rm[kk] = tile_offset<D>(lane & 31, kk * 16 + hh * 8);
    {
        const int c16 = lane & 15;
        const int row = (hh << 2) + (c16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int col = db * 32 + (((lane >> 4) & 1) << 4) + ((c16 & 3) << 2);
            off.tr[db][0] = tile_offset<D>(row, col);
            off.tr[db][1] = tile_offset<D>(row + 8, col);
        }
    }
    off.st = 2 * G::kTileBytes + hh * 16;
    // `off` holds the addresses of the current tile's stage and is moved from stage to stage by adding the
    // distance (one set of address registers instead of one per stage in use)
    auto shifted = [&](const DkvAddr<D>& a0, int bytes) {
        DkvAddr<D> a;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) a.rm[kk] = a0.rm[kk] + bytes;
#pragma unroll
        for (int db = 0; db < DB; ++db) { a.tr[db][0] = a0.tr[db][0] + bytes; a.tr[db][1] = a0.tr[db][1] + bytes; }
        a.st = a0.st + bytes;
        return a;
    };

    wait_tile_loads();
    __syncthreads();   // tiles 0, 1 and 2 are in LDS

    // prologue: G1(0) computed directly on top of block 0's statistics; P = dS = 0 for the non-existent block -1
    {
        const DkvAddr<D>& a0 = off;   // stage 0
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(lds + a0.st + i4 * 32);
            const f32x4 b = *reinterpret_cast<const f32x4*>(lds + a0.st + i4 * 32 + 256);
#pragma unroll
            for (int j = 0; j < 4; ++j) { st.s[0][4 * i4 + j] = a[j]; st.dp[0][4 * i4 + j] = b[j]; }
        }
#pragma unroll
        for (int kk = 0; kk < K1; ++kk) {
            st.s[0] = mfma(lds_read128(lds, a0.rm[kk]), st.kf[kk], st.s[0]);
            st.dp[0] = mfma(lds_read128(lds, a0.rm[kk] + G::kTileBytes), st.vf[kk], st.dp[0]);
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            st.qtf[kk] = lds_read128(lds, a0.rm[kk]);      // any finite operand: it meets P = dS = 0
            st.dotf[kk] = st.qtf[kk];
        }
        union { u32x4 u; bf16x8 v; } z;
        z.u = u32x4{0u, 0u, 0u, 0u};
        st.pprev[0] = st.pprev[1] = st.dsprev[0] = st.dsprev[1] = z.v;
    }

    // One tile = two iterations.  The two q tiles next to the diagonal hold the (row < key) pairs of some wave
    // and take the masked code; all other tiles take the unmasked code.  Two loops instead of a branch inside
    // one: the ~400 live registers then meet at a join once per head, not once per iteration.
    int stage = 0;   // stage of tile u
    DkvTileLoad<D> no_load{};
    auto tile_step = [&](int u, int qt, auto masked) {
        constexpr bool kMask = decltype(masked)::value;
        if (u > 0) {
            // tile u+1 must have landed; the copies of tile u+2 (the newest kLoadsPerTile of this wave) may still fly
            if (u + 2 < n_tiles) wait_tile_loads_except<kLoadsPerTile>(); else wait_tile_loads();
            __syncthreads();   // ... for every wave; and every wave is done with tile u-1
        }
        const int stage1 = stage + 1 == G::kStages ? 0 : stage + 1;
        const int stage3 = (stage + 3) % G::kStages;
        if (u + 3 < n_tiles) load_tile(u + 3, stage3);
        // block 2u+2 lives in the next tile; the last tile has none: it re-reads itself (result unused)
        const int to_next = (stage1 - stage) * G::kStageBytes;
        const DkvAddr<D> next = shifted(off, u + 1 < n_tiles ? to_next : 0);
        const int dkey0 = my_key - shift - qt * BQ - 4 * hh;
        dkv_iteration<D, KD, 0, kMask, false>(st, lds, off, off, dkey0, c, no_load);
        dkv_iteration<D, KD, 1, kMask, false>(st, lds, next, off, dkey0 - 32, c, no_load);
        off = shifted(off, to_next);
        stage = stage1;
    };
    // The same for an unmasked tile that is at least three tiles above the head's last one: the tile loaded
    // meanwhile (u + 3) belongs to the same head and is a whole tile, so its copies need no case distinction
    // and are issued from inside the two iterations.
    // `load` arrives pointing at the first rows of tile qt - 3 of the head and leaves pointing one tile lower.
    auto tile_step_spread = [&](int u, int qt, DkvTileLoad<D>& load) {
        if (u > 0) {
            wait_tile_loads_except<kLoadsPerTile>();   // u + 2 < n_tiles here
            __syncthreads();
        }
        const int stage1 = stage + 1 == G::kStages ? 0 : stage + 1;
        const int stage3 = stage == 0 ? G::kStages - 1 : stage - 1;   // (stage + 3) % kStages
        load.stage = lds0 + stage3 * G::kStageBytes;
        load.stat_dst = load.stage + 2 * G::kTileBytes + (wave & 1) * 256;
        const int to_next = (stage1 - stage) * G::kStageBytes;
        const DkvAddr<D> next = shifted(off, to_next);
        const int dkey0 = my_key - shift - qt * BQ - 4 * hh;
        dkv_iteration<D, KD, 0, false, true>(st, lds, off, off, dkey0, c, load);
        dkv_iteration<D, KD, 1, false, true>(st, lds, next, off, dkey0 - 32, c, load);
        off = shifted(off, to_next);
        load.q_row -= (int64_t)BQ * p.q_stride;
        load.do_row -= (int64_t)BQ * p.q_heads * hd;
        load.stat -= BQ;
        stage = stage1;
    };
    // Every head is walked from its LAST q tile down to the diagonal.  All key tiles of one (sequence, kv head)
    // run on one XCD at about the same time; walking down from the common end keeps them on the same Q / dO
    // tiles at the same time (one L2 fill serves them all), whereas walking up from each item's own diagonal
    // would spread them over the whole sequence.
    // q tiles that hold some (row, key) pair above the shifted diagonal for the keys of this workgroup:
    // qt BQ + shift < key0 + BKV - 1; the two nearest the diagonal when there is no shift
    const int n_masked = BLOCK ? (key0 + BKV - 2 - shift < 0 ? 0 : max(0, min(per_head, (key0 + BKV - 2 - shift) / BQ - first_qt + 1)))
                               : min(2, per_head);
    const int n_general = max(3, n_masked);   // tiles below this index (from the diagonal) take the general path
    for (int h = 0, u = 0; h < p.group; ++h) {
        int j = per_head - 1;
        if (j >= n_general) {
            const int hq = g * p.group + h;
            const int64_t row = item.q_start + (int64_t)(first_qt + j - 3) * BQ;   // first row of the tile loaded first
            DkvTileLoad<D> load;
            load.qcopy = &qcopy;
            load.docopy = &docopy;
            load.q_row = p.q + row * p.q_stride + (int64_t)hq * hd;
            load.do_row = p.d_o + (row * p.q_heads + hq) * hd;
            load.stat = ((wave & 1) == 0 ? p.nlse : p.negd) + (int64_t)hq * p.total_tokens + row;
            load.wave = wave;
            load.lane = lane;
            for (; j >= n_general; --j, ++u) tile_step_spread(u, first_qt + j, load);
        }
        for (; j >= n_masked; --j, ++u) tile_step(u, first_qt + j, std::false_type{});
        for (; j >= 0; --j, ++u) tile_step(u, first_qt + j, std::true_type{});
    }

    // epilogue: G2 of the last block
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int tt = kk / DB, db = kk % DB;
        st.dv[db] = mfma(st.dotf[kk], st.pprev[tt], st.dv[db]);
        st.dk[db] = mfma(st.qtf[kk], st.dsprev[tt], st.dk[db]);
    }

    // whole rows per store instruction, staged through LDS (free once every wave has left the tile loop)
    const bool rope = p.rope_table != nullptr;
    __syncthreads();
    char* wave_lds = lds + wave * (32 * D * 4);
    const int64_t row0_elem = ((int64_t)(item.k_start + wave_key0) * p.kv_heads + g) * hd;
    const int64_t row_stride = (int64_t)p.kv_heads * hd;
    const int rows = min(32, Lk - wave_key0);
    if (rope) {
        // dK with respect to the keys before their rotary embedding; key positions inside the sequence
        store_tile_rope_transposed<D>(wave_lds, st.dk, p.scale, p.dk, row0_elem, p.grad_f32 != 0, row_stride, rows, hd,
                                      p.rope_table + (int64_t)(item.q_pos - item.offset + wave_key0) * hd, lane);
    } else if (p.grad_f32 != 0) {
        store_tile_f32<D, false>(wave_lds, st.dk, p.scale, static_cast<float*>(p.dk) + row0_elem, row_stride, rows, hd, lane);
    } else {
        store_tile_bf16<D>(wave_lds, st.dk, p.scale, static_cast<uint16_t*>(p.dk) + row0_elem, row_stride, rows, hd, lane);
    }
    if (p.grad_f32 != 0) {
        store_tile_f32<D, false>(wave_lds, st.dv, 1.f, static_cast<float*>(p.dv) + row0_elem, row_stride, rows, hd, lane);
    } else {
        store_tile_bf16<D>(wave_lds, st.dv, 1.f, static_cast<uint16_t*>(p.dv) + row0_elem, row_stride, rows, hd, lane);
    }
}

hipError_t launch_bwd_dkv(const BwdParams& p, int head_dim, int64_t num_items, bool block, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), threads(kThreads);
    if (tile_width(head_dim) == 128) {
        if (contraction_steps(head_dim) <= 7) {
            if (block) hipLaunchKernelGGL((bwd_dkv_kernel<128, true, 7>), grid, threads, 0, stream, p);
            else hipLaunchKernelGGL((bwd_dkv_kernel<128, false, 7>), grid, threads, 0, stream, p);
        } else {
            if (block) hipLaunchKernelGGL((bwd_dkv_kernel<128, true>), grid, threads, 0, stream, p);
            else hipLaunchKernelGGL((bwd_dkv_kernel<128, false>), grid, threads, 0, stream, p);
        }
    } else {
        if (block) hipLaunchKernelGGL((bwd_dkv_kernel<64, true>), grid, threads, 0, stream, p);
        else hipLaunchKernelGGL((bwd_dkv_kernel<64, false>), grid, threads, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

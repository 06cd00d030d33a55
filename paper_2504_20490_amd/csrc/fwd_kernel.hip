// Forward kernel: one workgroup per (sequence, 128-row q tile, q head) work item.
//
// Each of the 4 waves owns 32 query rows.  For every 64-key tile of the causal prefix the
// workgroup stages K and V in LDS (coalesced 16-byte global->LDS copies, double buffered, one
// barrier per tile); each wave computes S^T = K Q^T on MFMA (keys along rows, its queries along
// columns), runs the online-softmax recurrence with one lane per query, and feeds the bf16
// P^T fragments straight back into MFMA as the B operand of O^T += V^T P^T, V^T being read
// from the row-major V tile with the LDS transpose read.
//
// The loop is software-pipelined by one tile: the MFMAs of S^T(kt+1) run under the exp work of tile kt's
// first key block, the first MFMAs of tile kt's P V under that of its second key block.  K therefore
// runs one tile ahead of V in LDS.  Both phases are written MFMA step by MFMA step (operand reads a few
// steps ahead, a scheduling barrier after each step).  Tiles that lie wholly below the diagonal take
// code without any mask; only the tiles on the diagonal compare key and row indices.  With BLOCK the
// query rows and the keys are separate chunks and the diagonal is shifted (one step of context-parallel
// attention): partial O in fp32, LSE = -inf for rows that see no key.
#include "attn_device.hpp"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

namespace {

// KD: 16-column steps of the contraction over head_dim that hold data (D / 16, or fewer when head_dim ends before the
// tile width: the steps beyond it would multiply the zero padding of the query fragments)
template <int D, int KD>
struct FwdGeom {
    static_assert(KD >= 1 && KD <= D / 16, "k-steps inside the tile width");
    static constexpr int KK = KD;       // k-steps of S^T = K Q^T
    static constexpr int DB = D / 32;   // 32-row blocks of O^T
    static constexpr int kTileBytes = kFwdKTile * D * 2;
};

template <int D, int KD>
struct FwdState {
    using G = FwdGeom<D, KD>;
    bf16x8 qf[G::KK];      // this lane's query row (B operand of S^T = K Q^T)
    f32x16 acc[G::DB];     // O^T accumulator
    f32x16 s[2];           // S^T of the current tile (two 32-key blocks)
    float m, l;            // running row max of the raw scores; this lane's share of the running row sum
    float tnext;           // this lane's maximum over s[] as it stands (all keys taken as visible)
    int rm[G::KK];         // per-lane LDS offsets of the K fragments (row-major read), block 0 of a tile
    int tr[G::DB][2];      // per-lane LDS offsets of the V^T fragments (transpose read), k-step 0 of a tile
};

// this wave's single copy instructions of one whole K tile and one whole V tile
template <int D>
struct FwdTileLoad {
    using Copy = TileCopy<D, kFwdKTile>;
    const Copy* copy;
    const uint16_t* k_row;   // first row of the K tile, this kv head, column 0
    const uint16_t* v_row;
    uint32_t k_dst;          // LDS byte addresses
    uint32_t v_dst;
    int wave;
    __device__ __forceinline__ void k_piece(int i) const {
#pragma unroll
        for (int n = 0; n < Copy::kPerWave; ++n)
            if (n == i) copy->issue_full_one_at(n, k_dst, k_row, wave);
    }
    __device__ __forceinline__ void v_piece(int i) const {
#pragma unroll
        for (int n = 0; n < Copy::kPerWave; ++n)
            if (n == i) copy->issue_full_one_at(n, v_dst, v_row, wave);
    }
};

// this lane's maximum over the 32 scores of a tile (v_max3: two scores per instruction)
__device__ __forceinline__ float lane_max(const f32x16 (&s)[2]) {
    float t = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int e = 2; e < 32; ++e) t = fmaxf(t, s[e >> 4][e & 15]);   // a chain: pairs of steps become one v_max3
    return t;
}

__device__ __forceinline__ float pair_max(float x) {
    // v_permlane32_swap: first result = the value held by lane l % 32, second = the value of lane l % 32 + 32
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// One iteration on key tile kt, whose scores are already in st.s:
//   first  : VALU only: running max of tile kt; accumulator rescale if some lane's max moved
//   phase A: MFMA S^T(kt+1) = K(kt+1) Q^T   |  VALU: exp2, row sum, bf16 pack of tile kt's first key block
//   phase B: MFMA O^T += V(kt)^T P^T(kt)     |  VALU: the same for its second key block, under the first MFMAs
// kbuf: K tile kt+1; vbuf: V tile kt.  MASK: tile kt touches the diagonal (keys beyond a lane's own row get
// weight 0); LAST: there is no tile kt+1.
// SPREAD: the iteration also issues this wave's share of the copies of K(kt+2) and V(kt+1), both whole
// tiles, one instruction per MFMA step of phase A.  Issued back to back after the barrier, the copies of
// all waves queue up in front of the CU's one address unit.
// BLOCK: a lane's row may have no visible key so far (its running max is still -inf): the maximum that the
// exponentials are taken against is then replaced by 0, which keeps every weight and the rescale factor at 0.
template <int D, int KD, bool MASK, bool LAST, bool SPREAD, bool BLOCK>
__device__ __forceinline__ void fwd_iteration(FwdState<D, KD>& st, const char* kbuf, const char* vbuf, float c,
                                              int dkey /* my_row - key0 - 4 * (lane / 32) */,
                                              const FwdTileLoad<D>& load) {
    using G = FwdGeom<D, KD>;
    constexpr int KK = G::KK, DB = G::DB;
    constexpr int NP = FwdTileLoad<D>::Copy::kPerWave;   // copy instructions per wave and tile

    // ---------------- running max of tile kt and the (rare) accumulator rescale: a short VALU-only stretch
    if constexpr (MASK) {
        // element i of block jb is key 32 jb + 8 (i / 4) + i % 4 (+ 4 (lane / 32), folded into dkey)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (32 * jb + 8 * (i >> 2) + (i & 3) > dkey) st.s[jb][i] = -INFINITY;
    }
    // An unmasked tile's maximum was taken while the scores were still warm: under the last MFMAs of the iteration
    // that produced them, which have no other VALU work to run beside them (st.tnext).
    float tmax = st.tnext;
    if constexpr (MASK) tmax = lane_max(st.s);
    tmax = pair_max(tmax);
    // st.m is the reference that the exponentials are taken against, not the exact running maximum: it moves only
    // when the maximum has risen by more than kMaxSlack in the exponent (base-2) domain.  Weights then lie in
    // (0, 2^kMaxSlack] instead of (0, 1] -- the same relative precision in bf16 and fp32, and O and LSE do not depend on
    // the reference -- while the accumulator rescale, which a moving maximum of ANY of the wave's 32 rows triggers,
    // becomes rare after the first tiles.  (-inf - -inf = NaN compares false: a row without a visible key keeps -inf.)
    constexpr float kMaxSlack = 8.f;
    const float m_new = (tmax - st.m) * c > kMaxSlack ? tmax : st.m;
    const float m_ref = (BLOCK && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2((st.m - m_ref) * c);
    const float mc = m_ref * c;
    if (__any(m_new > st.m)) {      // wave-uniform: skip the accumulator rescale when no lane's max moved
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.acc[db][i] *= alpha;
    }
    st.m = m_new;
    __builtin_amdgcn_sched_barrier(0);

    // The two waves of a SIMD (one of each resident workgroup) compete for its issue slots: the one that is in its
    // MFMA phases goes first, so that the matrix pipe does not wait behind the other's VALU-only stretch.
    __builtin_amdgcn_s_setprio(1);
    // ---------------- phase A: S^T(kt+1) on the MFMA, exp2 / row sum / bf16 pack of tile kt on the VALU.
    // Written out step by step with a scheduling barrier after each: step n issues the K fragment read of
    // MFMA n + kAheadK, MFMA n, and the softmax work on two scores.
    f32x16 sn[2];
    float psum = 0.f;
    union { u32x4 u; bf16x8 v; } pw[4];
    auto softmax_pair = [&](int n) {   // scores 2n, 2n+1 of the tile's 32 per lane -> one packed bf16 pair
        const int jb = n >> 3, i = (n & 7) * 2;
        const float e0 = fast_exp2(fmaf(st.s[jb][i], c, -mc));
        const float e1 = fast_exp2(fmaf(st.s[jb][i + 1], c, -mc));
        psum += e0 + e1;
        // the sum is needed only at the end of the iteration, and left alone the compiler keeps all 32 weights in
        // registers and adds them up there, in one stretch of 32 VALU instructions with no MFMA to run under;
        // an (empty) statement that reads and writes the sum keeps each pair's two additions in this step
        asm volatile("" : "+v"(psum));
        pw[jb * 2 + (i >> 3)].u[(i >> 1) & 3] = pack_bf16(e0, e1);
    };
    if constexpr (!LAST) {
        constexpr int kAheadK = 4;
        constexpr int NM = 2 * KK;               // MFMAs of the phase
        static_assert(2 * NP <= NM, "one copy instruction per MFMA step");
        auto k_frag = [&](int n) {
            return *reinterpret_cast<const bf16x8*>(kbuf + st.rm[n % KK] + (n / KK) * 32 * D * 2);
        };
        bf16x8 kq[kAheadK + 1];
#pragma unroll
        for (int n = 0; n < kAheadK; ++n) kq[n] = k_frag(n);
#pragma unroll
        for (int i = 0; i < 16; ++i) { sn[0][i] = 0.f; sn[1][i] = 0.f; }
#pragma unroll
        for (int n = 0; n < NM; ++n) {
            if (n + kAheadK < NM) kq[(n + kAheadK) % (kAheadK + 1)] = k_frag(n + kAheadK);
            sn[n / KK] = mfma(kq[n % (kAheadK + 1)], st.qf[n % KK], sn[n / KK]);
            // the first 8 of the 16 score pairs (key block 0, P fragments 0 and 1) spread over the NM MFMAs; the
            // other 8 go under the first P V MFMAs of phase B, which only need fragments 0 and 1
            if constexpr (NM > 8) {
                // pairs 0 .. NM/2 - 1 at the even steps; with fewer than 16 steps the remaining ones at the last odd steps
                if (n % 2 == 0) softmax_pair(n / 2);
                else if (7 - (NM - 1 - n) / 2 >= NM / 2) softmax_pair(7 - (NM - 1 - n) / 2);
            } else {
                static_assert(NM == 8, "eight score pairs over the steps of the phase");
                softmax_pair(n);
            }
            if constexpr (SPREAD) {
                // all copies early in the iteration: both tiles are needed right after the next barrier
                if (n < NP) load.k_piece(n);
                else if (n < 2 * NP) load.v_piece(n - NP);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int n = 0; n < 8; ++n) softmax_pair(n);
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---------------- phase B: O^T += V(kt)^T P^T(kt), transpose reads kAheadV MFMAs ahead
    {
        constexpr int kAheadV = 3;
        constexpr int NM = 4 * DB;
        auto v_frag = [&](int n) {
            const int t = n / DB, db = n % DB;
            const int off = t * 16 * D * 2;
            union { struct { s16x4 a, b; } s; bf16x8 v; } u;
            u.s.a = lds_transpose_read(vbuf + st.tr[db][0] + off);
            u.s.b = lds_transpose_read(vbuf + st.tr[db][1] + off);
            return u.v;
        };
        bf16x8 vq[kAheadV + 1];
#pragma unroll
        for (int n = 0; n < kAheadV; ++n) vq[n] = v_frag(n);
        // the next tile's maximum, a share of its 32 scores per step (the scores are complete since phase A)
        float tnext = -INFINITY;
        auto max_share = [&](int e0, int count) {
#pragma unroll
            for (int e = e0; e < e0 + count; ++e) tnext = fmaxf(tnext, sn[e >> 4][e & 15]);   // a chain: v_max3 per pair
            // (an empty statement on the running value keeps the share in its step: nothing else needs the value
            // before the end of the iteration, and the compiler would collect all 32 there)
            asm volatile("" : "+v"(tnext));
        };
#pragma unroll
        for (int n = 0; n < NM; ++n) {
            if (n + kAheadV < NM) vq[(n + kAheadV) % (kAheadV + 1)] = v_frag(n + kAheadV);
            st.acc[n % DB] = mfma(vq[n % (kAheadV + 1)], pw[n / DB].v, st.acc[n % DB]);
            // score pairs 8 .. 15 (key block 1, P fragments 2 and 3) under the MFMAs of fragments 0 and 1
            if constexpr (DB == 4) {
                if (n < 8) softmax_pair(8 + n);
                else if (!LAST) max_share((n - 8) * 4, 4);
            } else {
                if (n < 4) { softmax_pair(8 + 2 * n); softmax_pair(9 + 2 * n); }
                else if (!LAST) max_share((n - 4) * 8, 8);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (!LAST) st.tnext = tnext;
    }
    __builtin_amdgcn_s_setprio(0);
    st.l = st.l * alpha + psum;
    if constexpr (!LAST) {
        st.s[0] = sn[0];
        st.s[1] = sn[1];
    }
}

}  // namespace

template <int D, bool BLOCK, int KD = D / 16>
__global__ __launch_bounds__(kThreads, 2) void fwd_kernel(FwdParams p) {
    using G = FwdGeom<D, KD>;
    constexpr int BQ = kFwdQTile, BK = kFwdKTile;
    constexpr int KK = G::KK, DB = G::DB;
    constexpr int kTileBytes = G::kTileBytes;
    // K tiles kt+1 / kt+2 and V tiles kt / kt+1: two buffers each
    __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];
    __shared__ int next_slot;
    char* const kbuf0 = lds;
    char* const vbuf0 = lds + 2 * kTileBytes;
    const uint32_t kdst0 = lds_address(lds), vdst0 = kdst0 + 2 * kTileBytes;   // the same buffers as copy destinations

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5;
    const int hd = p.head_dim;   // elements per head in memory, <= D (columns hd .. D-1 exist only in LDS and registers)
    const float c = p.scale_log2;

    // what does not depend on the item: copy geometry and per-lane LDS offsets of the operand fragments
    TileCopy<D, BK> kvcopy;   // K and V share stride and geometry
    kvcopy.init(p.kv_stride, wave, lane, hd);
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

    // ---- one work item: a 128-row q tile of one (sequence, q head)
    ItemQueue queue;
    queue.init(p.queue);
    int drawn = 0;
    auto run_item = [&](const ItemGeom& item) {
        // The lane index as the item's own code sees it: an empty statement makes it a new value per item, so that what
        // the prologue and the epilogue derive from it (row numbers, addresses of the staged stores) is computed per
        // item.  Derived from the kernel-wide lane index, those values would be loop-invariant, would be moved out of
        // the item loop and would then occupy registers all through the tile loop, which has none to spare.
        int lane = tid & 63;
        asm volatile("" : "+v"(lane));
        const int hh = lane >> 5;
        // the item's state is a new object: nothing of the previous item stays alive (a state kept across items would
        // hold the previous scores in registers through the prologue, wherever a wave might have no tile of its own)
        FwdState<D, KD> st;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) st.rm[kk] = rm[kk];
#pragma unroll
        for (int db = 0; db < DB; ++db) { st.tr[db][0] = tr[db][0]; st.tr[db][1] = tr[db][1]; }
        const int Lq = item.q_len, L = item.k_len, off = item.offset;   // L: keys of the chunk (= rows when !BLOCK)
        const int h = item.head, hk = h / p.group;
        const int q_row0 = item.tile * BQ;
        const int wave_row0 = q_row0 + wave * 32;
        const int my_row = wave_row0 + (lane & 31);

        const uint16_t* qbase = p.q + (int64_t)item.q_start * p.q_stride + (int64_t)h * hd;
        const uint16_t* kbase = p.k + (int64_t)item.k_start * p.kv_stride + (int64_t)hk * hd;
        const uint16_t* vbase = p.v + (int64_t)item.k_start * p.kv_stride + (int64_t)hk * hd;

        // key j is visible to row r iff j <= r + off: the tile's last row sees keys 0 .. kv_end-1
        const int kv_end = max(0, min(L, min(Lq, q_row0 + BQ) + off));
        const int n_tiles = (kv_end + BK - 1) / BK;
        // last key this lane's row may see, as an index into the chunk
        const int my_limit = BLOCK ? min(my_row + off, L - 1) : my_row;
        // this wave's own share: the tiles that hold a key visible to one of its 32 rows, and those among them that
        // are visible to all of them (a wave whose rows lie past the end of the chunk computes nothing).  On the
        // diagonal the upper waves of a workgroup see fewer tiles than the lower ones.
        const int kv_end_w = wave_row0 < Lq ? max(0, min(L, min(Lq, wave_row0 + 32) + off)) : 0;
        const int n_tiles_w = (kv_end_w + BK - 1) / BK;
        const int n_interior_w = max(0, min(min(n_tiles_w, (wave_row0 + off + 1) / BK), L / BK));
        if (BLOCK && n_tiles == 0) {
            // no key of the chunk is visible to any row of the tile: O = 0, LSE = -inf
            if (my_row < Lq) {
                float* orow = p.o_f32 + ((int64_t)(item.q_start + my_row) * p.q_heads + h) * hd;
    #pragma unroll
                for (int c4 = 0; c4 < D / 8; ++c4)
                    if (hh * (D / 2) + c4 * 4 < hd)
                        *reinterpret_cast<f32x4*>(orow + hh * (D / 2) + c4 * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
                if (hh == 0) p.lse[(int64_t)h * p.total_tokens + item.q_start + my_row] = -INFINITY;
            }
            if (tid == 0) drawn = queue.draw();
            return;
        }

        // K(0), V(0), K(1)
        kvcopy.issue(kdst0, kbase, p.kv_stride, 0, L, wave, lane);
        kvcopy.issue(vdst0, vbase, p.kv_stride, 0, L, wave, lane);
        if (n_tiles > 1) kvcopy.issue(kdst0 + kTileBytes, kbase, p.kv_stride, BK, L, wave, lane);

    #pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            union { u32x4 u; bf16x8 v; } t;
            t.u = u32x4{0u, 0u, 0u, 0u};
            if (my_row < Lq && kk * 16 + hh * 8 < hd)
                t.u = *reinterpret_cast<const u32x4*>(qbase + (int64_t)my_row * p.q_stride + kk * 16 + hh * 8);
            st.qf[kk] = t.v;
        }
    #pragma unroll
        for (int db = 0; db < DB; ++db)
    #pragma unroll
            for (int i = 0; i < 16; ++i) st.acc[db][i] = 0.f;
        st.m = -INFINITY;
        st.l = 0.f;

        wait_tile_loads();
        __syncthreads();
        // S^T(0), not pipelined
        if (n_tiles_w > 0)
    #pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
    #pragma unroll
            for (int i = 0; i < 16; ++i) st.s[jb][i] = 0.f;
    #pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                st.s[jb] = mfma(*reinterpret_cast<const bf16x8*>(kbuf0 + st.rm[kk] + jb * 32 * D * 2), st.qf[kk], st.s[jb]);
        }
        st.tnext = n_tiles_w > 0 ? lane_max(st.s) : -INFINITY;

        // iteration kt: K(kt+1) in kbuf[(kt+1) & 1], V(kt) in vbuf[kt & 1]; issues K(kt+2) -> kbuf[kt & 1] and
        // V(kt+1) -> vbuf[(kt+1) & 1], both free since the barrier at the top
        FwdTileLoad<D> no_load{};
        auto step = [&](int kt, auto masked, auto last) {
            if (kt > 0) {
                wait_tile_loads();
                __syncthreads();   // K(kt+1) and V(kt) have landed; every wave is done with iteration kt-1
            }
            if (kt + 2 < n_tiles) kvcopy.issue(kdst0 + (kt & 1) * kTileBytes, kbase, p.kv_stride, (kt + 2) * BK, L, wave, lane);
            if (kt + 1 < n_tiles) kvcopy.issue(vdst0 + ((kt + 1) & 1) * kTileBytes, vbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
            fwd_iteration<D, KD, decltype(masked)::value, decltype(last)::value, false, BLOCK>(
                st, kbuf0 + ((kt + 1) & 1) * kTileBytes, vbuf0 + (kt & 1) * kTileBytes, c, my_limit - kt * BK - 4 * hh, no_load);
        };
        // the same for an unmasked tile whose successors kt+1 and kt+2 are whole tiles: their copies need no case
        // distinction and are issued from inside the iteration
        // `parity` = kt & 1, as a run-time value or as a std::integral_constant: with a constant the LDS buffers of the
        // iteration are compile-time offsets and the operand reads need no address arithmetic
        auto step_spread = [&](int kt, auto parity) {
            const int par = parity;
            if (kt > 0) {
                wait_tile_loads();
                __syncthreads();
            }
            FwdTileLoad<D> load;
            load.copy = &kvcopy;
            load.k_row = kbase + (int64_t)(kt + 2) * BK * p.kv_stride;
            load.v_row = vbase + (int64_t)(kt + 1) * BK * p.kv_stride;
            load.k_dst = kdst0 + par * kTileBytes;
            load.v_dst = vdst0 + (1 - par) * kTileBytes;
            load.wave = wave;
            fwd_iteration<D, KD, false, false, true, BLOCK>(st, kbuf0 + (1 - par) * kTileBytes, vbuf0 + par * kTileBytes, c,
                                                        my_limit - kt * BK - 4 * hh, load);
        };
        // a tile past this wave's own diagonal: the barrier and the wave's share of the copies, nothing else
        auto idle = [&](int kt) {
            if (kt > 0) {
                wait_tile_loads();
                __syncthreads();
            }
            if (kt + 2 < n_tiles) kvcopy.issue(kdst0 + (kt & 1) * kTileBytes, kbase, p.kv_stride, (kt + 2) * BK, L, wave, lane);
            if (kt + 1 < n_tiles) kvcopy.issue(vdst0 + ((kt + 1) & 1) * kTileBytes, vbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
        };
        // separate loops instead of branches inside one: unmasked tiles (with and without whole successors), masked
        // tiles, and the wave's final tile (which has no successor to compute scores for); the large register state
        // then meets at a join once per loop, not per tile.  Every wave passes the barrier of every tile of the
        // workgroup, in whichever loop it happens to be.
        const int n_plain = min(n_interior_w, n_tiles_w - 1);
        const int n_spread = max(0, min(n_plain, L / BK - 2));   // tile kt+2 exists and is whole
        int kt = 0;
        // the long loop of a long sequence runs in pairs (even tile, odd tile) with constant buffer offsets
        for (; kt + 1 < n_spread; kt += 2) {
            step_spread(kt, std::integral_constant<int, 0>{});
            step_spread(kt + 1, std::integral_constant<int, 1>{});
        }
        for (; kt < n_spread; ++kt) step_spread(kt, kt & 1);
        for (; kt < n_plain; ++kt) step(kt, std::false_type{}, std::false_type{});
        for (; kt < n_tiles_w - 1; ++kt) step(kt, std::true_type{}, std::false_type{});
        if (n_tiles_w > 0) {
            step(kt, std::true_type{}, std::true_type{});   // the wave's final tile touches its diagonal (always, when !BLOCK)
            ++kt;
        }
        for (; kt < n_tiles; ++kt) idle(kt);

        // the next slot is requested when the tiles are done (not earlier: a slot reserved at the start of a long item
        // would wait for that item while other workgroups run out of work) and looked at after the stores
        if (tid == 0) drawn = queue.draw();
        const float l_row = st.l + partner32(st.l);
        // O leaves through LDS (free once every wave has left the tile loop) so that every store instruction writes
        // whole rows; a row that saw no key (BLOCK only) has l = 0 and m = -inf: O = 0, LSE = -inf
        __syncthreads();
        const float inv = (!BLOCK || l_row > 0.f) ? 1.f / l_row : 0.f;
        const int rows = min(32, Lq - wave_row0);
        const int64_t row0_elem = ((int64_t)(item.q_start + wave_row0) * p.q_heads + h) * hd;
        // the normaliser differs per row (= per lane): scale the fragments in place, then store with factor 1
    #pragma unroll
        for (int db = 0; db < DB; ++db)
    #pragma unroll
            for (int i = 0; i < 16; ++i) st.acc[db][i] *= inv;
        if constexpr (BLOCK) {
            store_tile_f32<D, false>(lds + wave * (32 * D * 4), st.acc, 1.f, p.o_f32 + row0_elem, (int64_t)p.q_heads * hd, rows,
                                     hd, lane);
        } else {
            store_tile_bf16<D>(lds + wave * (32 * D * 2), st.acc, 1.f, p.o + row0_elem, (int64_t)p.q_heads * hd, rows, hd, lane);
        }
        if (my_row < Lq && hh == 0)
            p.lse[(int64_t)h * p.total_tokens + item.q_start + my_row] =
                (!BLOCK || l_row > 0.f) ? (st.m * c + __log2f(l_row)) * kLn2 : -INFINITY;

    };

    // ---- the persistent loop: the first item is the workgroup's own slot, the others are drawn from its queue
    int slot = blockIdx.x;
    for (;;) {
        const ItemGeom item = load_item<BLOCK>(p.items, p.block_items, slot);
        if (item.tile < 0) break;          // padding at the end of the queue: nothing left
        run_item(item);
        if (tid == 0) next_slot = drawn;
        __syncthreads();                   // publishes next_slot; every wave has left the item's LDS areas
        slot = __builtin_amdgcn_readfirstlane(next_slot);
        if (slot >= p.num_items) break;
    }
    if (tid == 0) queue.leave();
}

hipError_t launch_fwd(const FwdParams& p, int head_dim, int64_t num_items, bool block, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const int workgroups = persistent_grid(num_items, 2);
    if (workgroups <= 0) return hipErrorInvalidDevice;
    const dim3 grid((unsigned)workgroups), threads(kThreads);
    if (tile_width(head_dim) == 128) {
        if (contraction_steps(head_dim) <= 7) {
            // e.g. head_dim 104: the eighth 16-column step of the contraction over head_dim is all padding
            if (block) hipLaunchKernelGGL((fwd_kernel<128, true, 7>), grid, threads, 0, stream, p);
            else hipLaunchKernelGGL((fwd_kernel<128, false, 7>), grid, threads, 0, stream, p);
        } else {
            if (block) hipLaunchKernelGGL((fwd_kernel<128, true>), grid, threads, 0, stream, p);
            else hipLaunchKernelGGL((fwd_kernel<128, false>), grid, threads, 0, stream, p);
        }
    } else {
        if (block) hipLaunchKernelGGL((fwd_kernel<64, true>), grid, threads, 0, stream, p);
        else hipLaunchKernelGGL((fwd_kernel<64, false>), grid, threads, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

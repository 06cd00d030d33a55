// Forward kernel: one workgroup per (sequence, 128-row q tile, q head) work item.
//
// Each of the 4 waves owns 32 query rows.  For every 64-key tile of the causal prefix the
// workgroup stages K and V in LDS (coalesced 16-byte global->LDS copies, double buffered, one
// barrier per tile); each wave computes S^T = K Q^T on MFMA (keys along rows, its queries along
// columns), runs the online-softmax recurrence with one lane per query, and feeds the bf16
// P^T fragments straight back into MFMA as the B operand of O^T += V^T P^T, V^T being read
// from the row-major V tile with the LDS transpose read.
//
// The loop is software-pipelined by one tile: while the VALU works through the softmax step of tile
// kt, the MFMAs of S^T(kt+1) run; then the MFMAs of tile kt's P V.  K therefore runs one tile ahead of
// V in LDS.  Tiles that lie wholly below the diagonal take code without any mask; only the last two
// tiles of an item compare key and row indices.
#include "attn_device.hpp"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

namespace {

template <int D>
struct FwdGeom {
    static constexpr int KK = D / 16;   // k-steps of S^T = K Q^T
    static constexpr int DB = D / 32;   // 32-row blocks of O^T
    static constexpr int kTileBytes = kFwdKTile * D * 2;
};

template <int D>
struct FwdState {
    using G = FwdGeom<D>;
    bf16x8 qf[G::KK];      // this lane's query row (B operand of S^T = K Q^T)
    f32x16 acc[G::DB];     // O^T accumulator
    f32x16 s[2];           // S^T of the current tile (two 32-key blocks)
    float m, l;            // running row max of the raw scores; this lane's share of the running row sum
    int rm[G::KK];         // per-lane LDS offsets of the K fragments (row-major read), block 0 of a tile
    int tr[G::DB][2];      // per-lane LDS offsets of the V^T fragments (transpose read), k-step 0 of a tile
};

__device__ __forceinline__ float pair_max(float x) {
    // v_permlane32_swap: first result = the value held by lane l % 32, second = the value of lane l % 32 + 32
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// One iteration on key tile kt, whose scores are already in st.s:
//   phase A: MFMA S^T(kt+1) = K(kt+1) Q^T   |  VALU: softmax step of tile kt (max, exp2, row sum, bf16 pack)
//   phase B: MFMA O^T += V(kt)^T P^T(kt)
// kbuf: K tile kt+1; vbuf: V tile kt.  MASK: tile kt touches the diagonal (keys beyond a lane's own row get
// weight 0); LAST: there is no tile kt+1.
template <int D, bool MASK, bool LAST>
__device__ __forceinline__ void fwd_iteration(FwdState<D>& st, const char* kbuf, const char* vbuf, float c,
                                              int dkey /* my_row - key0 - 4 * (lane / 32) */) {
    using G = FwdGeom<D>;
    constexpr int KK = G::KK, DB = G::DB;

    // ---------------- phase A
    f32x16 sn[2];
    if constexpr (!LAST) {
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sn[jb][i] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kbuf + st.rm[kk] + jb * 32 * D * 2);
                sn[jb] = mfma(kf, st.qf[kk], sn[jb]);
            }
        }
    }
    if constexpr (MASK) {
        // element i of block jb is key 32 jb + 8 (i / 4) + i % 4 (+ 4 (lane / 32), folded into dkey)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (32 * jb + 8 * (i >> 2) + (i & 3) > dkey) st.s[jb][i] = -INFINITY;
    }
    float tmax = fmaxf(st.s[0][0], st.s[0][1]);
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int i = (jb == 0 ? 2 : 0); i < 16; ++i) tmax = fmaxf(tmax, st.s[jb][i]);
    tmax = pair_max(tmax);
    const float m_new = fmaxf(st.m, tmax);
    const float alpha = fast_exp2((st.m - m_new) * c);
    const bool rescale = __any(m_new > st.m);      // wave-uniform: skip the accumulator rescale when no max moved
    const float mc = m_new * c;
    st.m = m_new;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
        float e[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            e[i] = fast_exp2(fmaf(st.s[jb][i], c, -mc));
            psum += e[i];
        }
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            union { u32x4 u; bf16x8 v; } r;
#pragma unroll
            for (int w = 0; w < 4; ++w) r.u[w] = pack_bf16(e[8 * tt + 2 * w], e[8 * tt + 2 * w + 1]);
            pf[jb * 2 + tt] = r.v;
        }
    }
    st.l = st.l * alpha + psum;
    if constexpr (!LAST) {
        // per MFMA: one K fragment read and a share of the softmax VALU work
        InterleaveHint<2 * KK, 1, (MASK ? 13 : 9), 0>::apply();
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---------------- phase B
    if (rescale) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.acc[db][i] *= alpha;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int off = t * 16 * D * 2;
            const s16x4 lo = lds_transpose_read(vbuf + st.tr[db][0] + off);
            const s16x4 hi = lds_transpose_read(vbuf + st.tr[db][1] + off);
            union { struct { s16x4 a, b; } s; bf16x8 v; } u;
            u.s.a = lo;
            u.s.b = hi;
            st.acc[db] = mfma(u.v, pf[t], st.acc[db]);
        }
    }
    if constexpr (!LAST) {
        st.s[0] = sn[0];
        st.s[1] = sn[1];
    }
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kThreads, 2) void fwd_kernel(FwdParams p) {
    using G = FwdGeom<D>;
    constexpr int BQ = kFwdQTile, BK = kFwdKTile;
    constexpr int KK = G::KK, DB = G::DB;
    constexpr int kTileBytes = G::kTileBytes;
    // K tiles kt+1 / kt+2 and V tiles kt / kt+1: two buffers each
    __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];
    char* const kbuf0 = lds;
    char* const vbuf0 = lds + 2 * kTileBytes;

    const hspmd_work_item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = item.seq_len, h = item.head, hk = h / p.group;
    const int q_row0 = item.tile * BQ;
    const int wave_row0 = q_row0 + wave * 32;
    const int my_row = wave_row0 + (lane & 31);
    const int hh = lane >> 5;

    const uint16_t* qbase = p.q + (int64_t)item.token_start * p.q_stride + (int64_t)h * D;
    const uint16_t* kbase = p.k + (int64_t)item.token_start * p.kv_stride + (int64_t)hk * D;
    const uint16_t* vbase = p.v + (int64_t)item.token_start * p.kv_stride + (int64_t)hk * D;

    const int kv_end = min(L, q_row0 + BQ);
    const int n_tiles = (kv_end + BK - 1) / BK;
    const int n_interior = min(n_tiles, 2 * item.tile);   // tiles whose every key precedes every row of this q tile

    TileCopy<D, BK> kvcopy;   // K and V share stride and geometry
    kvcopy.init(p.kv_stride, wave, lane);
    // K(0), V(0), K(1)
    kvcopy.issue(kbuf0, kbase, p.kv_stride, 0, L, wave, lane);
    kvcopy.issue(vbuf0, vbase, p.kv_stride, 0, L, wave, lane);
    if (n_tiles > 1) kvcopy.issue(kbuf0 + kTileBytes, kbase, p.kv_stride, BK, L, wave, lane);

    FwdState<D> st;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        union { u32x4 u; bf16x8 v; } t;
        t.u = u32x4{0u, 0u, 0u, 0u};
        if (my_row < L) t.u = *reinterpret_cast<const u32x4*>(qbase + (int64_t)my_row * p.q_stride + kk * 16 + hh * 8);
        st.qf[kk] = t.v;
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) st.acc[db][i] = 0.f;
    st.m = -INFINITY;
    st.l = 0.f;
    const float c = p.scale_log2;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) st.rm[kk] = tile_offset<D>(lane & 31, kk * 16 + hh * 8);
    {
        const int c16 = lane & 15;
        const int row = (hh << 2) + (c16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int col = db * 32 + (((lane >> 4) & 1) << 4) + ((c16 & 3) << 2);
            st.tr[db][0] = tile_offset<D>(row, col);
            st.tr[db][1] = tile_offset<D>(row + 8, col);
        }
    }

    wait_tile_loads();
    __syncthreads();
    // S^T(0), not pipelined
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) st.s[jb][i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            st.s[jb] = mfma(*reinterpret_cast<const bf16x8*>(kbuf0 + st.rm[kk] + jb * 32 * D * 2), st.qf[kk], st.s[jb]);
    }

    // iteration kt: K(kt+1) in kbuf[(kt+1) & 1], V(kt) in vbuf[kt & 1]; issues K(kt+2) -> kbuf[kt & 1] and
    // V(kt+1) -> vbuf[(kt+1) & 1], both free since the barrier at the top
    auto step = [&](int kt, auto masked, auto last) {
        if (kt > 0) {
            wait_tile_loads();
            __syncthreads();   // K(kt+1) and V(kt) have landed; every wave is done with iteration kt-1
        }
        if (kt + 2 < n_tiles) kvcopy.issue(kbuf0 + (kt & 1) * kTileBytes, kbase, p.kv_stride, (kt + 2) * BK, L, wave, lane);
        if (kt + 1 < n_tiles) kvcopy.issue(vbuf0 + ((kt + 1) & 1) * kTileBytes, vbase, p.kv_stride, (kt + 1) * BK, L, wave, lane);
        fwd_iteration<D, decltype(masked)::value, decltype(last)::value>(
            st, kbuf0 + ((kt + 1) & 1) * kTileBytes, vbuf0 + (kt & 1) * kTileBytes, c, my_row - kt * BK - 4 * hh);
    };
    // three loops instead of branches inside one: unmasked tiles, masked tiles, and the final tile (which has no
    // successor to compute scores for); the large register state then meets at a join once per loop, not per tile
    const int n_plain = min(n_interior, n_tiles - 1);
    int kt = 0;
    for (; kt < n_plain; ++kt) step(kt, std::false_type{}, std::false_type{});
    for (; kt < n_tiles - 1; ++kt) step(kt, std::true_type{}, std::false_type{});
    step(kt, std::true_type{}, std::true_type{});   // the final tile always touches the diagonal

    const float l_row = st.l + partner32(st.l);
    if (my_row < L) {
        const float inv = 1.f / l_row;
        uint16_t* orow = p.o + ((int64_t)(item.token_start + my_row) * p.q_heads + h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                u32x2 w;
                w[0] = pack_bf16(st.acc[db][4 * i4 + 0] * inv, st.acc[db][4 * i4 + 1] * inv);
                w[1] = pack_bf16(st.acc[db][4 * i4 + 2] * inv, st.acc[db][4 * i4 + 3] * inv);
                *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + hh * 4) = w;
            }
        if (hh == 0) p.lse[(int64_t)h * p.total_tokens + item.token_start + my_row] = (st.m * c + __log2f(l_row)) * kLn2;
    }
}

hipError_t launch_fwd(const FwdParams& p, int head_dim, int64_t num_items, hipStream_t stream) {
    if (num_items == 0) return hipSuccess;
    const dim3 grid((unsigned)num_items), block(kThreads);
    if (head_dim == 128) {
        hipLaunchKernelGGL(fwd_kernel<128>, grid, block, 0, stream, p);
    } else {
        hipLaunchKernelGGL(fwd_kernel<64>, grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace hspmd

// Forward kernel: one workgroup per (sequence, 128-row q tile, q head) work item.
//
// Each of the 4 waves owns 32 query rows.  For every 64-key tile of the causal prefix the
// workgroup stages K and V in LDS (coalesced 16-byte global->LDS copies issued one tile ahead,
// double buffered, one barrier per tile), each wave computes S^T = K Q^T on MFMA (keys along rows, its queries along
// columns), runs the online-softmax recurrence with one lane per query, and feeds the bf16
// P^T fragments straight back into MFMA as the B operand of O^T += V^T P^T, V^T being read
// from the row-major V tile with the LDS transpose read.
#include "attn_device.hpp"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

template <int D>
__global__ __launch_bounds__(kThreads, 2) void fwd_kernel(FwdParams p) {
    constexpr int BQ = kFwdQTile, BK = kFwdKTile;
    constexpr int KK = D / 16;   // k-steps of S^T = K Q^T
    constexpr int DB = D / 32;   // 32-row blocks of O^T
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

    const uint16_t* qbase = p.q + (int64_t)item.token_start * p.q_stride + (int64_t)h * D;
    const uint16_t* kbase = p.k + (int64_t)item.token_start * p.kv_stride + (int64_t)hk * D;
    const uint16_t* vbase = p.v + (int64_t)item.token_start * p.kv_stride + (int64_t)hk * D;

    const int kv_end = min(L, q_row0 + BQ);
    const int n_tiles = (kv_end + BK - 1) / BK;

    TileCopy<D, BK> kvcopy;   // K and V share stride and geometry
    kvcopy.init(p.kv_stride, wave, lane);
    kvcopy.issue(lds, kbase, p.kv_stride, 0, L, wave, lane);
    kvcopy.issue(lds + kTileBytes, vbase, p.kv_stride, 0, L, wave, lane);

    // this lane's query row as B operand fragments (zero for rows past the sequence end)
    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        union { u32x4 u; bf16x8 v; } t;
        t.u = u32x4{0u, 0u, 0u, 0u};
        if (my_row < L) t.u = *reinterpret_cast<const u32x4*>(qbase + (int64_t)my_row * p.q_stride + kk * 16 + hh * 8);
        qf[kk] = t.v;
    }

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;
    float m = -INFINITY;   // running row max of the raw scores <q, k>
    float l = 0.f;         // this lane's share of the running row sum
    const float c = p.scale_log2;

    for (int kt = 0; kt < n_tiles; ++kt) {
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
        // 32-key blocks whose first key is beyond this wave's last query are fully masked
        const int nblk = (key0 > wave_row0 + 31) ? 0 : ((key0 + 32 > wave_row0 + 31) ? 1 : 2);
        if (nblk == 0) continue;

        f32x16 s[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) s[jb][i] = 0.f;
            if (jb < nblk) {
                bf16x8 kf[KK];
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) kf[kk] = read_rowmajor_frag<D>(ktile, jb, kk, lane);
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) s[jb] = mfma(kf[kk], qf[kk], s[jb]);
            }
        }
        // causal mask, only where the block straddles the diagonal
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int kb = key0 + jb * 32;
            if (jb >= nblk) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[jb][i] = -INFINITY;
            } else if (kb + 31 > wave_row0) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (kb + acc_row(i, lane) > my_row) s[jb][i] = -INFINITY;
            }
        }
        float tmax = s[0][0];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, s[jb][i]);
        tmax = fmaxf(tmax, partner32(tmax));
        const float m_new = fmaxf(m, tmax);
        const float alpha = fast_exp2((m - m_new) * c);
        const bool rescale = __any(m_new > m);      // wave-uniform: skip the accumulator rescale when no max moved
        const float mc = m_new * c;
        m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float e = fast_exp2(fmaf(s[jb][i], c, -mc));
                s[jb][i] = e;
                psum += e;
            }
        l = l * alpha + psum;
        if (rescale) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[db][i] *= alpha;
        }
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            if (jb < nblk) {
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const bf16x8 pf = frag_to_bf16(s[jb], tt);
                    bf16x8 vf[DB];
#pragma unroll
                    for (int db = 0; db < DB; ++db) vf[db] = read_transposed_frag<D>(vtile, db, jb * 2 + tt, lane);
#pragma unroll
                    for (int db = 0; db < DB; ++db) acc[db] = mfma(vf[db], pf, acc[db]);
                }
            }
        }
    }

    const float l_row = l + partner32(l);
    if (my_row < L) {
        const float inv = 1.f / l_row;
        uint16_t* orow = p.o + ((int64_t)(item.token_start + my_row) * p.q_heads + h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                u32x2 w;
                w[0] = pack_bf16(acc[db][4 * i4 + 0] * inv, acc[db][4 * i4 + 1] * inv);
                w[1] = pack_bf16(acc[db][4 * i4 + 2] * inv, acc[db][4 * i4 + 3] * inv);
                *reinterpret_cast<u32x2*>(orow + db * 32 + i4 * 8 + hh * 4) = w;
            }
        if (hh == 0) p.lse[(int64_t)h * p.total_tokens + item.token_start + my_row] = (m * c + __log2f(l_row)) * kLn2;
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

// Matrix-core rate probe: back-to-back MFMAs on register operands, no memory traffic.  Gives the rate the
// attention kernels are measured against beside the nominal peak (the shader clock under a pure MFMA load
// is higher than under the attention kernels' mix of MFMA, VALU and LDS work).
#include "attn_device.hpp"
#include "kernels.hpp"

namespace hspmd {

namespace {
static_assert(kProbeThreads == kThreads, "probe workgroups are the kernels' 4 waves");
constexpr int kProbeGroupsPerCu = 2;   // workgroups of 4 waves per compute unit: 2 waves per SIMD
constexpr int kProbeUnroll = 16;
}  // namespace

// VARIED = false: constant operands (1.0 and a small value): few bits toggle between consecutive products.
// VARIED = true: four operand pairs of pseudo-random values in +-[0.5, 2), different in every lane, used in turn:
// the switching activity of real data.  The chip limits its power, so the clock it sustains depends on that.
template <bool VARIED>
__global__ __launch_bounds__(kThreads, 2) void mfma_probe_kernel(float* out, int64_t rounds) {
    union { u32x4 u; bf16x8 v; } a[4], b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if constexpr (VARIED) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // integer hash of (thread, operand, word): sign and the low exponent / mantissa bits of two bf16 values vary
                uint32_t h = (threadIdx.x * 4u + j) * 8u + i;
                h = (h ^ 61u) ^ (h >> 16); h *= 9u; h ^= h >> 4; h *= 0x27d4eb2du; h ^= h >> 15;
                uint32_t g = h * 0x9e3779b9u; g ^= g >> 13;
                a[j].u[i] = (h & 0x80ff80ffu) | 0x3f003f00u;
                b[j].u[i] = (g & 0x80ff80ffu) | 0x3f003f00u;
            }
        } else {
            a[j].u = u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};          // 1.0 x 8
            const uint32_t w = 0x3c003c00u + (threadIdx.x & 3);                         // small values
            b[j].u = u32x4{w, w, w, w};
        }
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int64_t r = 0; r < rounds; ++r) {
#pragma unroll
        for (int j = 0; j < kProbeUnroll; ++j) acc[j & 3] = mfma(a[(j >> 2) & 3].v, b[(j + (j >> 2)) & 3].v, acc[j & 3]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

// Variants of the varied-operand loop, for the questions the attention kernels raise about this chip:
//   SHAPE  32: v_mfma_f32_32x32x16_bf16; 16: v_mfma_f32_16x16x32_bf16 (the same flops per round: 16 or 32 MFMAs)
//   LDSFED the A operand of every product is read from LDS (one 1 KB fragment per 32x32x16 MFMA, or per two 16x16x32
//          MFMAs that share it), as the kernels stream their tiles; B operands stay in registers
//   SLEEP  s_sleep argument after every round of 16 (32) MFMAs = 512 matrix-pipe cycles: idle time of 64 SLEEP clocks
//          (meaningful with one wave per SIMD: launch `compute_units` workgroups)
template <int SHAPE, bool LDSFED, int SLEEP>
__global__ __launch_bounds__(kThreads, 2) void mfma_probe_ex_kernel(float* out, int64_t rounds) {
    __shared__ __attribute__((aligned(1024))) u32x4 frags[LDSFED ? 4096 : 1];   // 64 KB of pseudo-random fragments
    union { u32x4 u; bf16x8 v; } a[4], b[8];
    auto noise = [](uint32_t h) {
        h = (h ^ 61u) ^ (h >> 16); h *= 9u; h ^= h >> 4; h *= 0x27d4eb2du; h ^= h >> 15;
        return h;
    };
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t h = noise((threadIdx.x * 8u + j) * 8u + i);
            b[j].u[i] = (h & 0x80ff80ffu) | 0x3f003f00u;                      // +-[0.5, 2)
            if (j < 4) a[j].u[i] = ((h * 0x9e3779b9u) & 0x80ff80ffu) | 0x3f003f00u;
        }
    if constexpr (LDSFED) {
        for (int i = threadIdx.x; i < 4096; i += kThreads) {
            const uint32_t h = noise(i * 2654435761u);
            frags[i] = u32x4{(h & 0x80ff80ffu) | 0x3f003f00u, ((h * 3u) & 0x80ff80ffu) | 0x3f003f00u,
                             ((h * 5u) & 0x80ff80ffu) | 0x3f003f00u, ((h * 7u) & 0x80ff80ffu) | 0x3f003f00u};
        }
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    if constexpr (SHAPE == 32) {
        f32x16 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
        for (int64_t r = 0; r < rounds; ++r) {
#pragma unroll
            for (int j = 0; j < kProbeUnroll; ++j) {
                union { u32x4 u; bf16x8 v; } f;
                if constexpr (LDSFED) f.u = frags[(r & 3) * 1024 + j * 64 + lane]; else f.v = a[(j >> 2) & 3].v;
                acc[j & 3] = mfma(f.v, b[(j + (j >> 2)) & 7].v, acc[j & 3]);
            }
            if constexpr (SLEEP > 0) __builtin_amdgcn_s_sleep(SLEEP);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) s += acc[j][i];
    } else {
        f32x4 acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int64_t r = 0; r < rounds; ++r) {
#pragma unroll
            for (int j = 0; j < kProbeUnroll; ++j) {
                // one A fragment (16 rows x 32 k) meets two B fragments (two groups of 16 columns)
                union { u32x4 u; bf16x8 v; } f;
                if constexpr (LDSFED) f.u = frags[(r & 3) * 1024 + j * 64 + lane]; else f.v = a[(j >> 2) & 3].v;
                acc[(j & 3) * 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.v, b[j & 3].v, acc[(j & 3) * 2], 0, 0, 0);
                acc[(j & 3) * 2 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.v, b[4 + (j & 3)].v, acc[(j & 3) * 2 + 1], 0, 0, 0);
            }
            if constexpr (SLEEP > 0) __builtin_amdgcn_s_sleep(SLEEP);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) s += acc[j][i];
    }
    out[(int64_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

int probe_grid(int compute_units) { return compute_units * kProbeGroupsPerCu; }

int probe_mode_grid(int mode, int compute_units) {
    return mode >= HSPMD_PROBE_IDLE_0 ? compute_units : compute_units * kProbeGroupsPerCu;   // idle series: one wave per SIMD
}

hipError_t launch_mfma_probe_mode(int mode, float* out, int64_t rounds, int grid, hipStream_t stream) {
    const dim3 g((unsigned)grid), t(kThreads);
    switch (mode) {
        case HSPMD_PROBE_32X32X16_CONSTANT: hipLaunchKernelGGL(mfma_probe_kernel<false>, g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_32X32X16: hipLaunchKernelGGL((mfma_probe_ex_kernel<32, false, 0>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_16X16X32: hipLaunchKernelGGL((mfma_probe_ex_kernel<16, false, 0>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_32X32X16_LDS: hipLaunchKernelGGL((mfma_probe_ex_kernel<32, true, 0>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_16X16X32_LDS: hipLaunchKernelGGL((mfma_probe_ex_kernel<16, true, 0>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_IDLE_0: hipLaunchKernelGGL((mfma_probe_ex_kernel<32, false, 0>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_IDLE_256: hipLaunchKernelGGL((mfma_probe_ex_kernel<32, false, 4>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_IDLE_512: hipLaunchKernelGGL((mfma_probe_ex_kernel<32, false, 8>), g, t, 0, stream, out, rounds); break;
        case HSPMD_PROBE_IDLE_1024: hipLaunchKernelGGL((mfma_probe_ex_kernel<32, false, 16>), g, t, 0, stream, out, rounds); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_mfma_probe(float* out, int64_t rounds, int grid, bool varied_operands, hipStream_t stream) {
    if (varied_operands) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)grid), dim3(kThreads), 0, stream, out, rounds);
    else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)grid), dim3(kThreads), 0, stream, out, rounds);
    return hipGetLastError();
}

}  // namespace hspmd

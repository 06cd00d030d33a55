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

int probe_grid(int compute_units) { return compute_units * kProbeGroupsPerCu; }

hipError_t launch_mfma_probe(float* out, int64_t rounds, int grid, bool varied_operands, hipStream_t stream) {
    if (varied_operands) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)grid), dim3(kThreads), 0, stream, out, rounds);
    else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)grid), dim3(kThreads), 0, stream, out, rounds);
    return hipGetLastError();
}

}  // namespace hspmd

// Measures what the matrix pipe delivers: a register-only loop of independent
// v_mfma_f32_32x32x2_f32 chains, optionally with ordinary vector FMAs interleaved.  Gives the
// on-box fp32 MFMA ceiling the roofline fractions are quoted against, and shows how much matrix
// throughput every extra vector instruction in a main loop costs.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace ucd {

typedef float f32x16 __attribute__((ext_vector_type(16)));

// NACC accumulator tiles per wave: 4 (64 registers, several waves per SIMD) or 16 (256 registers,
// one wave per SIMD: the situation of a kernel that keeps all 16 Winograd points of a tile resident).
// REP > 1: every accumulator takes REP consecutive MFMAs (each depends on the one before it) before
// the next accumulator's turn, as in a loop that walks the reduction index innermost.
template <int VALU, int NACC, int REP = 1>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *out, int iters, float seed)
{
    f32x16 acc[NACC];
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float a = seed + threadIdx.x, b = seed * 2 + threadIdx.x;
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = seed + i + threadIdx.x;
    for (int it = 0; it < iters; it += REP) {   // 16 * REP MFMAs per trip
#pragma unroll
        for (int u = 0; u < 16 / NACC; ++u)
#pragma unroll
            for (int i = 0; i < NACC; ++i)
#pragma unroll
                for (int r = 0; r < REP; ++r) {
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < VALU; ++v) x[v] = x[v] * 1.0001f + 0.5f;
                }
    }
    float s = 0;
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    for (int i = 0; i < 8; ++i) s += x[i];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// out must hold blocks * 256 floats.  flops counted: blocks * 4 waves * iters * 16 MFMAs * 4096.
// valu_per_mfma: 0, 2, 4, 8 (4 accumulator tiles per wave), 100 + {0, 2, 4} (16 tiles per wave), or
// 200 + {0, 2} (16 tiles per wave, 4 consecutive MFMAs per tile; iters must be a multiple of 4).
hipError_t mfma_probe(int valu_per_mfma, int blocks, int iters, float *out, hipStream_t s)
{
    switch (valu_per_mfma) {
    case 0: mfma_probe_kernel<0, 4><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 2: mfma_probe_kernel<2, 4><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 4: mfma_probe_kernel<4, 4><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 8: mfma_probe_kernel<8, 4><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 100: mfma_probe_kernel<0, 16><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 102: mfma_probe_kernel<2, 16><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 104: mfma_probe_kernel<4, 16><<<blocks, 256, 0, s>>>(out, iters, 1.f); break;
    case 200:
    case 202:
        if (iters % 4) return hipErrorInvalidValue;
        if (valu_per_mfma == 200) mfma_probe_kernel<0, 16, 4><<<blocks, 256, 0, s>>>(out, iters, 1.f);
        else mfma_probe_kernel<2, 16, 4><<<blocks, 256, 0, s>>>(out, iters, 1.f);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace ucd

// 16-point complex FFT in registers (radix-2, decimation in time, fully unrolled: every index and
// twiddle is a compile-time constant).  SIGN = -1: X[u] = sum_i x[i] e^{-2 pi i u i / 16};
// SIGN = +1: the same sum with e^{+...} (the unnormalised inverse).
#pragma once

#if defined(__HIPCC__)
#define UCD_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define UCD_HD inline
#endif

namespace ucd {

template <int SIGN>
UCD_HD void fft16(float (&re)[16], float (&im)[16])
{
    constexpr int rev[16] = {0, 8, 4, 12, 2, 10, 6, 14, 1, 9, 5, 13, 3, 11, 7, 15};
    // cos and sin of 2 pi k / 16, k = 0..7
    constexpr float kc[8] = {1.f, 0.9238795325112867f, 0.7071067811865476f, 0.3826834323650898f,
                             0.f, -0.3826834323650898f, -0.7071067811865476f, -0.9238795325112867f};
    constexpr float ks[8] = {0.f, 0.3826834323650898f, 0.7071067811865476f, 0.9238795325112867f,
                             1.f, 0.9238795325112867f, 0.7071067811865476f, 0.3826834323650898f};
    float tr[16], ti[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        tr[i] = re[rev[i]];
        ti[i] = im[rev[i]];
    }
#pragma unroll
    for (int len = 2; len <= 16; len <<= 1) {
#pragma unroll
        for (int i = 0; i < 16; i += len) {
#pragma unroll
            for (int k = 0; k < len / 2; ++k) {
                const int tw = k * (16 / len);
                const float c = kc[tw], s = SIGN * ks[tw];
                const int a = i + k, b = i + k + len / 2;
                const float xr = tr[b] * c - ti[b] * s, xi = tr[b] * s + ti[b] * c;
                tr[b] = tr[a] - xr;
                ti[b] = ti[a] - xi;
                tr[a] += xr;
                ti[a] += xi;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        re[i] = tr[i];
        im[i] = ti[i];
    }
}

}  // namespace ucd

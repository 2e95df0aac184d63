// Philox4x32-10 counter stream and Box-Muller normals: the device code behind dp_add_noise, shared by every kernel
// that adds the noise while it holds the sums (one definition, so that all of them produce the same bits).
#pragma once
#include "dp_common.h"
#include "dp_internal.h"

namespace dpk {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11) and Box-Muller normals.
// ---------------------------------------------------------------------------
struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    return U4{c0, c1, c2, c3};
}

// u = ((w >> 9) + 1/2) / 2^23, exact in float32 and strictly inside (0, 1)
__device__ __forceinline__ float uniform23(uint32_t w) { return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f; }

__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float& z_even, float& z_odd) {
    const float r = sqrtf(-2.0f * logf(uniform23(wa)));
    float s, c;
    sincospif(2.0f * uniform23(wb), &s, &c);
    z_even = r * c;
    z_odd = r * s;
}

// The four normals of Philox block q = (offset + j) / 4, scaled: what k_add_noise adds to grad[j .. j + 3] when
// offset + j is a multiple of 4.  Used by the split-K reduce kernels to add the noise while the sums are in
// registers (same values, same single multiply-add per element as the stand-alone kernel).
__device__ __forceinline__ void add_noise4(float4& g, uint64_t q, const NoiseArgs& nz) {
    const U4 w = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, nz.k0, nz.k1);
    float z[4];
    box_muller(w.x, w.y, z[0], z[1]);
    box_muller(w.z, w.w, z[2], z[3]);
    g.x += nz.stddev * z[0]; g.y += nz.stddev * z[1]; g.z += nz.stddev * z[2]; g.w += nz.stddev * z[3];
}

}  // namespace dpk

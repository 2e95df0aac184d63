// Device-side helpers shared by the dpclip kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dpk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;
constexpr int kThreads = 256;   // every tiled kernel runs 4 waves per workgroup

__device__ __forceinline__ float bf16_lo(uint32_t d) { return __uint_as_float(d << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t d) { return __uint_as_float(d & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32); lo in bits 15:0.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// The two 16-bit input formats of the MFMA kernels.  The kernels move the 16-bit values as bits (typed bf16x8
// whatever the format); only these four operations look inside them.
template <bool F16> struct In16;
template <> struct In16<false> {                   // bfloat16
    static __device__ __forceinline__ float lo(uint32_t d) { return bf16_lo(d); }
    static __device__ __forceinline__ float hi(uint32_t d) { return bf16_hi(d); }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return pack_bf16(lo, hi); }
    static __device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {      // 16 x 16 tile, 32 deep
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct In16<true> {                    // IEEE half
    static __device__ __forceinline__ float lo(uint32_t d) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(d & 0xffffu)); }
    static __device__ __forceinline__ float hi(uint32_t d) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(d >> 16)); }
    // round to nearest even, lo in bits 15:0
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
    static __device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};

// (a.lo16, b.lo16) and (a.hi16, b.hi16) packs, a in the low half of the result.
__device__ __forceinline__ uint32_t pack_lo16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// nu = 1 / max(1, sqrt(s) / C)   (clip function of Section 3.2); the max lets a NaN norm through
__device__ __forceinline__ float clip_factor_of(float s, float C) {
    const float m = sqrtf(s) / C;
    return 1.0f / (!(m <= 1.0f) ? m : 1.0f);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Sum over the 256 threads of a workgroup in a fixed order; result valid in thread 0.
// `red` is 4 floats of LDS.  Callers must not reuse `red` before a barrier.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// LDS tile layout used by the bf16 MFMA kernels: rows of 64 bf16 (128 B = 8
// chunks of 16 B).  Chunk c of row r lives at chunk position c ^ swz(r), so
// that the 16 B-per-lane reads of 16 consecutive rows hit 16 distinct bank
// groups (row parity picks the upper/lower 32 banks, the xor spreads the rest).
__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 4)) & 7; }
__device__ __forceinline__ int lds_off_bytes(int row, int chunk) { return row * 128 + ((chunk ^ swz(row)) << 4); }

}  // namespace dpk

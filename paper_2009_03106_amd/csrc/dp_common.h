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

// (a.lo16, b.lo16) and (a.hi16, b.hi16) packs, a in the low half of the result.
__device__ __forceinline__ uint32_t pack_lo16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

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

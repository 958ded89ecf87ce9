// Device-side building blocks shared by the libapms kernels (gfx950, wave64).
//
// Tile layout.  A workgroup of 256 threads (4 waves) handles a tile of 4096
// consecutive elements of one chunk per iteration; each wave owns 1024 of them
// (32 sign words).  Inside a wave, lane l and row r (r = 0..3) own the four
// consecutive elements starting at
//       128*(l>>3) + 32*r + 4*(l&7)
// so the eight lanes of a group (l>>3) cover exactly one 32-element sign word
// per row, and the four rows of a group are four CONSECUTIVE words.  Every
// 128-bit load instruction of a wave therefore touches eight fully used 128-byte
// segments, and after an OR across the 8-lane group the group leader stores the
// four words of its rows as one 128-bit store (128 contiguous bytes per wave).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apms {

constexpr int kThreads = 256;
constexpr int kWaveSize = 64;
constexpr int kWaves = kThreads / kWaveSize;
constexpr int kRows = 4;                              // 128-bit rows per lane per tile
constexpr int kWaveTile = kWaveSize * 4 * kRows;      // 1024 elements = 32 words
constexpr int kTile = kWaves * kWaveTile;             // 4096 elements

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Offset of (wave, lane, row 0) inside a tile; row r adds 32*r.
__device__ __forceinline__ int lane_base_offset(int wave, int lane) {
    return wave * kWaveTile + (lane >> 3) * 128 + (lane & 7) * 4;
}

// Streaming (read-once / write-once) 128-bit accesses.
__device__ __forceinline__ f32x4 load_stream(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ void store_stream(float* p, f32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}

// +s where the bit is set, -s where it is clear.
__device__ __forceinline__ float signed_scale(bool positive, float s) {
    return positive ? s : -s;
}

// Sign nibble of four elements: bit c = (u[c] >= 0), so -0.0 and +0.0 give 1.
__device__ __forceinline__ uint32_t sign_nibble(f32x4 u) {
    return (u.x >= 0.0f ? 1u : 0u) | (u.y >= 0.0f ? 2u : 0u) |
           (u.z >= 0.0f ? 4u : 0u) | (u.w >= 0.0f ? 8u : 0u);
}

// OR across the 8 lanes of a group; every lane of the group gets the result.
__device__ __forceinline__ uint32_t or_across_group8(uint32_t v) {
    v |= static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 1));
    v |= static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 2));
    v |= static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), 4));
    return v;
}

// Sum of one binary64 value per thread over the workgroup, in a fixed order:
// butterfly-free shuffle tree inside each wave (offsets 32,16,...,1), then the
// four wave sums added in wave order by thread 0.  Valid result in thread 0.
__device__ __forceinline__ double block_sum_f64(double v, double* lds /* kWaves doubles */) {
#pragma unroll
    for (int off = kWaveSize / 2; off > 0; off >>= 1)
        v += __shfl_down(v, off);
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += lds[w];
    }
    __syncthreads();
    return total;
}

}  // namespace apms

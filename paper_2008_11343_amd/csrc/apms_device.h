// Device-side building blocks shared by the libapms kernels (gfx950, wave64).
//
// Two ways of laying a tile of kThreads*4*ROWS consecutive elements over a workgroup:
//
//  * packing layout (kernels that PRODUCE sign words).  Each wave owns 256*ROWS consecutive
//    elements; lane l and row r (r < ROWS) own the four consecutive elements starting at
//        32*ROWS*(l>>3) + 32*r + 4*(l&7)
//    so the eight lanes of a group (l>>3) cover exactly one 32-element sign word per row, and the
//    ROWS rows of a group are ROWS CONSECUTIVE words.  Every 128-bit load of a wave touches eight
//    fully used 128-byte segments; after an OR across the 8-lane group the group leader stores its
//    ROWS words with one wide store.
//
//  * plain layout (kernels that only READ sign words).  Row r of thread t starts at element
//    r*kThreads*4 + 4*t: every wave access is 1 KB contiguous; the thread's four elements sit at bit
//    4*(t&7) of word (offset >> 5).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "apms_launch.h"

namespace apms {

constexpr int kWaveSize = 64;
constexpr int kWaves = kThreads / kWaveSize;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Packing layout: offset of (wave, lane, row 0) inside a tile; row r adds 32*r.
template <int ROWS>
__device__ __forceinline__ int packing_lane_offset(int wave, int lane) {
    return wave * (kWaveSize * 4 * ROWS) + (lane >> 3) * (32 * ROWS) + (lane & 7) * 4;
}

// Streaming (read-once / write-once) 128-bit accesses.
__device__ __forceinline__ f32x4 load_stream(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ void store_stream(float* p, f32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}

// Four consecutive gradient values starting at element p, widened to binary32 (exact for both 16-bit
// formats: binary16 through the hardware conversion, bfloat16 by placing its bits in the upper half).
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));
template <int G>
__device__ __forceinline__ f32x4 load_grad4(const void* g, int64_t p) {
    if constexpr (G == kGradF32) {
        return load_stream(static_cast<const float*>(g) + p);
    } else if constexpr (G == kGradF16) {
        const f16x4 h = __builtin_nontemporal_load(reinterpret_cast<const f16x4*>(static_cast<const _Float16*>(g) + p));
        return f32x4{static_cast<float>(h.x), static_cast<float>(h.y), static_cast<float>(h.z), static_cast<float>(h.w)};
    } else {
        const u16x4 h = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(static_cast<const uint16_t*>(g) + p));
        f32x4 out;
#pragma unroll
        for (int c = 0; c < 4; ++c) out[c] = __builtin_bit_cast(float, static_cast<uint32_t>(h[c]) << 16);
        return out;
    }
}

// +s where the bit is set, -s where it is clear.
__device__ __forceinline__ float signed_scale(bool positive, float s) {
    return positive ? s : -s;
}

// |s| with the sign bit taken from the top bit of t (set = negative).  s is a chunk scale, a square root,
// hence never negative, so this equals signed_scale(!(t >> 31), s).
__device__ __forceinline__ float scale_signed_by_msb(uint32_t t, float s) {
    return __builtin_bit_cast(float, (__builtin_bit_cast(uint32_t, s) & 0x7fffffffu) | (t & 0x80000000u));
}

// The same as ONE VALU instruction (bit-field insert: magnitude bits from s, sign bit from t), for the server
// kernel's inner loop, where this runs once per worker and element; written as C++ it compiles to an AND and
// an OR.  `magnitude_bits` must hold 0x7fffffff; it and s are taken in vector registers because an
// instruction may read only one value from the scalar side.
__device__ __forceinline__ float scale_signed_by_msb_bfi(uint32_t magnitude_bits, float s, uint32_t t) {
    float out;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(out) : "v"(magnitude_bits), "v"(s), "v"(t));
    return out;
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

// The leader of an 8-lane group stores the ROWS consecutive sign words of its rows, starting at
// word index w0: wide stores when the tile is full and w0 is suitably aligned, else word by word.
template <int ROWS, bool kFull>
__device__ __forceinline__ void store_group_words(uint32_t* __restrict__ dst, int64_t w0,
                                                  const uint32_t (&words)[ROWS], const bool (&ok)[ROWS]) {
    if constexpr (ROWS % 4 == 0) {
        if (kFull && (w0 & 3) == 0) {
#pragma unroll
            for (int r = 0; r < ROWS; r += 4) {
                u32x4 pk = {words[r], words[r + 1], words[r + 2], words[r + 3]};
                *reinterpret_cast<u32x4*>(dst + w0 + r) = pk;
            }
            return;
        }
    } else if constexpr (ROWS == 2) {
        if (kFull && (w0 & 1) == 0) {
            u32x2 pk = {words[0], words[1]};
            *reinterpret_cast<u32x2*>(dst + w0) = pk;
            return;
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        if (ok[r]) dst[w0 + r] = words[r];
}

// Sum of one binary64 value per thread over the workgroup, in a fixed order: shuffle tree inside each
// wave (offsets 32,16,...,1), then the wave sums added in wave order by thread 0.  Valid in thread 0.
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

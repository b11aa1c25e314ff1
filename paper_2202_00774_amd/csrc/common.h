// Shared device/host helpers of the SDGP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sdgp.h"

namespace sdgp {

// ---------------------------------------------------------------- bit casts

__host__ __device__ __forceinline__ float bits_to_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__host__ __device__ __forceinline__ uint32_t float_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// bfloat16 is the upper half of a binary32.
__host__ __device__ __forceinline__ float bf16_to_float(uint32_t h) { return bits_to_float(h << 16); }

// binary32 -> bfloat16 bits, round to nearest, ties to even; NaN stays NaN.
__host__ __device__ __forceinline__ uint32_t float_to_bf16(float f) {
    uint32_t u = float_to_bits(f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : r;
}

// Two binary32 values -> two bfloat16 in one dword (first value in the low half), round to nearest even.  On the
// device this is one v_cvt_pk_bf16_f32; the same bits as float_to_bf16 for every finite input.
__host__ __device__ __forceinline__ uint32_t float2_to_bf16x2(float lo, float hi) {
#if defined(__HIP_DEVICE_COMPILE__)
    typedef float sdgp_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 sdgp_bf16x2 __attribute__((ext_vector_type(2)));
    const sdgp_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, sdgp_bf16x2));
#else
    return float_to_bf16(lo) | (float_to_bf16(hi) << 16);
#endif
}

// ------------------------------------------------------- counter-based hash
//
// Key of flat element e under `seed` for the random pruning function
// (Sec. III-B, "Random"; the paper names no generator, this is the library's
// definition).  With x = low and y = high word of e, s0/s1 the words of seed:
//   v = 0xA54FF53A ^ (x >> 2) ^ s0*0x9E3779B9 ^ y*0xBB67AE85 ^ s1*0x510E527F
//   v ^= v>>16; v *= 0x6A09E667; v ^= v>>15; v *= 0xBB67AE85; v ^= v>>16
//   key = (v rotated left by 8 * (x & 3) bits) with the low four bits cleared
// One mixed word serves an aligned quad of elements (hash_quad), each element
// taking one of its four byte rotations: two multiplies per quad instead of per
// element.  A key is 28 bits wide (equal keys tie, the lower position wins): the kernels put a 4-bit position code
// below it and rank single 32-bit words.  The seed terms are folded on the host (seed_mix), the y term once
// per group (hash_row).

__host__ __device__ inline uint32_t seed_mix(uint64_t seed) {
    return 0xA54FF53Au ^ ((uint32_t)seed * 0x9E3779B9u) ^ ((uint32_t)(seed >> 32) * 0x510E527Fu);
}

__host__ __device__ __forceinline__ uint32_t hash_row(uint32_t mix, uint32_t e_hi) { return mix ^ (e_hi * 0xBB67AE85u); }

// The mixed word of the quad that holds element e_lo.
__host__ __device__ __forceinline__ uint32_t hash_quad(uint32_t row, uint32_t e_lo) {
    uint32_t v = row ^ (e_lo >> 2);
    v ^= v >> 16;
    v *= 0x6A09E667u;
    v ^= v >> 15;
    v *= 0xBB67AE85u;
    v ^= v >> 16;
    return v;
}

// Key of element i (0..3) of a quad from the quad's mixed word.
__host__ __device__ __forceinline__ uint32_t hash_lane(uint32_t quad_word, uint32_t i) {
    return __builtin_rotateleft32(quad_word, 8u * (i & 3u)) & 0xFFFFFFF0u;
}

__host__ __device__ __forceinline__ uint32_t hash_elem(uint32_t row, uint32_t e_lo) {
    return hash_lane(hash_quad(row, e_lo), e_lo);
}

// ------------------------------------------------------------ host helpers

inline bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Consumes and maps the HIP error state after a launch.
inline int launch_status() { return hipGetLastError() == hipSuccess ? SDGP_OK : SDGP_ERR_HIP; }

}  // namespace sdgp

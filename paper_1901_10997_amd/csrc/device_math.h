// Device-side helpers: gate nonlinearities, bf16 rounding, wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace l355 {

__device__ __forceinline__ float sigmoidf_fast(float z) { return 1.0f / (1.0f + __expf(-z)); }

// tanh(z) = 1 - 2 / (1 + e^{2z}); saturates cleanly to +-1 when e^{2z} overflows or underflows.
__device__ __forceinline__ float tanhf_fast(float z) { return 1.0f - 2.0f / (1.0f + __expf(2.0f * z)); }

// nearest-even rounding of an fp32 value to bf16 precision, result kept in fp32 (finite inputs)
__device__ __forceinline__ float round_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    return __uint_as_float(u);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// sum over the 64 lanes of a wavefront; every lane receives the total
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum four per-lane values over the wavefront with 7 exchanges instead of 24: lanes first split the four
// values between the two halves (and then the quarters) of the wave, then finish with a 16-lane butterfly.
// On return every lane of quarter q = lane/16 holds the total of value q; r[0..3] receive all four totals
// (wave-uniform) through lane reads.
__device__ __forceinline__ void wave_sum4(float a0, float a1, float a2, float a3, float r[4])
{
    const int lane = __lane_id();
    const bool hi32 = (lane & 32) != 0;
    // halves: lower keeps (a0,a1), upper keeps (a2,a3)
    float keep0 = hi32 ? a2 : a0, keep1 = hi32 ? a3 : a1;
    float send0 = hi32 ? a0 : a2, send1 = hi32 ? a1 : a3;
    keep0 += __shfl_xor(send0, 32, 64);
    keep1 += __shfl_xor(send1, 32, 64);
    // quarters: within a half, lanes with bit 4 clear keep the first value
    const bool hi16 = (lane & 16) != 0;
    float keep = hi16 ? keep1 : keep0;
    float send = hi16 ? keep0 : keep1;
    keep += __shfl_xor(send, 16, 64);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) keep += __shfl_xor(keep, off, 64);
    r[0] = __shfl(keep, 0, 64);
    r[1] = __shfl(keep, 16, 64);
    r[2] = __shfl(keep, 32, 64);
    r[3] = __shfl(keep, 48, 64);
}

}  // namespace l355

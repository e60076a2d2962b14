// Device-side helpers: gate nonlinearities, bf16 rounding, wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace l355 {

// Gate nonlinearities from the hardware exp2 and reciprocal (each accurate to about 1 ulp, which keeps the
// absolute error of sigmoid and tanh near 1e-7).
// sigmoid(z) = 1 / (1 + 2^(-z log2 e))
__device__ __forceinline__ float sigmoidf_fast(float z)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}
// tanh(z) = 1 - 2 / (1 + e^{2z}); saturates cleanly to +-1 when e^{2z} overflows or underflows.
__device__ __forceinline__ float tanhf_fast(float z)
{
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.8853900817779268f * z));
}

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

// v + (v moved by the DPP control CTRL): one step of a butterfly inside a 16-lane row
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// v[p] (p = 0..15) holds this lane's partial sum of quantity p.  Returns, in lane l of every 16-lane row, the sum of
// v[l] over the 16 lanes of the row.  Four stages: the lanes are paired by row mirror (l ^ 15), half-row mirror (l ^ 7),
// quad mirror (l ^ 3) and neighbour swap (l ^ 1) -- together they reach all 16 lanes -- and after adding its partner's
// value a lane keeps the quantities whose index bit 3, 2, 1, 0 equals its own lane-index bit (which differs between the
// two partners in every stage), so the registers halve: 8, 4, 2, 1.
__device__ __forceinline__ float row16_transpose_sum(const float (&v)[16], int lane_in_row)
{
    float a[8], b[4], c[2];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const float lo = dpp_add<0x140>(v[p]), hi = dpp_add<0x140>(v[p + 8]);
        // lanes 8..15 (DPP banks 2, 3) take the upper eight quantities
        a[p] = __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(lo), __float_as_int(hi), 0xE4, 0xF, 0xC, false));
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float lo = dpp_add<0x141>(a[p]), hi = dpp_add<0x141>(a[p + 4]);
        // lanes 4..7 and 12..15 (banks 1, 3)
        b[p] = __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(lo), __float_as_int(hi), 0xE4, 0xF, 0xA, false));
    }
    const bool b1 = (lane_in_row & 2) != 0, b0 = (lane_in_row & 1) != 0;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float lo = dpp_add<0x1B>(b[p]), hi = dpp_add<0x1B>(b[p + 2]);   // quad_perm [3,2,1,0]
        c[p] = b1 ? hi : lo;
    }
    const float lo = dpp_add<0xB1>(c[0]), hi = dpp_add<0xB1>(c[1]);           // quad_perm [1,0,3,2]
    return b0 ? hi : lo;
}

// Sum four per-lane values over the wavefront: returns a register in which every lane of row q (lanes
// 16q..16q+15) holds the wave-wide total of a_q.  The four values are first distributed over the four 16-lane
// rows with the gfx950 lane-swap instructions (lanes 32..63 of one register against lanes 0..31 of another, then
// odd rows against even rows), each swap halving the number of lanes a value occupies while adding the halves; a
// 16-lane DPP butterfly (quad swaps, half-row mirror, row mirror) finishes it.  Ten vector instructions, no LDS.
__device__ __forceinline__ float wave_sum4_rows(float a0, float a1, float a2, float a3)
{
    const auto s02 = __builtin_amdgcn_permlane32_swap(__float_as_uint(a0), __float_as_uint(a2), false, false);
    const auto s13 = __builtin_amdgcn_permlane32_swap(__float_as_uint(a1), __float_as_uint(a3), false, false);
    const float k02 = __uint_as_float(s02[0]) + __uint_as_float(s02[1]);
    const float k13 = __uint_as_float(s13[0]) + __uint_as_float(s13[1]);
    const auto sr = __builtin_amdgcn_permlane16_swap(__float_as_uint(k02), __float_as_uint(k13), false, false);
    float v = __uint_as_float(sr[0]) + __uint_as_float(sr[1]);
    v = dpp_add<0xB1>(v);
    v = dpp_add<0x4E>(v);
    v = dpp_add<0x141>(v);
    v = dpp_add<0x140>(v);
    return v;
}

__device__ __forceinline__ float lane_read(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Gate nonlinearities with the four gates of one hidden unit spread over the four 16-lane rows of a wave
// (row 0 forget, 1 input, 2 output: sigmoid; row 3 candidate: tanh), so that one exp2 and one reciprocal
// serve all four.  gate = A + Bm / (1 + 2^(sc * pre)) with (sc, A, Bm) = (-log2 e, 0, 1) for the sigmoid rows
// and (2 log2 e, 1, -2) for the tanh row.  Then the cell update of the paper's Section 4:
// c <- f*c + i*g, h = o*tanh(c).  pre: per-lane pre-activation (row q: gate q).  Returns h; c is updated.
__device__ __forceinline__ float lstm_cell_rows(float pre, int lane, float& c)
{
    const bool cand = lane >= 48;
    const float sc = cand ? 2.8853900817779268f : -1.4426950408889634f;
    const float rr = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc * pre));
    const float gate = cand ? fmaf(-2.0f, rr, 1.0f) : rr;
    const float f = lane_read(gate, 0), i = lane_read(gate, 16), o = lane_read(gate, 32), g = lane_read(gate, 48);
    c = fmaf(f, c, i * g);
    return o * tanhf_fast(c);
}

}  // namespace l355

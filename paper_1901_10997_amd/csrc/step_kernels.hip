// One LSTM timestep per launch: recurrent product W_h.h_{t-1}, gate nonlinearities, cell and hidden update
// (paper Section 4, cell equations).  This is the shape-agnostic path: any H, any B, dense or row-compressed W_h.
// One wavefront owns one hidden unit (its four packed gate rows) for a tile of BT batch columns; lanes split the
// reduction dimension and combine with cross-lane exchanges, so no atomics and a fixed summation order.
#include "common.h"
#include "device_math.h"

namespace l355 {

constexpr int BT = 4;  // batch columns per wave

__device__ __forceinline__ void cell_update_and_store(const StepArgs& a, int j, int b, const float pre[4])
{
    const float4 p = *reinterpret_cast<const float4*>(a.P + ((size_t)a.t * a.B + b) * (4 * (size_t)a.H) + 4 * j);
    const float f = sigmoidf_fast(pre[0] + p.x);
    const float i = sigmoidf_fast(pre[1] + p.y);
    const float o = sigmoidf_fast(pre[2] + p.z);
    const float g = tanhf_fast(pre[3] + p.w);
    const size_t ci = (size_t)b * a.H + j;
    const float cn = f * a.c[ci] + i * g;
    const float hn = o * tanhf_fast(cn);
    a.c[ci] = cn;
    a.y_t[(size_t)b * a.y_ld + j] = hn;
    if (a.last) {
        if (a.hT) a.hT[ci] = hn;
        if (a.cT) a.cT[ci] = cn;
    }
}

template <typename TW>
__device__ __forceinline__ float w_to_f32(TW w);
template <>
__device__ __forceinline__ float w_to_f32<float>(float w) { return w; }
template <>
__device__ __forceinline__ float w_to_f32<uint16_t>(uint16_t w) { return bf16_bits_to_f32(w); }

template <typename TW>
__global__ __launch_bounds__(256) void step_dense_kernel(StepArgs a, const TW* __restrict__ Wh)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= a.H) return;  // whole wave leaves together
    const int b0 = blockIdx.y * BT;
    float acc[4][BT];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < BT; ++i) acc[q][i] = 0.f;
    if (a.h_prev) {
        const TW* w = Wh + (size_t)(4 * j) * a.H;
        for (int k = lane; k < a.H; k += 64) {
            float wv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) wv[q] = w_to_f32<TW>(w[(size_t)q * a.H + k]);
#pragma unroll
            for (int i = 0; i < BT; ++i) {
                const int b = b0 + i;
                float hv = (b < a.B) ? a.h_prev[(size_t)b * a.h_prev_ld + k] : 0.f;
                if (a.round_h_bf16) hv = round_bf16(hv);
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q][i] = fmaf(wv[q], hv, acc[q][i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < BT; ++i) {
        float pre[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) pre[q] = wave_sum(acc[q][i]);
        if (lane == 0 && b0 + i < a.B) cell_update_and_store(a, j, b0 + i, pre);
    }
}

__global__ __launch_bounds__(256) void step_csr_kernel(StepArgs a, const int32_t* __restrict__ row_ptr,
                                                       const uint16_t* __restrict__ col, const float* __restrict__ val)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= a.H) return;
    const int b0 = blockIdx.y * BT;
    float acc[4][BT];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < BT; ++i) acc[q][i] = 0.f;
    if (a.h_prev) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int beg = row_ptr[4 * j + q], end = row_ptr[4 * j + q + 1];
            for (int e = beg + lane; e < end; e += 64) {
                const float wv = val[e];
                const int k = col[e];
#pragma unroll
                for (int i = 0; i < BT; ++i) {
                    const int b = b0 + i;
                    float hv = (b < a.B) ? a.h_prev[(size_t)b * a.h_prev_ld + k] : 0.f;
                    if (a.round_h_bf16) hv = round_bf16(hv);
                    acc[q][i] = fmaf(wv, hv, acc[q][i]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < BT; ++i) {
        float pre[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) pre[q] = wave_sum(acc[q][i]);
        if (lane == 0 && b0 + i < a.B) cell_update_and_store(a, j, b0 + i, pre);
    }
}

hipError_t launch_step_dense(const StepArgs& a, const void* Wh, bool w_bf16, hipStream_t s)
{
    if (a.B <= 0 || a.H <= 0) return hipSuccess;
    dim3 grid((a.H + 3) / 4, (a.B + BT - 1) / BT), block(256);
    if (w_bf16)
        hipLaunchKernelGGL(step_dense_kernel<uint16_t>, grid, block, 0, s, a, (const uint16_t*)Wh);
    else
        hipLaunchKernelGGL(step_dense_kernel<float>, grid, block, 0, s, a, (const float*)Wh);
    return hipGetLastError();
}

hipError_t launch_step_csr(const StepArgs& a, const int32_t* row_ptr, const uint16_t* col, const float* val,
                           hipStream_t s)
{
    if (a.B <= 0 || a.H <= 0) return hipSuccess;
    dim3 grid((a.H + 3) / 4, (a.B + BT - 1) / BT), block(256);
    hipLaunchKernelGGL(step_csr_kernel, grid, block, 0, s, a, row_ptr, col, val);
    return hipGetLastError();
}

}  // namespace l355

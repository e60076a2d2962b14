// Shape-agnostic kernels of the H-LSTM cell (paper Section 4, cell equations with one hidden layer inside each
// gate), one timestep per pair of launches:
//   stage 1   u[b][r] = relu( P1[t][b][r] + sum_k W1h[r][k] * h_{t-1}[b][k] )        r over the 4G hidden-layer rows
//   stage 2   a_q = b2[4j+q] + sum_g W2[4j+q][g] * u[b][4g+q];  f,i,o = sigmoid, g = tanh;
//             c <- f*c + i*g;  h = o*tanh(c)
// P1 = W1x.x + b1 comes from the projection kernels.  Rows are packed: row 4g+q of W1h / P1 / u is hidden unit g of
// gate q, row 4j+q of W2 / b2 is output j of gate q; gate q reads the hidden layer of gate q only, i.e. the entries
// u[4g+q].  One wave per row (stage 1) or per hidden unit (stage 2), BT batch columns per wave; matrices dense or
// row-compressed (row_ptr / 16-bit columns / values).  These are the correctness net and the path for shapes the
// persistent H-LSTM kernel does not cover.
#include "common.h"
#include "device_math.h"

namespace l355 {

namespace {
constexpr int HBT = 4;  // batch columns per wave
}

__global__ __launch_bounds__(256) void hstage1_kernel(HStage1Args a)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int R = 4 * a.G;
    if (r >= R) return;  // whole wave leaves together
    const int b0 = blockIdx.y * HBT;
    float acc[HBT];
#pragma unroll
    for (int i = 0; i < HBT; ++i) acc[i] = 0.f;
    if (a.h_prev) {
        if (a.w_dense) {
            const float* w = a.w_dense + (size_t)r * a.H;
            for (int k = lane; k < a.H; k += 64) {
                const float wv = w[k];
#pragma unroll
                for (int i = 0; i < HBT; ++i) {
                    const int b = b0 + i;
                    const float hv = (b < a.B) ? a.h_prev[(size_t)b * a.h_prev_ld + k] : 0.f;
                    acc[i] = fmaf(wv, hv, acc[i]);
                }
            }
        } else {
            const int beg = a.row_ptr[r], end = a.row_ptr[r + 1];
            for (int e = beg + lane; e < end; e += 64) {
                const float wv = a.val[e];
                const int k = a.col[e];
#pragma unroll
                for (int i = 0; i < HBT; ++i) {
                    const int b = b0 + i;
                    const float hv = (b < a.B) ? a.h_prev[(size_t)b * a.h_prev_ld + k] : 0.f;
                    acc[i] = fmaf(wv, hv, acc[i]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < HBT; ++i) {
        const float s = wave_sum(acc[i]);
        const int b = b0 + i;
        if (lane == 0 && b < a.B) {
            const float v = a.P1[((size_t)a.t * a.B + b) * R + r] + s;
            a.u[(size_t)b * R + r] = v > 0.f ? v : 0.f;
        }
    }
}

__global__ __launch_bounds__(256) void hstage2_kernel(HStage2Args a)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= a.H) return;
    const int b0 = blockIdx.y * HBT;
    const int R = 4 * a.G;
    float acc[4][HBT];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < HBT; ++i) acc[q][i] = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (a.w_dense) {
            const float* w = a.w_dense + (size_t)(4 * j + q) * a.G;
            for (int g = lane; g < a.G; g += 64) {
                const float wv = w[g];
#pragma unroll
                for (int i = 0; i < HBT; ++i) {
                    const int b = b0 + i;
                    const float uv = (b < a.B) ? a.u[(size_t)b * R + 4 * g + q] : 0.f;
                    acc[q][i] = fmaf(wv, uv, acc[q][i]);
                }
            }
        } else {
            const int beg = a.row_ptr[4 * j + q], end = a.row_ptr[4 * j + q + 1];
            for (int e = beg + lane; e < end; e += 64) {
                const float wv = a.val[e];
                const int g = a.col[e];
#pragma unroll
                for (int i = 0; i < HBT; ++i) {
                    const int b = b0 + i;
                    const float uv = (b < a.B) ? a.u[(size_t)b * R + 4 * g + q] : 0.f;
                    acc[q][i] = fmaf(wv, uv, acc[q][i]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < HBT; ++i) {
        float pre[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) pre[q] = wave_sum(acc[q][i]) + a.bias2[4 * j + q];
        const int b = b0 + i;
        if (lane == 0 && b < a.B) {
            const float f = sigmoidf_fast(pre[0]), ig = sigmoidf_fast(pre[1]), o = sigmoidf_fast(pre[2]), g = tanhf_fast(pre[3]);
            const size_t ci = (size_t)b * a.H + j;
            const float cn = fmaf(f, a.c[ci], ig * g);
            const float hn = o * tanhf_fast(cn);
            a.c[ci] = cn;
            a.y_t[(size_t)b * a.y_ld + j] = hn;
            if (a.last) {
                if (a.hT) a.hT[ci] = hn;
                if (a.cT) a.cT[ci] = cn;
            }
        }
    }
}

hipError_t launch_hstage1(const HStage1Args& a, hipStream_t s)
{
    if (a.B <= 0 || a.G <= 0) return hipSuccess;
    dim3 grid((4 * a.G + 3) / 4, (a.B + HBT - 1) / HBT), block(256);
    hipLaunchKernelGGL(hstage1_kernel, grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_hstage2(const HStage2Args& a, hipStream_t s)
{
    if (a.B <= 0 || a.H <= 0) return hipSuccess;
    dim3 grid((a.H + 3) / 4, (a.B + HBT - 1) / HBT), block(256);
    hipLaunchKernelGGL(hstage2_kernel, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace l355

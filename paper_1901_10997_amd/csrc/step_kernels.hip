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

// ---------------------------------------------------------------------------------------------------------
// Row-compressed step for small batches, both directions of a layer in one launch.
// A 1024-thread workgroup serves 16 hidden units (one per wave) for a tile of 8 batch columns.  The tile of
// h_{t-1} is staged in LDS with the 8 batch values of one k adjacent, so that one kept weight costs two 16-byte
// LDS reads and eight FMAs.  Lanes split a row's kept entries (the 64-lane slices built at weight set-up);
// the 4 x 8 partial sums are reduced with the lane-swap reduction, the gates of all eight columns are
// evaluated with one exp2 and one reciprocal, and lanes 0..7 update c and h of their batch column.
// ---------------------------------------------------------------------------------------------------------
struct StepDir {
    const float* P;        // [T*B][4H]
    const float* h_prev;   // (b,k) at h_prev[b*h_prev_ld + k]; nullptr = zeros
    int h_prev_ld;
    float* c;              // [B][H]
    float* y_t;            // h_t -> y_t[b*y_ld + j]
    int y_ld;
    float* hT;
    float* cT;
    int t;
    const float* ell_val;  // [4H][slots][64]
    const uint16_t* ell_col;
    int slots;
};
struct StepPairArgs {
    StepDir d[2];
    int B, H, last, round_h_bf16;
};

template <int NZ>
__global__ __launch_bounds__(1024) void step_csr_pair_kernel(StepPairArgs a)
{
    extern __shared__ float hbuf[];  // [H][8]
    const StepDir& D = a.d[blockIdx.z];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = blockIdx.x * 16 + wave;
    const int b0 = blockIdx.y * 8;
    const int H = a.H;
    const int lb = lane & 15, row = lane >> 4;
    const bool col_ok = lb < 8 && (b0 + lb) < a.B;
    // everything that does not depend on the staged tile is requested first: this wave's kept weights, its
    // slice of the projection, the cell state
    float wv[4][NZ];
    int wc[4][NZ];
    const int jj = j < H ? j : H - 1;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < NZ; ++i) {
            float w = 0.f;
            int k = 0;
            if (i < D.slots && D.h_prev != nullptr) {
                const size_t idx = ((size_t)(4 * jj + q) * D.slots + i) * 64 + lane;
                w = D.ell_val[idx];
                k = D.ell_col[idx];
            }
            wv[q][i] = w;
            wc[q][i] = k;
        }
    float pin = 0.f, cprev = 0.f;
    if (col_ok) pin = D.P[((size_t)D.t * a.B + b0 + lb) * (4 * (size_t)H) + 4 * jj + row];
    if (lane < 8 && col_ok) cprev = D.c[(size_t)(b0 + lane) * H + jj];
    // stage the h tile: eight independent coalesced global reads per thread (one per batch column), then two
    // 16-byte LDS writes that lay the eight values of one k next to each other
    for (int k = tid; k < H; k += 1024) {
        float v[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool ok = (b0 + b < a.B) && D.h_prev != nullptr;
            v[b] = ok ? D.h_prev[(size_t)(b0 + b) * D.h_prev_ld + k] : 0.f;
        }
        if (a.round_h_bf16) {
#pragma unroll
            for (int b = 0; b < 8; ++b) v[b] = round_bf16(v[b]);
        }
        // the two 16-byte halves of row k swap places when bit 2 of k is set: gathers of random k then spread
        // over all eight 4-bank groups instead of four
        const int sw = (k >> 2) & 1;
        *reinterpret_cast<float4*>(hbuf + k * 8 + 4 * sw) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(hbuf + k * 8 + 4 * (sw ^ 1)) = make_float4(v[4], v[5], v[6], v[7]);
    }
    __syncthreads();
    if (j >= H) return;  // whole wave; no barrier follows
    float acc[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[q][b] = 0.f;
    {
#pragma unroll
        for (int i = 0; i < NZ; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float w = wv[q][i];
                const int k = wc[q][i];
                const int sw = (k >> 2) & 1;
                const float4 lo = *reinterpret_cast<const float4*>(hbuf + k * 8 + 4 * sw);
                const float4 hi = *reinterpret_cast<const float4*>(hbuf + k * 8 + 4 * (sw ^ 1));
                acc[q][0] = fmaf(w, lo.x, acc[q][0]);
                acc[q][1] = fmaf(w, lo.y, acc[q][1]);
                acc[q][2] = fmaf(w, lo.z, acc[q][2]);
                acc[q][3] = fmaf(w, lo.w, acc[q][3]);
                acc[q][4] = fmaf(w, hi.x, acc[q][4]);
                acc[q][5] = fmaf(w, hi.y, acc[q][5]);
                acc[q][6] = fmaf(w, hi.z, acc[q][6]);
                acc[q][7] = fmaf(w, hi.w, acc[q][7]);
            }
        }
    }
    // lane 16*q + b  <-  total of gate q, batch column b
    float G = 0.f;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const float r = wave_sum4_rows(acc[0][b], acc[1][b], acc[2][b], acc[3][b]);
        G = (lb == b) ? r : G;
    }
    G += pin;
    const bool cand = row == 3;
    const float sc = cand ? 2.8853900817779268f : -1.4426950408889634f;
    const float rr = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc * G));
    const float gate = cand ? fmaf(-2.0f, rr, 1.0f) : rr;
    const float gi = __shfl(gate, 16 + lb, 64), go = __shfl(gate, 32 + lb, 64), gg = __shfl(gate, 48 + lb, 64);
    if (lane < 8 && col_ok) {
        const size_t ci = (size_t)(b0 + lane) * H + j;
        const float cn = fmaf(gate, cprev, gi * gg);
        const float hn = go * tanhf_fast(cn);
        D.c[ci] = cn;
        D.y_t[(size_t)(b0 + lane) * D.y_ld + j] = hn;
        if (a.last) {
            if (D.hT) D.hT[ci] = hn;
            if (D.cT) D.cT[ci] = cn;
        }
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

bool step_csr_pair_supported(int H, int slots) { return H >= 1 && H <= 2048 && slots >= 1 && slots <= 6; }

// ndir = 1 or 2 directions of one layer advanced by one timestep in a single launch.
hipError_t launch_step_csr_pair(const StepArgs* a, const float* const* ell_val, const uint16_t* const* ell_col,
                                const int* slots, int ndir, hipStream_t s)
{
    if (a[0].B <= 0 || a[0].H <= 0) return hipSuccess;
    StepPairArgs p{};
    for (int d = 0; d < ndir; ++d) {
        p.d[d].P = a[d].P;
        p.d[d].h_prev = a[d].h_prev;
        p.d[d].h_prev_ld = a[d].h_prev_ld;
        p.d[d].c = a[d].c;
        p.d[d].y_t = a[d].y_t;
        p.d[d].y_ld = a[d].y_ld;
        p.d[d].hT = a[d].hT;
        p.d[d].cT = a[d].cT;
        p.d[d].t = a[d].t;
        p.d[d].ell_val = ell_val[d];
        p.d[d].ell_col = ell_col[d];
        p.d[d].slots = slots[d];
    }
    p.B = a[0].B;
    p.H = a[0].H;
    p.last = a[0].last;
    p.round_h_bf16 = a[0].round_h_bf16;
    dim3 grid((p.H + 15) / 16, (p.B + 7) / 8, ndir), block(1024);
    const size_t lds = (size_t)p.H * 8 * sizeof(float);
    int nz = 1;
    for (int d = 0; d < ndir; ++d) nz = slots[d] > nz ? slots[d] : nz;
    switch (nz) {
        case 1: hipLaunchKernelGGL(step_csr_pair_kernel<1>, grid, block, lds, s, p); break;
        case 2: hipLaunchKernelGGL(step_csr_pair_kernel<2>, grid, block, lds, s, p); break;
        case 3: hipLaunchKernelGGL(step_csr_pair_kernel<3>, grid, block, lds, s, p); break;
        case 4: hipLaunchKernelGGL(step_csr_pair_kernel<4>, grid, block, lds, s, p); break;
        case 5: hipLaunchKernelGGL(step_csr_pair_kernel<5>, grid, block, lds, s, p); break;
        case 6: hipLaunchKernelGGL(step_csr_pair_kernel<6>, grid, block, lds, s, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace l355

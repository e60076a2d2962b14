// Input projection  P[t*B+b][r] = b[r] + sum_k W_x[r][k] * x[t][b][k]  for all timesteps at once
// (the x-part of the gate pre-activation W.[x_t, h_{t-1}] + b of the paper's cell equations, Section 4).
// Rows r are in packed order (4*unit + gate), so each hidden unit's four pre-activations form one float4.
#include "common.h"
#include "device_math.h"

namespace l355 {

// ---------------------------------------------------------------------------------------------
// Plain LDS-tiled vector-FMA GEMM (64x64 tile per 256-thread block, 4x4 outputs per thread).
// Correct for every shape; the MFMA kernels take over where the shape makes the product a real
// dense contraction.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) { return bf16_bits_to_f32(p[i]); }

template <typename TX, typename TW, bool ROUND_X>
__global__ __launch_bounds__(256) void proj_dense_kernel(const TX* __restrict__ X, int ldx, const TW* __restrict__ W,
                                                         const float* __restrict__ bias, float* __restrict__ P, int M,
                                                         int N, int K)
{
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float Xs[TK][TM + 1];
    __shared__ float Ws[TK][TN + 1];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const int tx = tid & 15, ty = tid >> 4;  // thread computes rows m0+ty*4.., cols n0+tx*4..
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += TK) {
        // each thread loads 4 elements of each tile: element e -> (row = e / TK, kk = e % TK)
#pragma unroll
        for (int e = tid; e < TM * TK; e += 256) {
            const int r = e / TK, kk = e % TK;
            const int m = m0 + r, k = k0 + kk;
            float v = 0.f;
            if (m < M && k < K) {
                v = load_elem(X, (size_t)m * ldx + k);
                if (ROUND_X) v = round_bf16(v);
            }
            Xs[kk][r] = v;
            const int n = n0 + r;
            float w = 0.f;
            if (n < N && k < K) w = load_elem(W, (size_t)n * K + k);
            Ws[kk][r] = w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float xv[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = Xs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) P[(size_t)m * N + n] = acc[i][j] + bias[n];
        }
    }
}

hipError_t launch_proj_dense(const void* X, bool x_bf16, int ldx, const void* W, bool w_bf16, const float* bias,
                             float* P, int M, int N, int K, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
    if (!w_bf16) {
        if (x_bf16) return hipErrorInvalidValue;  // fp32 models take fp32 inputs
        hipLaunchKernelGGL((proj_dense_kernel<float, float, false>), grid, block, 0, s, (const float*)X, ldx,
                           (const float*)W, bias, P, M, N, K);
    } else if (x_bf16) {
        hipLaunchKernelGGL((proj_dense_kernel<uint16_t, uint16_t, false>), grid, block, 0, s, (const uint16_t*)X, ldx,
                           (const uint16_t*)W, bias, P, M, N, K);
    } else {
        // bf16 model reading the fp32 hidden sequence of the layer below: round the operand to bf16
        hipLaunchKernelGGL((proj_dense_kernel<float, uint16_t, true>), grid, block, 0, s, (const float*)X, ldx,
                           (const uint16_t*)W, bias, P, M, N, K);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Transposed fp32 copy of the layer input, XT[k][m], so that the compressed projection reads
// 64 consecutive m per kept weight.
// ---------------------------------------------------------------------------------------------
template <typename TX>
__global__ __launch_bounds__(256) void transpose_kernel(const TX* __restrict__ X, int ldx, float* __restrict__ XT,
                                                        int M, int K, int round_bf16_flag)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int m0 = blockIdx.y * 32, k0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8) {
        const int m = m0 + i, k = k0 + tx;
        float v = 0.f;
        if (m < M && k < K) {
            v = load_elem(X, (size_t)m * ldx + k);
            if (round_bf16_flag) v = round_bf16(v);
        }
        tile[i][tx] = v;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, m = m0 + tx;
        if (k < K && m < M) XT[(size_t)k * M + m] = tile[tx][i];
    }
}

hipError_t launch_transpose_to_f32(const void* X, bool x_bf16, int ldx, float* XT, int M, int K, bool round_bf16_flag,
                                   hipStream_t s)
{
    if (M <= 0 || K <= 0) return hipSuccess;
    dim3 grid((K + 31) / 32, (M + 31) / 32), block(256);
    if (x_bf16)
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, block, 0, s, (const uint16_t*)X, ldx, XT, M, K, 0);
    else
        hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, s, (const float*)X, ldx, XT, M, K,
                           round_bf16_flag ? 1 : 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Row-compressed projection.  One 256-thread block = the four gate rows of one hidden unit (one wave per
// row) times a strip of 64*MT values of m; lanes run along m so that every kept weight costs MT coalesced
// loads of XT.  The four row results are exchanged through LDS and written as one float4 per m.
// ---------------------------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(256) void proj_csr_kernel(const float* __restrict__ XT, const int32_t* __restrict__ row_ptr,
                                                       const uint16_t* __restrict__ col, const float* __restrict__ val,
                                                       const float* __restrict__ bias, float* __restrict__ P, int M,
                                                       int rows)
{
    __shared__ float out[4][64 * MT];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int unit = blockIdx.x;
    const int r = unit * 4 + q;
    const int mbase = blockIdx.y * 64 * MT;
    float acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = 0.f;
    const int beg = row_ptr[r], end = row_ptr[r + 1];
    for (int e = beg; e < end; ++e) {
        const float w = val[e];
        const float* xr = XT + (size_t)col[e] * M + mbase;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const int m = mbase + i * 64 + lane;
            const float xv = (m < M) ? xr[i * 64 + lane] : 0.f;
            acc[i] = fmaf(w, xv, acc[i]);
        }
    }
    const float bb = bias[r];
#pragma unroll
    for (int i = 0; i < MT; ++i) out[q][i * 64 + lane] = acc[i] + bb;
    __syncthreads();
    for (int mm = threadIdx.x; mm < 64 * MT; mm += 256) {
        const int m = mbase + mm;
        if (m < M) {
            float4 v = make_float4(out[0][mm], out[1][mm], out[2][mm], out[3][mm]);
            *reinterpret_cast<float4*>(P + (size_t)m * rows + unit * 4) = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Row-compressed projection for few input rows (M <= 64: batch-1 sequences, small T*B).  The kernel above gives a
// wave one output row and walks its kept entries one after the other with the input rows on the lanes, which is
// bound by dependent-load latency when M is small.  Here the lanes split a row's kept entries (the 64-lane slices
// built at weight set-up, streamed once, coalesced): a 1024-thread workgroup serves 16 units (4 packed rows each)
// for a tile of 8 input rows, the tile of X is staged in LDS with the 8 values of one k adjacent (one kept weight
// costs two 16-byte LDS reads and eight FMAs), and the 4 x 8 sums are reduced with the lane-swap reduction.
// ---------------------------------------------------------------------------------------------
template <typename TX>
__global__ __launch_bounds__(1024) void proj_ell_small_kernel(const TX* __restrict__ X, int ldx, int round_x_bf16,
                                                              const float* __restrict__ ell_val,
                                                              const uint16_t* __restrict__ ell_col, int slots,
                                                              const float* __restrict__ bias, float* __restrict__ P,
                                                              int M, int rows, int K)
{
    extern __shared__ float xbuf[];  // [K][8]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int unit = blockIdx.x * 16 + wave;
    const int m0 = blockIdx.y * 8;
    const int lb = lane & 15, row = lane >> 4;
    for (int k = tid; k < K; k += 1024) {
        float v[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            float xv = (m0 + b < M) ? load_elem(X, (size_t)(m0 + b) * ldx + k) : 0.f;
            if (round_x_bf16) xv = round_bf16(xv);
            v[b] = xv;
        }
        // the two 16-byte halves of row k swap places when bit 2 of k is set, so that gathers of random k spread
        // over all bank groups
        const int sw = (k >> 2) & 1;
        *reinterpret_cast<float4*>(xbuf + k * 8 + 4 * sw) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(xbuf + k * 8 + 4 * (sw ^ 1)) = make_float4(v[4], v[5], v[6], v[7]);
    }
    __syncthreads();
    if (4 * unit >= rows) return;  // whole wave; no barrier follows
    float acc[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[q][b] = 0.f;
    for (int i = 0; i < slots; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const size_t idx = ((size_t)(4 * unit + q) * slots + i) * 64 + lane;
            const float w = ell_val[idx];
            const int k = ell_col[idx];
            const int sw = (k >> 2) & 1;
            const float4 lo = *reinterpret_cast<const float4*>(xbuf + k * 8 + 4 * sw);
            const float4 hi = *reinterpret_cast<const float4*>(xbuf + k * 8 + 4 * (sw ^ 1));
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
    // lane 16*q + b  <-  total of packed row 4*unit + q, input row m0 + b
    float S = 0.f;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const float r = wave_sum4_rows(acc[0][b], acc[1][b], acc[2][b], acc[3][b]);
        S = (lb == b) ? r : S;
    }
    if (lb < 8 && m0 + lb < M) P[(size_t)(m0 + lb) * rows + 4 * unit + row] = S + bias[4 * unit + row];
}

bool proj_ell_small_supported(int M, int rows, int K, int slots)
{
    return M >= 1 && M <= 64 && rows >= 4 && (rows & 3) == 0 && slots >= 1 && (size_t)K * 8 * sizeof(float) <= 160 * 1024;
}

hipError_t launch_proj_ell_small(const void* X, bool x_bf16, int ldx, bool round_x_bf16, const float* ell_val,
                                 const uint16_t* ell_col, int slots, const float* bias, float* P, int M, int rows, int K,
                                 hipStream_t s)
{
    if (M <= 0 || rows <= 0) return hipSuccess;
    if (!proj_ell_small_supported(M, rows, K, slots)) return hipErrorInvalidValue;
    const size_t lds = (size_t)K * 8 * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)proj_ell_small_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)proj_ell_small_kernel<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((rows / 4 + 15) / 16, (M + 7) / 8), block(1024);
    if (x_bf16)
        hipLaunchKernelGGL(proj_ell_small_kernel<uint16_t>, grid, block, lds, s, (const uint16_t*)X, ldx, 0, ell_val, ell_col, slots, bias, P, M, rows, K);
    else
        hipLaunchKernelGGL(proj_ell_small_kernel<float>, grid, block, lds, s, (const float*)X, ldx, round_x_bf16 ? 1 : 0, ell_val, ell_col, slots, bias, P, M, rows, K);
    return hipGetLastError();
}

hipError_t launch_proj_csr(const float* XT, const int32_t* row_ptr, const uint16_t* col, const float* val,
                           const float* bias, float* P, int M, int rows, hipStream_t s)
{
    if (M <= 0 || rows <= 0) return hipSuccess;
    const int units = rows / 4;
    if (M <= 64) {
        dim3 grid(units, 1), block(256);
        hipLaunchKernelGGL(proj_csr_kernel<1>, grid, block, 0, s, XT, row_ptr, col, val, bias, P, M, rows);
    } else {
        dim3 grid(units, (M + 255) / 256), block(256);
        hipLaunchKernelGGL(proj_csr_kernel<4>, grid, block, 0, s, XT, row_ptr, col, val, bias, P, M, rows);
    }
    return hipGetLastError();
}

}  // namespace l355

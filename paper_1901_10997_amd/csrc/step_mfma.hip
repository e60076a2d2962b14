// One LSTM timestep per launch for bf16 models at large batch: recurrent product on the matrix cores with the
// gate nonlinearities and the cell update (paper Section 4, cell equations) fused into the epilogue.
//
//   R[b][n] = sum_k hb[b][k] * W_h[n][k]     (hb = h_{t-1} rounded to bf16, W_h packed rows n = 4*unit + gate)
//   a = P[t][b][n] + R[b][n];  f,i,o = sigmoid, g = tanh;  c <- f*c + i*g;  h = o*tanh(c)
//
// A workgroup of NW waves owns a 64 (batch) x 64 (packed rows = 16 hidden units) tile.  The step is short and
// latency-bound, so there is no LDS pipeline: the NW waves split K, each streams its operand fragments from
// global memory straight into registers (every lane reads 64 contiguous bytes of its row per 64-wide k block,
// so a pair of lanes consumes a whole 128-byte line once), and the NW partial tiles are summed through LDS.
// With eight waves and H = 1024 a wave's whole share of K is two blocks, both requested before the first MFMA,
// so the kernel pays one operand round trip; the epilogue's P and c values are requested before the product
// as well, which hides their (HBM) latency behind it.
// Which 8 k a lane contributes to which MFMA is the same for both operands, which is all a sum over k needs.
#include "common.h"
#include "device_math.h"

namespace l355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int NW>
__global__ __launch_bounds__(64 * NW) void step_mfma_bf16_kernel(StepMfmaArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float part[];  // [NW][64][68]
    constexpr int LDP = 68;
    constexpr int NT = 64 * NW;
    constexpr int PAIRS = 1024 / NT;  // (batch row, hidden unit) pairs each thread finishes
    const int gm = (a.B + 63) / 64, gn = (4 * a.H) / 64;
    const int nblk = gm * gn;
    const int per_xcd = (nblk + 7) / 8;
    const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (logical >= nblk) return;
    const int tile_n = logical / gm, tile_m = logical % gm;  // workgroups that share a W_h panel stay on one XCD
    const int m0 = tile_m * 64, n0 = tile_n * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fk = lane >> 5;
    const int K = a.H, Kq = K / NW;

    // epilogue operands, requested first
    float4 pre[PAIRS];
    float cold[PAIRS];
#pragma unroll
    for (int r = 0; r < PAIRS; ++r) {
        const int p = tid + NT * r;
        int b = m0 + (p >> 4);
        if (b > a.B - 1) b = a.B - 1;
        const int jn = n0 + 4 * (p & 15);
        pre[r] = *reinterpret_cast<const float4*>(a.P + ((size_t)a.t * a.B + b) * (4 * (size_t)a.H) + jn);
        cold[r] = a.c[(size_t)b * a.H + (jn >> 2)];
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (a.hb_prev != nullptr) {
        const uint16_t* arow[2];
        const uint16_t* brow[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int m = m0 + i * 32 + fr;
            if (m > a.B - 1) m = a.B - 1;  // rows beyond the batch are computed on a valid row and never stored
            arow[i] = a.hb_prev + (size_t)m * a.hb_prev_ld + wave * Kq + fk * 32;
            brow[i] = a.Wh + (size_t)(n0 + i * 32 + fr) * K + wave * Kq + fk * 32;
        }
        // software pipeline over 64-wide k blocks: the fragments of block kb+64 are requested before the MFMAs
        // of block kb are issued, so one memory round trip is exposed per wave instead of one per block
        uint4 fa[2][2][4], fb[2][2][4];
        auto request = [&](int buf, int kb) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    fa[buf][i][s] = *reinterpret_cast<const uint4*>(arow[i] + kb + s * 8);
                    fb[buf][i][s] = *reinterpret_cast<const uint4*>(brow[i] + kb + s * 8);
                }
        };
        auto consume = [&](int buf) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[buf][i][s]),
                                                                           __builtin_bit_cast(bf16x8, fb[buf][j][s]),
                                                                           acc[i][j], 0, 0, 0);
        };
        request(0, 0);
        for (int kb = 0; kb < Kq; kb += 128) {
            if (kb + 64 < Kq) request(1, kb + 64);
            consume(0);
            if (kb + 64 < Kq) {
                if (kb + 128 < Kq) request(0, kb + 128);
                consume(1);
            }
        }
    }
    // partial tiles -> LDS.  Accumulator register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32).
    float* mine = part + (size_t)wave * 64 * LDP;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = i * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                mine[m * LDP + j * 32 + fr] = acc[i][j][v];
            }
    __syncthreads();
    // epilogue: each thread finishes four (batch row, hidden unit) pairs
#pragma unroll
    for (int r = 0; r < PAIRS; ++r) {
        const int p = tid + NT * r;
        const int m = p >> 4, u = p & 15;
        const int b = m0 + m;
        if (b >= a.B) continue;
        const int jn = n0 + 4 * u;       // first packed row of the unit
        const int j = jn >> 2;           // hidden unit
        float4 sum = pre[r];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float4 q = *reinterpret_cast<const float4*>(part + ((size_t)w * 64 + m) * LDP + 4 * u);
            sum.x += q.x;
            sum.y += q.y;
            sum.z += q.z;
            sum.w += q.w;
        }
        const float f = sigmoidf_fast(sum.x), ig = sigmoidf_fast(sum.y), o = sigmoidf_fast(sum.z), g = tanhf_fast(sum.w);
        const size_t ci = (size_t)b * a.H + j;
        const float cn = fmaf(f, cold[r], ig * g);
        const float hn = o * tanhf_fast(cn);
        a.c[ci] = cn;
        a.y_t[(size_t)b * a.y_ld + j] = hn;
        a.hb_t[(size_t)b * a.hb_ld + j] = f32_to_bf16_bits(hn);
        if (a.last) {
            if (a.hT) a.hT[ci] = hn;
            if (a.cT) a.cT[ci] = cn;
        }
    }
}

// bf16 copy of an fp32 [rows][cols] block (used for h0)
__global__ void f32_to_bf16_kernel(const float* __restrict__ src, int src_ld, uint16_t* __restrict__ dst, int dst_ld,
                                   int rows, int cols)
{
    const size_t n = (size_t)rows * cols;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t r = i / cols, c = i % cols;
        dst[r * dst_ld + c] = f32_to_bf16_bits(src[r * src_ld + c]);
    }
}

bool step_mfma_supported(int B, int H) { return B >= 32 && H % 256 == 0; }

hipError_t launch_step_mfma_bf16(const StepMfmaArgs& a, hipStream_t s)
{
    if (a.B <= 0 || a.H <= 0) return hipSuccess;
    if (!step_mfma_supported(a.B, a.H)) return hipErrorInvalidValue;
    const int gm = (a.B + 63) / 64, gn = (4 * a.H) / 64;
    const int grid = ((gm * gn + 7) / 8) * 8;
    // eight waves when K divides into whole 64-wide blocks per wave and the grid does not need several
    // workgroups per compute unit to fill the device
    const bool wide = a.H % 512 == 0 && grid <= 512;
    const size_t lds = (size_t)(wide ? 8 : 4) * 64 * 68 * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)step_mfma_bf16_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           4 * 64 * 68 * (int)sizeof(float));
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)step_mfma_bf16_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                8 * 64 * 68 * (int)sizeof(float));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (wide)
        hipLaunchKernelGGL(step_mfma_bf16_kernel<8>, dim3(grid), dim3(512), lds, s, a);
    else
        hipLaunchKernelGGL(step_mfma_bf16_kernel<4>, dim3(grid), dim3(256), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_f32_to_bf16(const float* src, int src_ld, uint16_t* dst, int dst_ld, int rows, int cols, hipStream_t s)
{
    const size_t n = (size_t)rows * cols;
    if (n == 0) return hipSuccess;
    int g = (int)((n + 255) / 256);
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(g), dim3(256), 0, s, src, src_ld, dst, dst_ld, rows, cols);
    return hipGetLastError();
}

}  // namespace l355

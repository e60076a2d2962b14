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

// ---------------------------------------------------------------------------------------------------------
// Row-compressed H-LSTM stages for small batches, all directions of a layer in one launch.
// A 1024-thread workgroup serves 16 units (one per wave) for a tile of 8 batch columns.  The input vector of the
// stage (h_{t-1}: H values; u_t: 4G values, gate-major) is staged in LDS with the 8 batch values of one k adjacent,
// so that one kept weight costs two 16-byte LDS reads and eight FMAs; lanes split a row's kept entries (the 64-lane
// slices built at weight set-up); the 4 x 8 partial sums are reduced with the lane-swap reduction.
//   STAGE 1: unit = hidden-layer unit g; lane (gate q, column b) adds P1 and writes relu(.) to u[b][q*G + g]
//   STAGE 2: unit = output j; row q gathers from the block q*G.. of u; lane (q, b) adds b2; gates of all eight
//            columns with one exp2 and one reciprocal; lanes 0..7 update c and h of their batch column
// ---------------------------------------------------------------------------------------------------------
template <int NZ, int STAGE>
__global__ __launch_bounds__(1024) void hstep_pair_kernel(HStepPairArgs a)
{
    extern __shared__ float vbuf[];  // [K][8], K = H (stage 1) or 4G (stage 2)
    const HStepDir& D = a.d[blockIdx.z];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int unit = blockIdx.x * 16 + wave;
    const int b0 = blockIdx.y * 8;
    const int H = a.H, G = a.G;
    const int units = STAGE == 1 ? G : H;
    const int K = STAGE == 1 ? H : 4 * G;
    const float* vin = STAGE == 1 ? D.h_prev : D.u;
    const int vin_ld = STAGE == 1 ? D.h_prev_ld : 4 * G;
    const int lb = lane & 15, row = lane >> 4;
    const bool col_ok = lb < 8 && (b0 + lb) < a.B;
    const float* ell_val = STAGE == 1 ? D.ell_val_1h : D.ell_val_2;
    const uint16_t* ell_col = STAGE == 1 ? D.ell_col_1h : D.ell_col_2;
    const int slots = STAGE == 1 ? D.slots_1h : D.slots_2;
    float wv[4][NZ];
    int wc[4][NZ];
    const int uu = unit < units ? unit : units - 1;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < NZ; ++i) {
            float w = 0.f;
            int k = 0;
            if (i < slots && vin != nullptr) {
                const size_t idx = ((size_t)(4 * uu + q) * slots + i) * 64 + lane;
                w = ell_val[idx];
                k = ell_col[idx];
            }
            wv[q][i] = w;
            wc[q][i] = STAGE == 2 ? k + q * G : k;     // row q of W2 reads the hidden layer of gate q
        }
    float pin = 0.f, cprev = 0.f;
    if (STAGE == 1) {
        if (col_ok) pin = D.P1[((size_t)D.t * a.B + b0 + lb) * (4 * (size_t)G) + 4 * uu + row];
    } else {
        pin = D.bias2[4 * uu + row];
        if (lane < 8 && col_ok) cprev = D.c[(size_t)(b0 + lane) * H + uu];
    }
    for (int k = tid; k < K; k += 1024) {
        float v[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool ok = (b0 + b < a.B) && vin != nullptr;
            v[b] = ok ? vin[(size_t)(b0 + b) * vin_ld + k] : 0.f;
        }
        // the two 16-byte halves of row k swap places when bit 2 of k is set: gathers of random k then spread
        // over all eight 4-bank groups instead of four
        const int sw = (k >> 2) & 1;
        *reinterpret_cast<float4*>(vbuf + k * 8 + 4 * sw) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(vbuf + k * 8 + 4 * (sw ^ 1)) = make_float4(v[4], v[5], v[6], v[7]);
    }
    __syncthreads();
    if (unit >= units) return;  // whole wave; no barrier follows
    float acc[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[q][b] = 0.f;
#pragma unroll
    for (int i = 0; i < NZ; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float w = wv[q][i];
            const int k = wc[q][i];
            const int sw = (k >> 2) & 1;
            const float4 lo = *reinterpret_cast<const float4*>(vbuf + k * 8 + 4 * sw);
            const float4 hi = *reinterpret_cast<const float4*>(vbuf + k * 8 + 4 * (sw ^ 1));
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
    // lane 16*q + b  <-  total of gate q, batch column b
    float S = 0.f;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const float r = wave_sum4_rows(acc[0][b], acc[1][b], acc[2][b], acc[3][b]);
        S = (lb == b) ? r : S;
    }
    S += pin;
    if (STAGE == 1) {
        if (col_ok) D.u[(size_t)(b0 + lb) * (4 * (size_t)G) + (size_t)row * G + unit] = S > 0.f ? S : 0.f;
    } else {
        const bool cand = row == 3;
        const float sc = cand ? 2.8853900817779268f : -1.4426950408889634f;
        const float rr = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc * S));
        const float gate = cand ? fmaf(-2.0f, rr, 1.0f) : rr;
        const float gi = __shfl(gate, 16 + lb, 64), go = __shfl(gate, 32 + lb, 64), gg = __shfl(gate, 48 + lb, 64);
        if (lane < 8 && col_ok) {
            const size_t ci = (size_t)(b0 + lane) * H + unit;
            const float cn = fmaf(gate, cprev, gi * gg);
            const float hn = go * tanhf_fast(cn);
            D.c[ci] = cn;
            D.y_t[(size_t)(b0 + lane) * D.y_ld + unit] = hn;
            if (a.last) {
                if (D.hT) D.hT[ci] = hn;
                if (D.cT) D.cT[ci] = cn;
            }
        }
    }
}

bool hstep_pair_supported(int H, int G, int slots_1h, int slots_2)
{
    if (H < 1 || G < 1 || slots_1h < 1 || slots_2 < 1 || slots_1h > 6 || slots_2 > 6) return false;
    return (size_t)std::max(H, 4 * G) * 8 * sizeof(float) <= 160 * 1024 && H <= 65536 && 4 * (size_t)G <= (1u << 20);
}

template <int NZ, int STAGE>
static hipError_t launch_hstep_pair_nz(const HStepPairArgs& p, int ndir, hipStream_t s)
{
    const int units = STAGE == 1 ? p.G : p.H;
    const int K = STAGE == 1 ? p.H : 4 * p.G;
    const size_t lds = (size_t)K * 8 * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)hstep_pair_kernel<NZ, STAGE>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((units + 15) / 16, (p.B + 7) / 8, ndir), block(1024);
    hipLaunchKernelGGL((hstep_pair_kernel<NZ, STAGE>), grid, block, lds, s, p);
    return hipGetLastError();
}

// One timestep of ndir = 1 or 2 directions of an H-LSTM layer: stage 1 then stage 2 (two launches).
hipError_t launch_hstep_pair(const HStepPairArgs& p, int ndir, hipStream_t s)
{
    if (p.B <= 0 || p.H <= 0 || p.G <= 0) return hipSuccess;
    int nz1 = 1, nz2 = 1;
    for (int d = 0; d < ndir; ++d) {
        nz1 = std::max(nz1, p.d[d].slots_1h);
        nz2 = std::max(nz2, p.d[d].slots_2);
    }
    if (!hstep_pair_supported(p.H, p.G, nz1, nz2)) return hipErrorInvalidValue;
    hipError_t e = hipErrorInvalidValue;
    switch (nz1) {
        case 1: e = launch_hstep_pair_nz<1, 1>(p, ndir, s); break;
        case 2: e = launch_hstep_pair_nz<2, 1>(p, ndir, s); break;
        case 3: e = launch_hstep_pair_nz<3, 1>(p, ndir, s); break;
        case 4: e = launch_hstep_pair_nz<4, 1>(p, ndir, s); break;
        case 5: e = launch_hstep_pair_nz<5, 1>(p, ndir, s); break;
        case 6: e = launch_hstep_pair_nz<6, 1>(p, ndir, s); break;
    }
    if (e != hipSuccess) return e;
    switch (nz2) {
        case 1: return launch_hstep_pair_nz<1, 2>(p, ndir, s);
        case 2: return launch_hstep_pair_nz<2, 2>(p, ndir, s);
        case 3: return launch_hstep_pair_nz<3, 2>(p, ndir, s);
        case 4: return launch_hstep_pair_nz<4, 2>(p, ndir, s);
        case 5: return launch_hstep_pair_nz<5, 2>(p, ndir, s);
        case 6: return launch_hstep_pair_nz<6, 2>(p, ndir, s);
    }
    return hipErrorInvalidValue;
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

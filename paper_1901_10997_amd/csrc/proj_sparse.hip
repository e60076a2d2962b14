// Input projection with row-compressed weights for many input rows (T*B of the small-batch configurations):
//     P[m, 4j + q] = b[4j + q] + sum over the kept k of W_x[4j + q, k] * X[m, k]        (paper Section 4: W (x) Msk)
// The structure of the small-batch recurrence applied to the projection.  A 512-thread workgroup keeps the kept
// weights of its 8 * UPW units in registers for the whole launch, in the quarter-wave form (slot s of a unit is one
// 64-lane gather that serves all four gate rows, gate q on lanes 16q..16q+15), and walks over tiles of four input
// rows: the tile is staged in LDS as [k][4] (the four rows' values of one k adjacent),
// a kept weight costs one 16-byte gather and four multiply-adds, a row's four totals are butterflies inside
// its 16 lanes, and lane 16q + 4u + b writes P[m0 + b, 4 (u0 + u) + q].  The next tile's rows are requested from
// memory before the current tile's products and parked in the other half of the LDS buffer after them.
// Bound: LDS gather bandwidth (16 bytes per lane and four multiply-adds); at 10-15 % kept weights that is faster
// than the dense product on the matrix cores, which multiplies the zeros as well.
#include <type_traits>
#include "common.h"
#include "device_math.h"

namespace l355 {

namespace {
constexpr int kWaves = 8;
constexpr int kBW = 4;   // input rows per tile
}

template <int S, int UPW>
__global__ __launch_bounds__(512) void proj_q16_kernel(ProjQ16Args a)
{
    extern __shared__ __attribute__((aligned(16))) float xb[];   // two tile buffers [K][4], 32 KB apart
    constexpr int kBufFloats = 8192;   // a compile-time distance: the buffer becomes the immediate offset of the gathers
    constexpr int PAIRS = UPW * kBW;
    static_assert(PAIRS <= 16 && S % 2 == 0, "pairs fit a 16-lane row; slots come in pairs");
    const int K = a.K, M = a.M, H = a.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const ProjQ16Dir& D = a.d[blockIdx.z];
    const int u0 = (blockIdx.x * kWaves + wave) * UPW;   // first unit of this wave

    float wv[UPW][S];
    unsigned wc[UPW][S / 2];
    {
        const int slots = D.slots;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int unit = (u0 + u < H) ? (u0 + u) : (H - 1);
            float tv[S];
            unsigned tk[S];
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const int ii = i < slots ? i : slots - 1;
                const size_t idx = ((size_t)unit * slots + ii) * 64 + lane;
                tv[i] = D.val[idx];
                tk[i] = D.col[idx];
            }
#pragma unroll
            for (int i = 0; i < S / 2; ++i) wc[u][i] = 0u;
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const bool live = (u0 + u < H) && i < slots;
                wv[u][i] = live ? tv[i] : 0.f;
                wc[u][i >> 1] |= ((live ? tk[i] : 0u) * (kBW * 4u)) << (16 * (i & 1));
            }
        }
    }
    // the few entries of rows longer than 16 S (at most 6 per wave; most waves have none): lane e holds entry e
    float ovf_v = 0.f;
    unsigned ovf_off = 0u;
    int ovf_lane = 0, ovf_n = 0;
    if (D.ovf_ptr != nullptr && u0 < H) {
        const int first = D.ovf_ptr[u0];
        const int idx = first + lane;
        int pos = first;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int nxt = (u0 + u < H) ? D.ovf_ptr[u0 + u + 1] : pos;
            if (idx >= pos && idx < nxt) {
                const unsigned e = D.ovf_ent[idx];
                ovf_off = (e & 0xFFFFu) * (kBW * 4u);
                ovf_lane = 16 * (int)(e >> 16) + u * kBW;
                ovf_v = D.ovf_val[idx];
            }
            pos = nxt;
        }
        ovf_n = pos - first;
        ovf_n = ovf_n < 64 ? ovf_n : 64;
    }
    ovf_n = __builtin_amdgcn_readfirstlane(ovf_n);

    const int lp = lane & 15, row = lane >> 4;
    const int pu = lp / kBW, pb = lp % kBW;
    const int unit_l = u0 + pu;
    const bool pair_ok = lp < PAIRS && unit_l < H;
    const float bias = pair_ok ? D.bias[4 * unit_l + row] : 0.f;
    float* const Pout = D.P;

    // tiles of this workgroup: blockIdx.y, blockIdx.y + gridDim.y, ...
    const int ntiles = (M + kBW - 1) / kBW;
    // thread t stages k = t, t + 512, ...: four coalesced scalar loads per k (one per input row) and one 16-byte LDS
    // write, whose lanes hit consecutive 16-byte chunks (a register transpose of 16-byte loads wrote with a 64-byte
    // stride, four lanes to a bank group)
    constexpr int KPT = 4;                       // k per thread held in registers (covers K <= 2048)
    float xr[KPT][kBW];
    auto request = [&](int tile) {
        const int m0 = tile * kBW;
        const float* rowp[kBW];   // wave-uniform row bases: scalar address arithmetic, one 32-bit lane offset per k
#pragma unroll
        for (int b = 0; b < kBW; ++b) rowp[b] = a.X + (size_t)((m0 + b < M) ? (m0 + b) : (M - 1)) * a.ldx;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const int k = tid + j * 512;
#pragma unroll
            for (int b = 0; b < kBW; ++b) xr[j][b] = (k < K) ? rowp[b][k] : 0.f;
        }
    };
    auto park = [&](int buf) {
        float4* dst = reinterpret_cast<float4*>(xb + (size_t)buf * kBufFloats);
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const int k = tid + j * 512;
            if (k < K) dst[k] = make_float4(xr[j][0], xr[j][1], xr[j][2], xr[j][3]);
        }
    };
    int tile = blockIdx.y;
    if (tile < ntiles) {
        request(tile);
        park(0);
    }
    __syncthreads();
    // one tile; BUF (the buffer it reads) is a compile-time constant, so the gathers address LDS as packed offset +
    // immediate and need no address arithmetic
    auto do_tile = [&](auto buf_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int nxt = tile + gridDim.y;
        if (nxt < ntiles) request(nxt);           // in flight during this tile's products
        const float* hbuf = xb + BUF * kBufFloats;
        if constexpr (S * UPW >= 72) {
            // near the register limit the offsets stay packed two to a register
#pragma unroll
            for (int u = 0; u < UPW; ++u)
#pragma unroll
                for (int i = 0; i < S / 2; ++i) asm volatile("" : "+v"(wc[u][i]));
        }
        float G = 0.f;
        {
            // The wave's UPW * S gathers as one software-pipelined sequence: PD reads are in flight ahead of the
            // multiply-adds that consume them (a 16-byte gather answers after well over a hundred cycles, four
            // multiply-adds issue in sixteen), whatever unit they belong to.
            constexpr int NS = UPW * S;
            constexpr int PD = NS < 10 ? NS : 10;
            auto read_slot = [&](int n) {
                const int u = n / S, i = n % S;
                const unsigned off = (wc[u][i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(hbuf) + off);
            };
            float4 ring[PD];
#pragma unroll
            for (int n = 0; n < PD; ++n) ring[n] = read_slot(n);
            float acc[2][kBW];
            float tot[16];   // per-lane partial sums of the wave's (unit, input row) pairs, pair p = 4 u + b
#pragma unroll
            for (int p = PAIRS; p < 16; ++p) tot[p] = 0.f;
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int u = n / S, i = n % S;
                if (i == 0) {
#pragma unroll
                    for (int b = 0; b < kBW; ++b) acc[0][b] = acc[1][b] = 0.f;
                }
                const float w = wv[u][i];
                const float4 x = ring[n % PD];
                acc[i & 1][0] = fmaf(w, x.x, acc[i & 1][0]);
                acc[i & 1][1] = fmaf(w, x.y, acc[i & 1][1]);
                acc[i & 1][2] = fmaf(w, x.z, acc[i & 1][2]);
                acc[i & 1][3] = fmaf(w, x.w, acc[i & 1][3]);
                if (n + PD < NS) ring[n % PD] = read_slot(n + PD);
                __builtin_amdgcn_sched_barrier(0);
                if (i == S - 1) {
#pragma unroll
                    for (int b = 0; b < kBW; ++b) tot[u * kBW + b] = acc[0][b] + acc[1][b];
                }
            }
            // all sixteen sums over the 16 lanes of a row at once (45 instructions instead of 16 butterflies of four and
            // their selects): lane p of every row ends up with the row's total of pair p
            G = row16_transpose_sum(tot, lp);
        }
        if (ovf_n > 0) {   // wave-uniform; false in almost every wave
            const float4 x = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(hbuf) + ovf_off);
            const float pr[kBW] = {ovf_v * x.x, ovf_v * x.y, ovf_v * x.z, ovf_v * x.w};
            for (int e = 0; e < ovf_n; ++e) {
                const int tgt = __builtin_amdgcn_readlane(ovf_lane, e);
#pragma unroll
                for (int b = 0; b < kBW; ++b) {
                    const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr[b]), e));
                    G += (lane == tgt + b) ? v : 0.f;
                }
            }
        }
        if (nxt < ntiles) park(1 - BUF);          // the other half: nobody reads it during this tile
        __syncthreads();
        // the outputs after the hand-over: the wait for the parked rows would otherwise also wait for this store
        const int mrow = tile * kBW + pb;
        if (pair_ok && mrow < M) Pout[(size_t)mrow * (4 * (size_t)H) + 4 * unit_l + row] = G + bias;
    };
    while (tile < ntiles) {
        do_tile(std::integral_constant<int, 0>{});
        tile += gridDim.y;
        if (tile >= ntiles) break;
        do_tile(std::integral_constant<int, 1>{});
        tile += gridDim.y;
    }
}

// ------------------------------------------------------------------------------------------------ launch
bool proj_q16_supported(int M, int H, int K, int slots)
{
    if (M < 1 || H < 1 || slots < 2 || slots > 24 || (slots & 1)) return false;
    return K >= 1 && K <= 2048;   // four k per thread in registers; two 32 KB tile buffers; 16-bit LDS byte offsets
}


template <int S, int UPW>
static hipError_t launch_cfg(const ProjQ16Args& a, int ndir, hipStream_t s)
{
    const size_t lds = (size_t)2 * 8192 * sizeof(float);   // two tile buffers, 32 KB apart
    auto kern = proj_q16_kernel<S, UPW>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int ug = (a.H + kWaves * UPW - 1) / (kWaves * UPW);
    const int ntiles = (a.M + kBW - 1) / kBW;
    // one round of workgroups over the device (the weights are read once per workgroup)
    int chunks = device_num_cus() / (ug * ndir);
    if (chunks > ntiles) chunks = ntiles;
    if (chunks < 1) chunks = 1;
    hipLaunchKernelGGL(kern, dim3(ug, chunks, ndir), dim3(64 * kWaves), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_proj_q16(const ProjQ16Args& a, int ndir, int slots, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    if (!proj_q16_supported(a.M, a.H, a.K, slots) || ndir < 1 || ndir > 2) return hipErrorInvalidValue;
#define CASE_S(n, u) case n: return launch_cfg<n, u>(a, ndir, s);
    switch (slots) {
        CASE_S(2, 4) CASE_S(4, 4) CASE_S(6, 4) CASE_S(8, 4) CASE_S(10, 4) CASE_S(12, 4) CASE_S(14, 4) CASE_S(16, 4)
        CASE_S(18, 4) CASE_S(20, 4) CASE_S(22, 3) CASE_S(24, 3)
    }
#undef CASE_S
    return hipErrorInvalidValue;
}

}  // namespace l355

// Recurrence of a bf16 dense layer at large batch with the time loop on the device (paper Section 4, cell
// equations; Section 5.1 for the stack this serves).  One launch per (layer, direction).
//
//   R[b][n] = sum_k hb[b][k] * W_h[n][k]      (hb = h_{t-1} rounded to bf16, W_h packed rows n = 4*unit + gate)
//   a = P[t][b][n] + R[b][n];  f,i,o = sigmoid, g = tanh;  c <- f*c + i*g;  h = o*tanh(c)
//
// A 512-thread workgroup owns a 32 (batch) x 128 (packed rows = 32 hidden units) tile for the whole sequence, one
// workgroup per compute unit.  Its eight waves split K; each wave's slice of W_h (128 rows x H/8) stays in
// registers as MFMA operand fragments for all T steps (128 registers at H = 1024), and each thread keeps the cell
// state of its two (batch row, unit) pairs in registers.  What a launch per step re-reads from memory every step
// (W_h: the L2 does not keep it across launches) is read once.
//
// Hidden-state exchange.  h_t (B x H bf16, 512 KB at B = 256, H = 1024) is too large for the tagged 8-byte slots
// the small-batch kernels use, so data and readiness travel separately:
//   producer  the tile's 32 x 32 block of h_t is stored as two contiguous 1 KB pieces of a [H/16][Bp][16] buffer
//             with device-scope write-through stores (workgroup-scope stores, which stay in the XCD's L2, when the
//             tiles of the row block have been found to share an XCD); once the wave's stores have been acknowledged
//             (outstanding-memory counter at zero) and the workgroup has met at a barrier, one thread publishes
//             the step number in the tile's flag, with a store of the same scope.
//   consumer  every wave polls the flags of the tiles that produce the units of its own K slice (device-scope
//             loads, bounded) and then, without a workgroup barrier, reads its operand fragments with device-scope
//             8-byte loads, which do not hit stale lines of this compute unit's vector cache or this XCD's L2.
//             A wave issues its memory instructions in order and none past the branch that ends the poll.  (An
//             acquire fence followed by ordinary cached loads, which lets the 32 compute units of an XCD share one
//             fetch of each line, measured 0.9 us per step slower: the invalidate makes all of them miss first.)
// Two exchange buffers alternate: a tile writes h_{t+1} only after its eight waves, whose K slices together cover
// every tile of the row block, have seen all flags of h_t, and each of those tiles raised its flag after all of its
// waves had finished reading h_{t-1} from the buffer h_{t+1} goes to.
// Flags carry monotonically growing tags, so they are never cleared between steps or launches of one forward.
// Every wait is bounded; an expired wait raises the timeout flag and the kernel runs to its end.
#include "common.h"
#include "device_math.h"
#include "exchange.h"

namespace l355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// KS: k16 steps of a wave's K slice (H = 128 * KS); MT x NT: the tile in 32 x 32 blocks (batch rows x packed rows)
template <int KS, int MT, int NT>
__global__ __launch_bounds__(512) void persist_mfma_bf16_kernel(PersistMfmaArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float part[];  // [8][RM][LDP]
    constexpr int RM = 32 * MT, RN = 32 * NT, UT = RN / 4;       // tile rows (batch), packed rows, hidden units
    constexpr int LDP = RN + 4;
    constexpr int NW = 8, NTH = 512, PAIRS = RM * UT / NTH;
    static_assert(RM * UT % NTH == 0 && PAIRS >= 1, "pairs must divide evenly over the threads");
    const int gm = (a.B + RM - 1) / RM, gn = (4 * a.H) / RN;
    const int nblk = gm * gn;
    // Workgroups are dealt to the eight XCDs in turn.  The tiles of one block of batch rows -- the only ones that
    // exchange h among themselves -- take ids of one residue modulo 8 when the groups fit, so that they can hand h over
    // through one XCD's L2 (checked below); otherwise the tiles that share a W_h panel stay on one XCD.
    int tile_m, tile_n;
    if (a.xcd_local) {
        const int jj = blockIdx.x >> 3;
        tile_m = (blockIdx.x & 7) + 8 * (jj / gn);
        tile_n = jj % gn;
        if (tile_m >= gm) return;                              // padding ids take no part in the exchange
    } else {
        const int per_xcd = (nblk + 7) / 8;
        const int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
        if (logical >= nblk) return;
        tile_n = logical / gm; tile_m = logical % gm;
    }
    const int m0 = tile_m * RM, n0 = tile_n * RN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fk = lane >> 5;
    const int H = a.H, Bp = gm * RM;
    const int kbase = wave * (H / NW);

    // W_h fragments of this wave: rows n0 + 32 j + fr, k = kbase + 16 s + 8 fk .. + 8
    uint4 fb[NT][KS];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int s = 0; s < KS; ++s)
            fb[j][s] = *reinterpret_cast<const uint4*>(a.Wh + (size_t)(n0 + j * 32 + fr) * H + kbase + 16 * s + 8 * fk);

    // this thread's (batch row, unit) pairs
    int pb[PAIRS], pu[PAIRS];
    float c[PAIRS];
#pragma unroll
    for (int r = 0; r < PAIRS; ++r) {
        const int p = tid + NTH * r;
        pb[r] = m0 + p / UT;
        pu[r] = p % UT;
        const int bc = pb[r] < a.B ? pb[r] : a.B - 1;
        c[r] = a.c0 ? a.c0[(size_t)bc * H + (n0 >> 2) + pu[r]] : 0.0f;
    }
    // operand offsets (in bf16 elements) inside an exchange buffer: unit block kbase/16 + s, row m0 + 32 i + fr
    const size_t xbuf = (size_t)H * Bp;                        // elements per exchange buffer
    unsigned aoff[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) aoff[i] = (unsigned)(((kbase >> 4) * Bp + m0 + i * 32 + fr) * 16 + 8 * fk);
    unsigned* const myflag = a.flags + (size_t)tile_m * gn + tile_n;
    // flags of the tiles whose units this wave multiplies: tiles kbase / UT .. (kbase + H/8 - 1) / UT of the row block
    const int ft0 = kbase / UT, ft1 = (kbase + H / NW - 1) / UT;
    const unsigned* const pollflag = a.flags + (size_t)tile_m * gn + (ft0 + lane <= ft1 ? ft0 + lane : ft1);

    bool same_xcd = false;
    if (a.xcd_local)
        same_xcd = group_shares_xcd(a.xcc_ids + (size_t)tile_m * 64, gn, tile_n, a.tag_base + 1u, part, tid, NTH,
                                    a.timeout_flag, a.spin_limit) && !a.device_scope_only;

    for (int s = 0; s < a.T; ++s) {
        const int t = a.reverse ? a.T - 1 - s : s;
        // epilogue operand, requested first
        float4 pre[PAIRS];
#pragma unroll
        for (int r = 0; r < PAIRS; ++r) {
            const int bc = pb[r] < a.B ? pb[r] : a.B - 1;
            pre[r] = *reinterpret_cast<const float4*>(a.P + ((size_t)t * a.B + bc) * (4 * (size_t)H) + n0 + 4 * pu[r]);
        }
        f32x16 acc[MT][NT];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        if (s > 0 || a.has_h0) {
            if (s > 0) {
                // every wave waits for the tiles that produce its own K slice (H/8 units: H/256 tiles, at least one)
                // and goes on by itself: no workgroup barrier between the flags and the operand loads
                const unsigned want = a.tag_base + (unsigned)s;
                unsigned spins = 0;
                // "at least": a producer that has seen everybody's flag of this step may finish the step and raise its
                // flag to the next tag before a slower poller has looked; what that poller needs is still there (the
                // next h goes to the other buffer, and nobody can get two steps ahead of it)
                for (;;) {
                    const int behind = (int)(__hip_atomic_load(pollflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - want) < 0;
                    if (!__builtin_amdgcn_ballot_w64(behind != 0)) break;
                    if (++spins > a.spin_limit) {
                        __hip_atomic_store(a.timeout_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    if ((spins & 255u) == 0 &&
                        __hip_atomic_load(a.timeout_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                        break;
                }
            }
            const uint16_t* hx = a.hx + (size_t)(s & 1) * xbuf;
            uint4 fa[MT][KS];
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int q = 0; q < KS; ++q)
                {
                    // device-scope loads: they do not hit stale lines of this compute unit's vector cache or this XCD's
                    // L2, so no acquire fence (which would make every cached line of the workgroup miss) is needed
                    const unsigned long long* p8 = reinterpret_cast<const unsigned long long*>(hx + aoff[i] + (size_t)q * Bp * 16);
                    const unsigned long long lo = __hip_atomic_load(p8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const unsigned long long hi = __hip_atomic_load(p8 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    fa[i][q] = make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
                }
#pragma unroll
            for (int q = 0; q < KS; ++q)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i][q]),
                                                                           __builtin_bit_cast(bf16x8, fb[j][q]),
                                                                           acc[i][j], 0, 0, 0);
        }
        // partial tiles -> LDS.  Accumulator register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32).
        float* mine = part + (size_t)wave * RM * LDP;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = i * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                    mine[m * LDP + j * 32 + fr] = acc[i][j][v];
                }
        __syncthreads();
        uint16_t* hxo = a.hx + (size_t)((s + 1) & 1) * xbuf;
        const bool last = (s == a.T - 1);
        float hkeep[PAIRS];
#pragma unroll
        for (int r = 0; r < PAIRS; ++r) {
            const int m = pb[r] - m0, u = pu[r];
            float4 sum = pre[r];
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float4 q = *reinterpret_cast<const float4*>(part + ((size_t)w * RM + m) * LDP + 4 * u);
                sum.x += q.x;
                sum.y += q.y;
                sum.z += q.z;
                sum.w += q.w;
            }
            const float f = sigmoidf_fast(sum.x), ig = sigmoidf_fast(sum.y), o = sigmoidf_fast(sum.z), g = tanhf_fast(sum.w);
            const float cn = fmaf(f, c[r], ig * g);
            const float hn = o * tanhf_fast(cn);
            c[r] = cn;
            // two neighbouring units per 32-bit word of the exchange buffer (rows beyond the batch included: they
            // are only ever multiplied into accumulator rows that are never stored)
            const unsigned hbits = f32_to_bf16_bits(hn);
            const unsigned other = (unsigned)__builtin_amdgcn_update_dpp(0, (int)hbits, 0xB1, 0xF, 0xF, true);
            if ((u & 1) == 0 && !last)
                exchange_store(reinterpret_cast<unsigned*>(hxo + ((size_t)(((n0 >> 2) + u) >> 4) * Bp + pb[r]) * 16 + (u & 15)),
                               hbits | (other << 16), same_xcd);
            hkeep[r] = hn;
        }
        if (!last) {
            // exchange stores acknowledged by every wave, then the tile's flag; the barrier also keeps the next step's
            // partial tiles out of LDS until every thread has read this step's
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();
            if (tid == 0) exchange_store(myflag, a.tag_base + (unsigned)s + 1u, same_xcd);
        }
        // outputs after the publication: nothing on the way of h_t
#pragma unroll
        for (int r = 0; r < PAIRS; ++r) {
            if (pb[r] < a.B) {
                const int j = (n0 >> 2) + pu[r];
                const size_t row = (size_t)t * a.B + pb[r];
                if (a.y) a.y[row * a.y_ld + j] = hkeep[r];
                if (a.yb) a.yb[row * a.yb_ld + j] = (uint16_t)f32_to_bf16_bits(hkeep[r]);
                if (last) {
                    if (a.hT) a.hT[(size_t)pb[r] * H + j] = hkeep[r];
                    if (a.cT) a.cT[(size_t)pb[r] * H + j] = c[r];
                }
            }
        }
    }
}

// h0 (fp32 [B][H]) -> exchange buffer 0 in the [H/16][Bp][16] bf16 layout
__global__ void h0_to_exchange_kernel(const float* __restrict__ h0, uint16_t* __restrict__ hx, int B, int H, int Bp)
{
    const size_t n = (size_t)B * H;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t b = i / H, k = i % H;
        hx[((k >> 4) * Bp + b) * 16 + (k & 15)] = f32_to_bf16_bits(h0[i]);
    }
}

// The tile is 32 batch rows x 128 packed rows (32 hidden units): a compute unit pulls 64 KB of h per step.  (The first
// version used 64 x 64 tiles, 128 KB per step; the step is bound by that read, and the 32-row shape never needs more
// tiles than the 64-row one.)
constexpr int kMT = 1, kNT = 4;

bool persist_mfma_supported(int B, int H)
{
    if (B < 32 || H % 128 != 0 || H > 1024) return false;
    const int gn = 4 * H / (32 * kNT);
    const int tiles = ((B + 32 * kMT - 1) / (32 * kMT)) * gn;
    return ((tiles + 7) / 8) * 8 <= device_num_cus() && gn <= 64;
}

size_t persist_mfma_exchange_bytes(int B, int H)
{
    const size_t Bp = (size_t)((B + 32 * kMT - 1) / (32 * kMT)) * (32 * kMT);
    return 2 * (size_t)H * Bp * sizeof(uint16_t);
}
// flags (one per tile, rounded up to an even count), then 64 two-word slots per block of batch rows for the XCD ids
size_t persist_mfma_ids_offset(int B, int H)
{
    const size_t tiles = (size_t)((B + 32 * kMT - 1) / (32 * kMT)) * (4 * H / (32 * kNT));
    return (tiles + 1) & ~(size_t)1;
}
size_t persist_mfma_flag_count(int B, int H)
{
    return persist_mfma_ids_offset(B, H) + (size_t)((B + 32 * kMT - 1) / (32 * kMT)) * 64 * 2;
}

template <int KS, int MT, int NT>
static hipError_t launch_shape(const PersistMfmaArgs& a, const float* h0, bool cooperative, hipStream_t s)
{
    constexpr int RM = 32 * MT, RN = 32 * NT;
    const int gm = (a.B + RM - 1) / RM, gn = (4 * a.H) / RN;
    const size_t lds = (size_t)8 * RM * (RN + 4) * sizeof(float);
    PersistMfmaArgs args = a;
    args.has_h0 = h0 != nullptr;
    // one XCD holds an eighth of the compute units; its share of the row blocks (gn tiles each) must fit there
    const int groups_per_xcd = (gm + 7) / 8;
    args.xcd_local = (a.xcc_ids != nullptr && gn <= 64 && groups_per_xcd * gn <= device_num_cus() / 8) ? 1 : 0;
    const int grid = args.xcd_local ? 8 * groups_per_xcd * gn : ((gm * gn + 7) / 8) * 8;
    if (h0) {
        const size_t n = (size_t)a.B * a.H;
        int g = (int)((n + 255) / 256);
        if (g > 2048) g = 2048;
        hipLaunchKernelGGL(h0_to_exchange_kernel, dim3(g), dim3(256), 0, s, h0, a.hx, a.B, a.H, gm * RM);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const void* kern = (const void*)persist_mfma_bf16_kernel<KS, MT, NT>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    void* kargs[] = {(void*)&args};
    // every workgroup must be resident at the same time: at most one per compute unit (135-139 KB of LDS each)
    if (cooperative) return hipLaunchCooperativeKernel(kern, dim3(grid), dim3(512), kargs, (unsigned)lds, s);
    return hipLaunchKernel(kern, dim3(grid), dim3(512), kargs, lds, s);
}

template <int KS>
static hipError_t launch_ks(const PersistMfmaArgs& a, const float* h0, bool cooperative, hipStream_t s)
{
    return launch_shape<KS, kMT, kNT>(a, h0, cooperative, s);
}

hipError_t launch_persist_mfma_bf16(const PersistMfmaArgs& a, const float* h0, bool cooperative, hipStream_t s)
{
    if (a.B <= 0 || a.H <= 0 || a.T <= 0) return hipSuccess;
    if (!persist_mfma_supported(a.B, a.H)) return hipErrorInvalidValue;
    switch (a.H / 128) {
        case 1: return launch_ks<1>(a, h0, cooperative, s);
        case 2: return launch_ks<2>(a, h0, cooperative, s);
        case 3: return launch_ks<3>(a, h0, cooperative, s);
        case 4: return launch_ks<4>(a, h0, cooperative, s);
        case 5: return launch_ks<5>(a, h0, cooperative, s);
        case 6: return launch_ks<6>(a, h0, cooperative, s);
        case 7: return launch_ks<7>(a, h0, cooperative, s);
        case 8: return launch_ks<8>(a, h0, cooperative, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace l355

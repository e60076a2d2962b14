// Input projection on the matrix cores:  P[m][n] = bias[n] + sum_k X[m][k] * W[n][k]
// (the x-part of the gate pre-activation W.[x_t, h_{t-1}] + b of the paper's cell equations, Section 4, for
// all timesteps at once: m runs over (t, b), n over packed gate rows).  Both operands are contiguous along k.
//
// One 256-thread workgroup (2 x 2 wavefronts) computes a BM x BN tile; each wave owns TM x TN MFMA tiles of
// 32 x 32.  K is walked in slabs that are double-buffered in LDS: the global loads of slab i+1 are issued
// before the MFMAs of slab i and written to the other LDS buffer after them, one barrier per slab.
// LDS rows are padded by 16 bytes so that the 16-byte fragment reads of eight consecutive lanes fall into
// disjoint banks.  Workgroups are renumbered so that consecutive tiles (which share operand panels) land on
// the same XCD and therefore in the same L2: the hardware deals workgroup ids round-robin over the 8 XCDs.
#include "common.h"
#include "device_math.h"

namespace l355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kXcds = 8;
constexpr int kGroupM = 4;

// Map the hardware workgroup id to a tile, XCD-aware and grouped along m.  Returns false for padding ids.
__device__ __forceinline__ bool tile_of_block(int pid, int gm, int gn, int& tm, int& tn)
{
    const int nblk = gm * gn;
    const int per_xcd = (nblk + kXcds - 1) / kXcds;
    const int logical = (pid % kXcds) * per_xcd + pid / kXcds;
    if (logical >= nblk) return false;
    const int span = kGroupM * gn;
    const int group = logical / span, in = logical % span;
    const int first = group * kGroupM;
    const int gsz = (gm - first) < kGroupM ? (gm - first) : kGroupM;
    tm = first + in % gsz;
    tn = in / gsz;
    return true;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}

// ---------------------------------------------------------------------------------------------------------
// bf16 operands, fp32 accumulation.  X_F32: the operand X is stored as fp32 and rounded to bf16 on the way in.
// Requires K % 8 == 0 (16-byte chunks of bf16 along k).
// ---------------------------------------------------------------------------------------------------------
template <int TM, int TN, bool X_F32>
__global__ __launch_bounds__(256, 2) void proj_mfma_bf16_kernel(const void* __restrict__ Xv, int ldx,
                                                             const uint16_t* __restrict__ W, const float* __restrict__ bias,
                                                             float* __restrict__ P, int M, int N, int K, int gm, int gn)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32, BK = 32;
    constexpr int LDR = BK + 8;                      // padded row length in bf16 elements (80 bytes)
    constexpr int ACH = BM * (BK / 8) / 256;         // 16-byte chunks of the X slab per thread
    constexpr int BCH = BN * (BK / 8) / 256;
    static_assert(ACH >= 1 && BCH >= 1, "tile too small for 256 threads");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem);              // [2][BM][LDR]
    uint16_t* Bs = As + 2 * BM * LDR;                              // [2][BN][LDR]

    int tile_m, tile_n;
    if (!tile_of_block(blockIdx.x, gm, gn, tile_m, tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fk = lane >> 5;        // fragment row / k-half of this lane

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 ra[ACH], rb[BCH];
    auto load_slab = [&](int k0) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            const int m = m0 + row, k = k0 + 8 * kc;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (m < M && k < K) {
                if (X_F32) {
                    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(Xv) + (size_t)m * ldx + k);
                    const float4 lo = p[0], hi = p[1];
                    v.x = pack_bf16x2(lo.x, lo.y);
                    v.y = pack_bf16x2(lo.z, lo.w);
                    v.z = pack_bf16x2(hi.x, hi.y);
                    v.w = pack_bf16x2(hi.z, hi.w);
                } else {
                    v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(Xv) + (size_t)m * ldx + k);
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            const int n = n0 + row, k = k0 + 8 * kc;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (n < N && k < K) v = *reinterpret_cast<const uint4*>(W + (size_t)n * K + k);
            rb[i] = v;
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            *reinterpret_cast<uint4*>(As + ((size_t)buf * BM + row) * LDR + 8 * kc) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            *reinterpret_cast<uint4*>(Bs + ((size_t)buf * BN + row) * LDR + 8 * kc) = rb[i];
        }
    };

    const int nslab = (K + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();
    for (int kt = 0; kt < nslab; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nslab) load_slab((kt + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                            As + ((size_t)buf * BM + (wm * TM + i) * 32 + fr) * LDR + ks * 16 + fk * 8));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                            Bs + ((size_t)buf * BN + (wn * TN + j) * 32 + fr) * LDR + ks * 16 + fk * 8));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nslab) store_slab(buf ^ 1);
        __syncthreads();
    }
    // epilogue: accumulator register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32) of its 32x32 tile
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + fr;
        if (n >= N) continue;
        const float bn = bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mb = m0 + (wm * TM + i) * 32 + 4 * fk;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                if (m < M) P[(size_t)m * N + n] = acc[i][j][v] + bn;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// bf16 operands, slabs brought from global memory straight into LDS (no register staging), double-buffered.
// A direct load writes the 16 bytes of lane i at LDS offset base + 16*i, so one wave instruction fills 16 rows
// of 64 bytes; rows are not padded.  Bank conflicts are avoided by permuting the four 16-byte chunks of a row:
// chunk kc of row r is kept at position kc ^ ((r >> 1) & 3), both when a lane picks the global chunk that belongs
// at its LDS position and when a fragment is read.  Needs K % 32 == 0; rows beyond M / N are clamped to the
// last valid row (their products are never stored).
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void wait_vmcnt(int n)
{
    // s_waitcnt on gfx9: vmcnt = bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] left unconstrained
    if (n <= 0) __builtin_amdgcn_s_waitcnt(0x0F70);
    else if (n == 4) __builtin_amdgcn_s_waitcnt(0x0F74);
    else if (n == 6) __builtin_amdgcn_s_waitcnt(0x0F76);
    else if (n == 8) __builtin_amdgcn_s_waitcnt(0x0F78);
    else if (n == 12) __builtin_amdgcn_s_waitcnt(0x0F7C);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
}

template <int TM, int TN>
__global__ __launch_bounds__(256, 2) void proj_mfma_bf16_dlds_kernel(const uint16_t* __restrict__ X, int ldx,
                                                                   const uint16_t* __restrict__ W,
                                                                   const float* __restrict__ bias, float* __restrict__ P,
                                                                   int M, int N, int K, int gm, int gn)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32, BK = 32, NST = 2;
    constexpr int ROWB = BK * 2;                          // bytes per LDS row
    constexpr int STAGE = (BM + BN) * ROWB;               // bytes per stage
    constexpr int AI = BM / 64, BI = BN / 64;             // direct-load instructions per wave and slab (16 rows each)
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    int tile_m, tile_n;
    if (!tile_of_block(blockIdx.x, gm, gn, tile_m, tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fk = lane >> 5;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // per-lane source pointers of the direct loads (advance by BK elements per slab)
    const uint16_t* asrc[AI];
    const uint16_t* bsrc[BI];
#pragma unroll
    for (int i = 0; i < AI; ++i) {
        const int row = (wave * AI + i) * 16 + (lane >> 2);   // row inside the X slab
        const int kc = (lane & 3) ^ ((row >> 1) & 3);
        int m = m0 + row;
        if (m > M - 1) m = M - 1;
        asrc[i] = X + (size_t)m * ldx + 8 * kc;
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
        const int row = (wave * BI + i) * 16 + (lane >> 2);
        const int kc = (lane & 3) ^ ((row >> 1) & 3);
        int n = n0 + row;
        if (n > N - 1) n = N - 1;
        bsrc[i] = W + (size_t)n * K + 8 * kc;
    }
    auto issue_slab = [&](int kt) {
        unsigned char* st = smem + (size_t)(kt % NST) * STAGE;
        const size_t koff = (size_t)kt * BK;
#pragma unroll
        for (int i = 0; i < AI; ++i)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(asrc[i] + koff),
                                             (void __attribute__((address_space(3)))*)(st + (size_t)(wave * AI + i) * 16 * ROWB),
                                             16, 0, 0);
#pragma unroll
        for (int i = 0; i < BI; ++i)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(bsrc[i] + koff),
                                             (void __attribute__((address_space(3)))*)(st + (size_t)BM * ROWB + (size_t)(wave * BI + i) * 16 * ROWB),
                                             16, 0, 0);
    };

    const int nslab = K / BK;
    issue_slab(0);
    for (int kt = 0; kt < nslab; ++kt) {
        // slab kt must have landed; the compiler also waits for every outstanding direct load before LDS is
        // read, so the prefetch distance is one slab and latency is hidden by the other resident workgroups
        wait_vmcnt(0);
        __syncthreads();
        if (kt + 1 < nslab) issue_slab(kt + 1);      // refills the buffer every wave finished reading before the barrier
        const unsigned char* As = smem + (size_t)(kt % NST) * STAGE;
        const unsigned char* Bs = As + (size_t)BM * ROWB;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int rr = (wm * TM + i) * 32 + fr;
                const int pos = (ks * 2 + fk) ^ ((rr >> 1) & 3);
                fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(As + (size_t)rr * ROWB + pos * 16));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int rr = (wn * TN + j) * 32 + fr;
                const int pos = (ks * 2 + fk) ^ ((rr >> 1) & 3);
                fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Bs + (size_t)rr * ROWB + pos * 16));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + fr;
        if (n >= N) continue;
        const float bn = bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mb = m0 + (wm * TM + i) * 32 + 4 * fk;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                if (m < M) P[(size_t)m * N + n] = acc[i][j][v] + bn;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Large-M bf16 variant: 256 x 256 tile, eight waves (2 x 4, wave tile 128 x 64), 32-wide K slabs brought straight
// into LDS through a four-deep ring (128 KB of LDS, one workgroup per compute unit), so that three slabs are
// in flight while one is consumed: the L2 round trip (about 1.3 us under load) is longer than the MFMA work of
// one slab.  Fragment reads are issued as explicit ds_read_b128 instructions: the compiler cannot see that an
// LDS read depends on a particular direct-to-LDS load and would otherwise wait for ALL outstanding loads before
// every read, which collapses the ring to depth one.  The dependency is kept by hand instead: a counted
// s_waitcnt on the vector-memory counter (slab kt has landed once only the loads of the younger slabs are
// outstanding), then the workgroup barrier, then the reads.
// Chunk kc of row r lives at position kc ^ ((r >> 1) & 3) of its 64-byte row (bank-conflict-free 16-byte reads).
// Needs K % 32 == 0.
// ---------------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ u32x4 lds_read_b128(unsigned addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}

template <int NWN>  // waves along n: 4 -> eight waves of 128 x 64, 2 -> four waves of 128 x 128
__global__ __launch_bounds__(128 * NWN) void proj_mfma_bf16_big_kernel(const uint16_t* __restrict__ X, int ldx,
                                                                 const uint16_t* __restrict__ W,
                                                                 const float* __restrict__ bias, float* __restrict__ P,
                                                                 int M, int N, int K, int gm, int gn)
{
    constexpr int BM = 256, BN = 256, BK = 32, NST = 4;
    constexpr int NW = 2 * NWN;                           // waves per workgroup
    constexpr int TM = 4, TN = 8 / NWN;                   // 32x32 tiles per wave
    constexpr int ROWB = BK * 2;                          // 64 bytes per LDS row
    constexpr int STAGE = (BM + BN) * ROWB;               // 32 KB
    constexpr int LI = (BM + BN) / 16 / NW;               // direct-load instructions per wave and slab (16 rows each)
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    int tile_m, tile_n;
    if (!tile_of_block(blockIdx.x, gm, gn, tile_m, tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / NWN, wn = wave % NWN;           // 2 x NWN waves: rows wm*128, cols wn*32*TN
    const int fr = lane & 31, fk = lane >> 5;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // direct loads: instruction q (0..31) of a slab covers LDS rows 16q..16q+15 of the combined [X rows | W rows]
    const uint16_t* src[LI];
#pragma unroll
    for (int i = 0; i < LI; ++i) {
        const int q = wave * LI + i;
        const int row = q * 16 + (lane >> 2);             // 0..511: X rows then W rows
        const int kc = (lane & 3) ^ ((row >> 1) & 3);
        if (row < BM) {
            int m = m0 + row;
            if (m > M - 1) m = M - 1;
            src[i] = X + (size_t)m * ldx + 8 * kc;
        } else {
            int n = n0 + row - BM;
            if (n > N - 1) n = N - 1;
            src[i] = W + (size_t)n * K + 8 * kc;
        }
    }
    auto issue_slab = [&](int kt) {
        unsigned char* st = smem + (size_t)(kt % NST) * STAGE;
        const size_t koff = (size_t)kt * BK;
#pragma unroll
        for (int i = 0; i < LI; ++i)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(src[i] + koff),
                                             (void __attribute__((address_space(3)))*)(st + (size_t)(wave * LI + i) * 16 * ROWB),
                                             16, 0, 0);
    };
    // byte offsets of this lane's fragments inside a stage (two k16 steps per slab)
    unsigned offa[2][TM], offb[2][TN];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rr = (wm * TM + i) * 32 + fr;
            offa[ks][i] = (unsigned)(rr * ROWB + (((ks * 2 + fk) ^ ((rr >> 1) & 3)) * 16));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int rr = (wn * TN + j) * 32 + fr;
            offb[ks][j] = (unsigned)(BM * ROWB + rr * ROWB + (((ks * 2 + fk) ^ ((rr >> 1) & 3)) * 16));
        }
    }

    const int nslab = K / BK;
    issue_slab(0);
    if (nslab > 1) issue_slab(1);
    if (nslab > 2) issue_slab(2);
    for (int kt = 0; kt < nslab; ++kt) {
        // slab kt has landed once only the loads of slabs kt+1 and kt+2 (LI each) can still be outstanding
        const int younger = (nslab - 1 - kt) < 2 ? (nslab - 1 - kt) : 2;
        if (younger == 2) wait_vmcnt(2 * LI); else if (younger == 1) wait_vmcnt(LI); else wait_vmcnt(0);
        // bare barrier: __syncthreads() carries a workgroup fence, for which the compiler drains every outstanding
        // direct-to-LDS load; the ordering needed here is exactly the counted wait above plus the barrier
        __builtin_amdgcn_s_barrier();
        if (kt + 3 < nslab) issue_slab(kt + 3);          // refills the buffer consumed in iteration kt-1
        const unsigned st = lds0 + (unsigned)((kt % NST) * STAGE);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            u32x4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = lds_read_b128(st + offa[ks][i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = lds_read_b128(st + offb[ks][j]);
            // wait for the LDS reads; the fragments are operands of the wait so that no MFMA can move above it
            if constexpr (TN == 2)
                asm volatile("s_waitcnt lgkmcnt(0)"
                             : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1])
                             :
                             : "memory");
            else
                asm volatile("s_waitcnt lgkmcnt(0)"
                             : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]),
                               "+v"(fb[3])
                             :
                             : "memory");
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                                       __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + fr;
        if (n >= N) continue;
        const float bn = bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mb = m0 + (wm * TM + i) * 32 + 4 * fk;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                if (m < M) P[(size_t)m * N + n] = acc[i][j][v] + bn;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// fp32 operands on the fp32 matrix instruction (32x32x2).  Requires K % 4 == 0 (16-byte chunks along k).
// Each lane reads four consecutive k of its fragment row at once and feeds them to four MFMAs; which k a lane
// contributes to which MFMA is the same for both operands, which is all a sum over k needs.
// ---------------------------------------------------------------------------------------------------------
template <int TM, int TN>
__global__ __launch_bounds__(256) void proj_mfma_f32_kernel(const float* __restrict__ X, int ldx,
                                                            const float* __restrict__ W0, const float* __restrict__ bias0,
                                                            float* __restrict__ P0, const float* __restrict__ W1,
                                                            const float* __restrict__ bias1, float* __restrict__ P1,
                                                            int M, int N, int K, int gm, int gn)
{
    // blockIdx.y selects the direction: both directions of a layer read the same X, so one launch covers both
    // and the second direction's tiles fill the tail of the first
    const float* __restrict__ W = blockIdx.y ? W1 : W0;
    const float* __restrict__ bias = blockIdx.y ? bias1 : bias0;
    float* __restrict__ P = blockIdx.y ? P1 : P0;
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32, BK = 16;
    constexpr int LDR = BK + 4;                      // padded row length in floats (80 bytes)
    constexpr int ACH = (BM * (BK / 4) + 255) / 256;
    constexpr int BCH = (BN * (BK / 4) + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* As = reinterpret_cast<float*>(smem);                    // [2][BM][LDR]
    float* Bs = As + 2 * BM * LDR;                                 // [2][BN][LDR]

    int tile_m, tile_n;
    if (!tile_of_block(blockIdx.x, gm, gn, tile_m, tile_n)) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fk = lane >> 5;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    float4 ra[ACH], rb[BCH];
    auto load_slab = [&](int k0) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            const int m = m0 + row, k = k0 + 4 * kc;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < BM && m < M && k < K) v = *reinterpret_cast<const float4*>(X + (size_t)m * ldx + k);
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            const int n = n0 + row, k = k0 + 4 * kc;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < BN && n < N && k < K) v = *reinterpret_cast<const float4*>(W + (size_t)n * K + k);
            rb[i] = v;
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            if (row < BM) *reinterpret_cast<float4*>(As + ((size_t)buf * BM + row) * LDR + 4 * kc) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i, row = c >> 2, kc = c & 3;
            if (row < BN) *reinterpret_cast<float4*>(Bs + ((size_t)buf * BN + row) * LDR + 4 * kc) = rb[i];
        }
    };

    const int nslab = (K + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();
    for (int kt = 0; kt < nslab; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nslab) load_slab((kt + 1) * BK);
#pragma unroll
        for (int kg = 0; kg < BK / 8; ++kg) {
            float4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const float4*>(As + ((size_t)buf * BM + (wm * TM + i) * 32 + fr) * LDR + kg * 8 + fk * 4);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const float4*>(Bs + ((size_t)buf * BN + (wn * TN + j) * 32 + fr) * LDR + kg * 8 + fk * 4);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].x, fb[j].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].y, fb[j].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].z, fb[j].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i].w, fb[j].w, acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < nslab) store_slab(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + fr;
        if (n >= N) continue;
        const float bn = bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mb = m0 + (wm * TM + i) * 32 + 4 * fk;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                if (m < M) P[(size_t)m * N + n] = acc[i][j][v] + bn;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// fp32, at most 64 rows of X (batch-1 sequences: M = T).  The product is a stream over W (read once, 4H*K*4
// bytes) with X resident in L2, so there is no LDS pipeline: a workgroup owns 32 packed rows of W for all of
// X, its four waves split K and stream their operand fragments from global memory straight into registers
// (16 bytes per lane and row, eight k-blocks in flight), and the four partial 64 x 32 tiles are summed through
// LDS in a fixed order.  Requires K % 16 == 0.
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void proj_mfma_f32_skinny_kernel(const float* __restrict__ X, int ldx,
                                                                   const float* __restrict__ W,
                                                                   const float* __restrict__ bias, float* __restrict__ P,
                                                                   int M, int N, int K)
{
    __shared__ float part[4][64][33];
    const int n0 = blockIdx.x * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fk = lane >> 5;
    // K is cut into four contiguous quarters (multiples of 8), one per wave
    const int kq = ((K / 8 + 3) / 4) * 8;
    const int kbeg = wave * kq, kend = (kbeg + kq) < K ? (kbeg + kq) : K;
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    int m0r = fr, m1r = 32 + fr;
    if (m0r > M - 1) m0r = M - 1;   // rows beyond M are computed on a valid row and never stored
    if (m1r > M - 1) m1r = M - 1;
    int nr = n0 + fr;
    if (nr > N - 1) nr = N - 1;
    const float* a0 = X + (size_t)m0r * ldx + fk * 4;
    const float* a1 = X + (size_t)m1r * ldx + fk * 4;
    const float* bw = W + (size_t)nr * K + fk * 4;
    constexpr int UN = 8;            // k-blocks of 8 requested together
    for (int k0 = kbeg; k0 < kend; k0 += 8 * UN) {
        float4 fa0[UN], fa1[UN], fb[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + 8 * u;
            const bool ok = k < kend;
            fa0[u] = ok ? *reinterpret_cast<const float4*>(a0 + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            fa1[u] = ok ? *reinterpret_cast<const float4*>(a1 + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            fb[u] = ok ? *reinterpret_cast<const float4*>(bw + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa0[u].x, fb[u].x, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa1[u].x, fb[u].x, acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa0[u].y, fb[u].y, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa1[u].y, fb[u].y, acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa0[u].z, fb[u].z, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa1[u].z, fb[u].z, acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa0[u].w, fb[u].w, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa1[u].w, fb[u].w, acc[1], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) part[wave][i * 32 + 8 * (v >> 2) + 4 * fk + (v & 3)][fr] = acc[i][v];
    __syncthreads();
    for (int e = tid; e < 64 * 32; e += 256) {
        const int m = e >> 5, n = e & 31;
        if (m < M && n0 + n < N)
            P[(size_t)m * N + n0 + n] = ((part[0][m][n] + part[1][m][n]) + (part[2][m][n] + part[3][m][n])) + bias[n0 + n];
    }
}

// ------------------------------------------------------------------------------------------------ launchers
bool proj_mfma_supported(bool w_bf16, int K, int ldx);

template <int TM, int TN, bool X_F32>
static hipError_t launch_bf16(const void* X, int ldx, const uint16_t* W, const float* bias, float* P, int M, int N,
                              int K, hipStream_t s)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    const int gm = (M + BM - 1) / BM, gn = (N + BN - 1) / BN;
    const int grid = ((gm * gn + kXcds - 1) / kXcds) * kXcds;
    const size_t lds = 2 * (size_t)(BM + BN) * (32 + 8) * sizeof(uint16_t);
    auto kern = proj_mfma_bf16_kernel<TM, TN, X_F32>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, X, ldx, W, bias, P, M, N, K, gm, gn);
    return hipGetLastError();
}

template <int TM, int TN>
static hipError_t launch_bf16_dlds(const uint16_t* X, int ldx, const uint16_t* W, const float* bias, float* P, int M,
                                   int N, int K, hipStream_t s)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    const int gm = (M + BM - 1) / BM, gn = (N + BN - 1) / BN;
    const int grid = ((gm * gn + kXcds - 1) / kXcds) * kXcds;
    const size_t lds = 2 * (size_t)(BM + BN) * 64;
    auto kern = proj_mfma_bf16_dlds_kernel<TM, TN>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, X, ldx, W, bias, P, M, N, K, gm, gn);
    return hipGetLastError();
}

static hipError_t launch_bf16_big(const uint16_t* X, int ldx, const uint16_t* W, const float* bias, float* P, int M,
                                  int N, int K, hipStream_t s)
{
    const int gm = (M + 255) / 256, gn = (N + 255) / 256;
    const int grid = ((gm * gn + kXcds - 1) / kXcds) * kXcds;
    const size_t lds = 4 * (size_t)512 * 64;
    // eight waves of 128 x 64 measured 1.4x faster than four waves of 128 x 128 (whose 256 accumulator registers
    // leave one wave per SIMD and force accumulator/vector register shuffling)
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)proj_mfma_bf16_big_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(proj_mfma_bf16_big_kernel<4>, dim3(grid), dim3(512), lds, s, X, ldx, W, bias, P, M, N, K, gm, gn);
    return hipGetLastError();
}

template <int TM, int TN>
static hipError_t launch_f32(const float* X, int ldx, const float* W, const float* bias, float* P, const float* W1,
                             const float* bias1, float* P1, int M, int N, int K, hipStream_t s)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    const int gm = (M + BM - 1) / BM, gn = (N + BN - 1) / BN;
    const int grid = ((gm * gn + kXcds - 1) / kXcds) * kXcds;
    const size_t lds = 2 * (size_t)(BM + BN) * (16 + 4) * sizeof(float);
    hipLaunchKernelGGL((proj_mfma_f32_kernel<TM, TN>), dim3(grid, W1 ? 2 : 1), dim3(256), lds, s, X, ldx, W, bias, P, W1,
                       bias1, P1, M, N, K, gm, gn);
    return hipGetLastError();
}

// fp32, two directions of one layer (same X) in one launch
hipError_t launch_proj_mfma_f32_pair(const float* X, int ldx, const float* W0, const float* bias0, float* P0,
                                     const float* W1, const float* bias1, float* P1, int M, int N, int K, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    if (!proj_mfma_supported(false, K, ldx)) return hipErrorInvalidValue;
    if (M <= 64) return launch_f32<1, 1>(X, ldx, W0, bias0, P0, W1, bias1, P1, M, N, K, s);
    return launch_f32<2, 2>(X, ldx, W0, bias0, P0, W1, bias1, P1, M, N, K, s);
}

bool proj_mfma_supported(bool w_bf16, int K, int ldx)
{
    return w_bf16 ? (K % 8 == 0 && ldx % 8 == 0) : (K % 4 == 0 && ldx % 4 == 0);
}

hipError_t launch_proj_mfma(const void* X, bool x_bf16, int ldx, const void* W, bool w_bf16, const float* bias, float* P,
                            int M, int N, int K, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    if (!proj_mfma_supported(w_bf16, K, ldx)) return hipErrorInvalidValue;
    if (w_bf16) {
        const uint16_t* Wb = (const uint16_t*)W;
        if (M <= 64) {
            return x_bf16 ? launch_bf16<1, 1, false>(X, ldx, Wb, bias, P, M, N, K, s)
                          : launch_bf16<1, 1, true>(X, ldx, Wb, bias, P, M, N, K, s);
        }
        if (M <= 1024) {
            return x_bf16 ? launch_bf16<2, 2, false>(X, ldx, Wb, bias, P, M, N, K, s)
                          : launch_bf16<2, 2, true>(X, ldx, Wb, bias, P, M, N, K, s);
        }
        if (x_bf16 && K % 32 == 0 && M >= 2048 && N >= 512)
            return launch_bf16_big((const uint16_t*)X, ldx, Wb, bias, P, M, N, K, s);
        if (x_bf16 && K % 32 == 0)
            return launch_bf16_dlds<4, 2>((const uint16_t*)X, ldx, Wb, bias, P, M, N, K, s);
        return x_bf16 ? launch_bf16<4, 2, false>(X, ldx, Wb, bias, P, M, N, K, s)
                      : launch_bf16<4, 2, true>(X, ldx, Wb, bias, P, M, N, K, s);
    }
    if (x_bf16) return hipErrorInvalidValue;
    if (M <= 64 && K % 16 == 0 && ldx % 4 == 0) {
        hipLaunchKernelGGL(proj_mfma_f32_skinny_kernel, dim3((N + 31) / 32), dim3(256), 0, s, (const float*)X, ldx,
                           (const float*)W, bias, P, M, N, K);
        return hipGetLastError();
    }
    if (M <= 64) return launch_f32<1, 1>((const float*)X, ldx, (const float*)W, bias, P, nullptr, nullptr, nullptr, M, N, K, s);
    return launch_f32<2, 2>((const float*)X, ldx, (const float*)W, bias, P, nullptr, nullptr, nullptr, M, N, K, s);
}

}  // namespace l355

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

// Permutation of the 16-byte chunks of an unpadded LDS row r holding `ch` chunks (4: 64-byte rows, 8: 128-byte
// rows).  A 16-byte read by 16 consecutive rows at the same logical chunk then covers all 64 four-byte banks
// (256 bytes): with 128-byte rows bit 0 of r already selects the half of the bank space, with 64-byte rows bits
// 0-1 select the quarter, and the row bits above them are folded into the chunk position.  Measured at the full
// LDS read rate (256 bytes per cycle); folding in bits 1-2 of 64-byte rows instead reads at half of it.
__device__ __forceinline__ constexpr int chunk_swizzle(int r, int ch) { return ch == 8 ? ((r >> 1) & 7) : ((r >> 2) & 3); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}

// ---------------------------------------------------------------------------------------------------------
// bf16 operands, fp32 accumulation.  X_F32: the operand X is stored as fp32 and rounded to bf16 on the way in.
// Requires K % 8 == 0 (16-byte chunks of bf16 along k).
// ---------------------------------------------------------------------------------------------------------
// Epilogue shared by the MFMA projections: P = acc + bias for a wave's TM x TN grid of 32x32 tiles whose first
// element is (mw0, nw0).  Accumulator register v of lane l is element (8*(v/4) + 4*(l/32) + v%4, l%32) of its
// tile.  The bias is added to every accumulator before the first store, outside any bounds check: stores count on
// the same outstanding-memory counter as loads, so a wait for the bias placed inside each guarded store would
// also wait for the previous store to be acknowledged and serialise the whole epilogue.  Interior tiles take a
// path with no per-row checks.
template <int TM, int TN>
__device__ __forceinline__ void store_acc_tiles(f32x16 (&acc)[TM][TN], const float* __restrict__ bias,
                                                float* __restrict__ P, int M, int N, int mw0, int nw0, int fr, int fk)
{
    float bn[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = nw0 + j * 32 + fr;
        bn[j] = bias[n < N ? n : N - 1];
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] += bn[j];
    if (mw0 + TM * 32 <= M && nw0 + TN * 32 <= N) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                float* dst = P + (size_t)(mw0 + i * 32 + 4 * fk) * N + (nw0 + j * 32 + fr);
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[(size_t)(8 * (v >> 2) + (v & 3)) * N] = acc[i][j][v];
            }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = nw0 + j * 32 + fr;
            if (n >= N) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int mb = mw0 + i * 32 + 4 * fk;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = mb + 8 * (v >> 2) + (v & 3);
                    if (m < M) P[(size_t)m * N + n] = acc[i][j][v];
                }
            }
        }
    }
}

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
    store_acc_tiles<TM, TN>(acc, bias, P, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, fr, fk);
}

// ---------------------------------------------------------------------------------------------------------
// bf16 operands, slabs brought from global memory straight into LDS (no register staging), double-buffered.
// A direct load writes the 16 bytes of lane i at LDS offset base + 16*i, so one wave instruction fills 16 rows
// of 64 bytes; rows are not padded.  Bank conflicts are avoided by permuting the four 16-byte chunks of a row:
// chunk kc of row r is kept at position kc ^ chunk_swizzle(r, 4), both when a lane picks the global chunk that
// belongs at its LDS position and when a fragment is read.  Needs K % 32 == 0; rows beyond M / N are clamped to the
// last valid row (their products are never stored).
// ---------------------------------------------------------------------------------------------------------
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    // s_waitcnt on gfx9: vmcnt = bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] left unconstrained
    static_assert(N >= 0 && N < 64, "six-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
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
        const int kc = (lane & 3) ^ chunk_swizzle(row, 4);
        int m = m0 + row;
        if (m > M - 1) m = M - 1;
        asrc[i] = X + (size_t)m * ldx + 8 * kc;
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
        const int row = (wave * BI + i) * 16 + (lane >> 2);
        const int kc = (lane & 3) ^ chunk_swizzle(row, 4);
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
        wait_vmcnt<0>();
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
                const int pos = (ks * 2 + fk) ^ chunk_swizzle(rr, 4);
                fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(As + (size_t)rr * ROWB + pos * 16));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int rr = (wn * TN + j) * 32 + fr;
                const int pos = (ks * 2 + fk) ^ chunk_swizzle(rr, 4);
                fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Bs + (size_t)rr * ROWB + pos * 16));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
    store_acc_tiles<TM, TN>(acc, bias, P, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, fr, fk);
}

// ---------------------------------------------------------------------------------------------------------
// Large-M bf16 variant: 256 x 256 tile, eight waves (2 x 4, wave tile 128 x 64), K slabs brought straight into
// LDS through a ring of 128 KB (one workgroup per compute unit): four 32-wide slabs, three in flight while one is
// consumed, or two 64-wide slabs whose rows are whole 128-byte lines (a 32-wide slab uses half of every line it
// touches, and the other half has left the 32 KB vector cache by the time the next slab asks for it).  Fragment reads are issued as explicit ds_read_b128 instructions: the compiler cannot see that an
// LDS read depends on a particular direct-to-LDS load and would otherwise wait for ALL outstanding loads before
// every read, which collapses the ring to depth one.  The dependency is kept by hand instead: a counted
// s_waitcnt on the vector-memory counter (slab kt has landed once only the loads of the younger slabs are
// outstanding), then the workgroup barrier, then the reads.
// Chunk kc of row r lives at position kc ^ chunk_swizzle(r, chunks per row) of its row (bank-conflict-free
// 16-byte reads).  Needs K % BK == 0.
// ---------------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ u32x4 lds_read_b128(unsigned addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}

template <int BK>  // K extent of a slab: 32 (four-deep ring) or 64 (two-deep ring of whole 128-byte lines)
__global__ __launch_bounds__(512) void proj_mfma_bf16_big_kernel(const uint16_t* __restrict__ X, int ldx,
                                                                 const uint16_t* __restrict__ W,
                                                                 const float* __restrict__ bias, float* __restrict__ P,
                                                                 int M, int N, int K, int gm, int gn, int npid)
{
    constexpr int BM = 256, BN = 256;
    constexpr int NWN = 4, NW = 8;                        // eight waves, 2 (m) x 4 (n)
    constexpr int TM = 4, TN = 2;                         // 32x32 tiles per wave: wave tile 128 x 64
    constexpr int ROWB = BK * 2;                          // bytes per LDS row
    constexpr int CH = ROWB / 16;                         // 16-byte chunks per row
    constexpr int KS = BK / 16;                           // k16 steps per slab
    constexpr int STAGE = (BM + BN) * ROWB;               // 32 or 64 KB
    constexpr int NST = 131072 / STAGE;                   // ring depth: 4 or 2
    constexpr int RPI = 1024 / ROWB;                      // rows covered by one direct-load instruction
    constexpr int LI = (BM + BN) / RPI / NW;              // direct-load instructions per wave and slab
    static_assert(BK == 32 || BK == 64, "slab extent");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // same value, known to be wave-uniform
    const int wm = wave / NWN, wn = wave % NWN;           // rows wm*128, cols wn*64
    const int fr = lane & 31, fk = lane >> 5;

    // byte offsets of this lane's fragments inside a stage for the first k16 step; step ks flips chunk bits:
    // chunk (2 ks + fk) ^ swizzle = ((fk ^ swizzle) ^ 2 ks), i.e. offset ^ (ks << 5)
    unsigned offa[TM], offb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rr = (wm * TM + i) * 32 + fr;
        offa[i] = (unsigned)(rr * ROWB + ((fk ^ chunk_swizzle(rr, CH)) * 16));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int rr = (wn * TN + j) * 32 + fr;
        offb[j] = (unsigned)(BM * ROWB + rr * ROWB + ((fk ^ chunk_swizzle(rr, CH)) * 16));
    }
    const int nslab = K / BK;
    // slab `target` has landed once only the loads of the (at most NST - 2) younger slabs can still be outstanding
    auto wait_slab = [&](int target) {
        const int y = (nslab - 1 - target) < (NST - 2) ? (nslab - 1 - target) : (NST - 2);
        if (NST == 4 && y == 2) wait_vmcnt<2 * LI>();
        else if (NST == 4 && y == 1) wait_vmcnt<LI>();
        else wait_vmcnt<0>();
    };

  // one workgroup per compute unit walks over its share of the tiles
  for (int pid = blockIdx.x; pid < npid; pid += gridDim.x) {
    int tile_m, tile_n;
    if (!tile_of_block(pid, gm, gn, tile_m, tile_n)) continue;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // every wave has finished reading the previous tile's last slab before the ring is refilled
    if (pid != (int)blockIdx.x) __builtin_amdgcn_s_barrier();

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // direct loads: instruction q of a slab covers LDS rows RPI*q .. RPI*q + RPI-1 of the combined [X rows | W rows];
    // the CH lanes of a row fetch its chunks in swizzled order, so a row's lanes read one contiguous piece of a line
    // (the whole 128-byte line when BK = 64).  A wave's 64 rows all belong to one operand: scalar base pointer
    // plus one 32-bit element offset per instruction.
    const bool wave_loads_x = wave_s * 64 < BM;
    const uint16_t* opnd = wave_loads_x ? X + (size_t)m0 * ldx : W + (size_t)n0 * K;
    const int opnd_ld = wave_loads_x ? ldx : K;
    const int last_row = wave_loads_x ? (M - 1 - m0) : (N - 1 - n0);   // rows past the matrix re-read its last row
    unsigned soff[LI];
#pragma unroll
    for (int i = 0; i < LI; ++i) {
        const int row = wave_s * 64 + i * RPI + lane / CH;   // 0..511: X rows then W rows
        const int kc = (lane % CH) ^ chunk_swizzle(row, CH);
        int r = wave_loads_x ? row : row - BM;
        if (r > last_row) r = last_row;
        soff[i] = (unsigned)(r * opnd_ld + 8 * kc);
    }
    auto issue_slab = [&](int kt) {
        unsigned char* st = smem + (size_t)(kt % NST) * STAGE + (size_t)wave_s * LI * 1024;
        const uint16_t* from = opnd + (size_t)kt * BK;
#pragma unroll
        for (int i = 0; i < LI; ++i)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(from + soff[i]),
                                             (void __attribute__((address_space(3)))*)(st + (size_t)i * 1024), 16, 0, 0);
    };
    // Two fragment register sets, software-pipelined inside the wave: the LDS reads of the next k16 step are in
    // flight while the eight MFMAs of the current one execute, and the slab hand-over (counted wait on the
    // direct loads, workgroup barrier, refill of the freed ring buffer) sits in front of a slab's last MFMA
    // group, so the matrix pipe still has work queued while the wave waits there.
    u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    auto read_set0 = [&](unsigned st, int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa0[i] = lds_read_b128(st + (offa[i] ^ (unsigned)(ks << 5)));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb0[j] = lds_read_b128(st + (offb[j] ^ (unsigned)(ks << 5)));
    };
    auto read_set1 = [&](unsigned st, int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa1[i] = lds_read_b128(st + (offa[i] ^ (unsigned)(ks << 5)));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb1[j] = lds_read_b128(st + (offb[j] ^ (unsigned)(ks << 5)));
    };
    auto mfma_set0 = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa0[i]),
                                                                   __builtin_bit_cast(bf16x8, fb0[j]), acc[i][j], 0, 0, 0);
    };
    auto mfma_set1 = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa1[i]),
                                                                   __builtin_bit_cast(bf16x8, fb1[j]), acc[i][j], 0, 0, 0);
    };

#pragma unroll
    for (int q = 0; q < NST - 1; ++q)
        if (q < nslab) issue_slab(q);
    wait_slab(0);
    // bare barrier: __syncthreads() carries a workgroup fence, for which the compiler drains every outstanding
    // direct-to-LDS load; the ordering needed here is exactly the counted wait above plus the barrier
    __builtin_amdgcn_s_barrier();
    if (NST - 1 < nslab) issue_slab(NST - 1);
    read_set0(lds0, 0);
    for (int kt = 0; kt < nslab; ++kt) {
        const unsigned st = lds0 + (unsigned)((kt % NST) * STAGE);
#pragma unroll
        for (int ks = 0; ks < KS - 1; ++ks) {
            // LDS returns in order: all but the six youngest reads done = the current set is complete.  The
            // fragments are operands of the wait so that no MFMA can move above it.
            if ((ks & 1) == 0) {
                read_set1(st, ks + 1);
                asm volatile("s_waitcnt lgkmcnt(6)"
                             : "+v"(fa0[0]), "+v"(fa0[1]), "+v"(fa0[2]), "+v"(fa0[3]), "+v"(fb0[0]), "+v"(fb0[1])
                             :
                             : "memory");
                mfma_set0();
            } else {
                read_set0(st, ks + 1);
                asm volatile("s_waitcnt lgkmcnt(6)"
                             : "+v"(fa1[0]), "+v"(fa1[1]), "+v"(fa1[2]), "+v"(fa1[3]), "+v"(fb1[0]), "+v"(fb1[1])
                             :
                             : "memory");
                mfma_set1();
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // last step of the slab (set 1): once its reads have returned this wave is done with slab kt, so after
        // the barrier below the slab's ring buffer may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(fa1[0]), "+v"(fa1[1]), "+v"(fa1[2]), "+v"(fa1[3]), "+v"(fb1[0]), "+v"(fb1[1])
                     :
                     : "memory");
        if (kt + 1 < nslab) {
            wait_slab(kt + 1);
            __builtin_amdgcn_s_barrier();
            if (kt + NST < nslab) issue_slab(kt + NST);  // into the buffer of slab kt
            read_set0(lds0 + (unsigned)(((kt + 1) % NST) * STAGE), 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_set1();
        __builtin_amdgcn_sched_barrier(0);
    }
    store_acc_tiles<TM, TN>(acc, bias, P, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, fr, fk);
  }
}

// ---------------------------------------------------------------------------------------------------------
// fp32 operands on the fp32 matrix instruction (32x32x2).  Requires K % 4 == 0 (16-byte chunks along k).
// Each lane reads four consecutive k of its fragment row at once and feeds them to four MFMAs; which k a lane
// contributes to which MFMA is the same for both operands, which is all a sum over k needs.
// BK: k extent of a slab.  Both tile sizes run with 32 (half the barriers and twice the prefetch distance of 16:
// 5-7 % faster on the 4800-row speech projections, 15 % on products of a few hundred rows).
// ---------------------------------------------------------------------------------------------------------
template <int TM, int TN, int BK>
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
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int CPR = BK / 4;                      // 16-byte chunks per slab row
    constexpr int LDR = BK + 4;                      // padded row length in floats (80 bytes)
    constexpr int ACH = (BM * CPR + 255) / 256;
    constexpr int BCH = (BN * CPR + 255) / 256;
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
            const int c = tid + 256 * i, row = c / CPR, kc = c % CPR;
            const int m = m0 + row, k = k0 + 4 * kc;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < BM && m < M && k < K) v = *reinterpret_cast<const float4*>(X + (size_t)m * ldx + k);
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i, row = c / CPR, kc = c % CPR;
            const int n = n0 + row, k = k0 + 4 * kc;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < BN && n < N && k < K) v = *reinterpret_cast<const float4*>(W + (size_t)n * K + k);
            rb[i] = v;
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i, row = c / CPR, kc = c % CPR;
            if (row < BM) *reinterpret_cast<float4*>(As + ((size_t)buf * BM + row) * LDR + 4 * kc) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i, row = c / CPR, kc = c % CPR;
            if (row < BN) *reinterpret_cast<float4*>(Bs + ((size_t)buf * BN + row) * LDR + 4 * kc) = rb[i];
        }
    };

    // Slab kt+1 is requested one slab ahead and written to the other LDS buffer between the two halves of slab kt's
    // MFMAs (nobody reads that buffer any more: its last readers passed the barrier that ended slab kt-1), so the
    // refill and the request for slab kt+2 sit in the shadow of the matrix instructions instead of behind them.
    auto mma_groups = [&](int buf, int kg0, int kg1) {
#pragma unroll
        for (int kg = kg0; kg < kg1; ++kg) {
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
    };
    const int nslab = (K + BK - 1) / BK;
    constexpr int KG = BK / 8;
    load_slab(0);
    store_slab(0);
    if (nslab > 1) load_slab(BK);
    __syncthreads();
    for (int kt = 0; kt < nslab; ++kt) {
        const int buf = kt & 1;
        mma_groups(buf, 0, KG / 2);
        if (kt + 1 < nslab) {
            store_slab(buf ^ 1);                                   // slab kt+1, requested during slab kt-1
            if (kt + 2 < nslab) load_slab((kt + 2) * BK);
        }
        mma_groups(buf, KG / 2, KG);
        __syncthreads();
    }
    store_acc_tiles<TM, TN>(acc, bias, P, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, fr, fk);
}

// ---------------------------------------------------------------------------------------------------------
// fp32, at most 64 rows of X (batch-1 sequences: M = T; small batches), W stored in fragment order.  The product is a
// stream over W (read once, N*K*4 bytes) with X resident in L2.  Read row-major with one lane per row of W, as the
// matrix instruction wants its operand, every load instruction touches 32 rows, 32 bytes of a 128-byte line each, and
// the stream ran at a fifth of the memory rate.  So the weights are stored once more at set-up in the order the 16x16x4
// matrix instruction takes them -- tile (16 rows of W, 16 k): 64 lanes x 16 bytes, lane l holding
// W[16 nb + l % 16][16 kb + 4 (l / 16) .. + 3] -- so that a wave's load of a tile is 1 KB of consecutive bytes, and
// the rows of X (which stay in L2) are read 64 contiguous bytes per row.  With 16-row tiles a sequence of 35 rows
// costs three tiles of matrix work instead of the two 32-row tiles' worth of four.  A workgroup owns NT tiles of W
// rows for all of X; its eight waves split K, keep PD blocks of 16 k in flight, and their partial tiles are summed
// through LDS in a fixed order.  Requires K % 4 == 0 and ldx % 4 == 0 (16-byte loads of X).
// ---------------------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int MT, int NT, int PD>
__global__ __launch_bounds__(512) void proj_mfma_f32_skinny_kernel(const float* __restrict__ X, int ldx,
                                                                     const float4* __restrict__ Wf,
                                                                     const float* __restrict__ bias, float* __restrict__ P,
                                                                     int M, int N, int K)
{
    constexpr int NW = 8;
    __shared__ float part[NW][MT * 16][NT * 16];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, lk = lane >> 4;
    const int KB = (K + 15) >> 4, NB = (N + 15) >> 4;
    const int nb0 = blockIdx.x * NT;
    const int per = (KB + NW - 1) / NW;
    const int kb_beg = wave * per, kb_end = (kb_beg + per) < KB ? (kb_beg + per) : KB;
    f32x4 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    const float* xrow[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        int mr = 16 * i + lr;
        if (mr > M - 1) mr = M - 1;   // rows beyond M are computed on a valid row and never stored
        xrow[i] = X + (size_t)mr * ldx;
    }
    const float4* wtile[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int nb = (nb0 + j < NB) ? (nb0 + j) : (NB - 1);   // a tile beyond N repeats the last one and is never stored
        wtile[j] = Wf + (size_t)nb * KB * 64 + lane;
    }
    if (kb_beg < kb_end) {
        // The loads carry no condition: a prefetch past the wave's share reads the share's last block again and is never
        // multiplied, and a lane past K reads the last four values of its row against the zero padding of W.  (With a
        // branch or a select on a load the compiler waits for it where the paths join or where the select sits, and the
        // blocks no longer overlap.)
        float4 fa[PD][MT], fb[PD][NT];
        auto load = [&](int p, int kb) {
            const int kbc = kb < kb_end ? kb : (kb_end - 1);
            int k = 16 * kbc + 4 * lk;
            k = k < K - 4 ? k : K - 4;
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[p][i] = *reinterpret_cast<const float4*>(xrow[i] + k);
#pragma unroll
            for (int j = 0; j < NT; ++j) fb[p][j] = wtile[j][(size_t)kbc * 64];
        };
        auto mma = [&](int p) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[p][i].x, fb[p][j].x, acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[p][i].y, fb[p][j].y, acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[p][i].z, fb[p][j].z, acc[i][j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[p][i].w, fb[p][j].w, acc[i][j], 0, 0, 0);
        };
#pragma unroll
        for (int p = 0; p < PD; ++p) load(p, kb_beg + p);
        int kb = kb_beg;
        for (; kb + PD <= kb_end; kb += PD) {
#pragma unroll
            for (int p = 0; p < PD; ++p) {
                __builtin_amdgcn_sched_barrier(0);
                mma(p);
                __builtin_amdgcn_sched_barrier(0);
                load(p, kb + p + PD);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        const int rest = kb_end - kb;              // < PD blocks are left, already requested
#pragma unroll
        for (int p = 0; p < PD - 1; ++p)
            if (p < rest) mma(p);
    }
    // lane l of an accumulator tile holds rows 4 (l / 16) .. + 3 of column l % 16
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[wave][16 * i + 4 * lk + v][16 * j + lr] = acc[i][j][v];
    __syncthreads();
    for (int e = tid; e < MT * 16 * NT * 16; e += 512) {
        const int m = e / (NT * 16), n = 16 * nb0 + e % (NT * 16);
        if (m < M && n < N) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += part[w][m][e % (NT * 16)];
            P[(size_t)m * N + n] = sum + bias[n];
        }
    }
}

template <int MT>
static hipError_t launch_skinny(const float* X, int ldx, const float* Wf, const float* bias, float* P, int M, int N, int K,
                                  hipStream_t s)
{
    const int NB = (N + 15) / 16, KB = (K + 15) / 16;
    // Two tiles of W rows per workgroup halve the reads of X; taken when that still gives five in eight compute units a
    // workgroup (measured: 4H = 5248 rows and more are faster that way, 4096 rows much slower).  Blocks in flight per
    // wave: four where a wave's share of K is long enough to fill such a pipeline, else two.
    const bool nt2 = (NB + 1) / 2 >= (device_num_cus() * 5) / 8;
    const bool deep = (KB + 7) / 8 >= 24;
    const dim3 grid(nt2 ? (NB + 1) / 2 : NB), block(512);
    const float4* W4 = (const float4*)Wf;
    if (nt2 && deep) hipLaunchKernelGGL((proj_mfma_f32_skinny_kernel<MT, 2, 4>), grid, block, 0, s, X, ldx, W4, bias, P, M, N, K);
    else if (nt2) hipLaunchKernelGGL((proj_mfma_f32_skinny_kernel<MT, 2, 2>), grid, block, 0, s, X, ldx, W4, bias, P, M, N, K);
    else if (deep) hipLaunchKernelGGL((proj_mfma_f32_skinny_kernel<MT, 1, 4>), grid, block, 0, s, X, ldx, W4, bias, P, M, N, K);
    else hipLaunchKernelGGL((proj_mfma_f32_skinny_kernel<MT, 1, 2>), grid, block, 0, s, X, ldx, W4, bias, P, M, N, K);
    return hipGetLastError();
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
    const size_t lds = 131072;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)proj_mfma_bf16_big_kernel<32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)proj_mfma_bf16_big_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int num_cus = (device_num_cus() / kXcds) * kXcds;
    if (num_cus == 0) num_cus = kXcds;
    const int blocks = grid < num_cus ? grid : num_cus;
    if (K % 64 == 0)
        hipLaunchKernelGGL(proj_mfma_bf16_big_kernel<64>, dim3(blocks), dim3(512), lds, s, X, ldx, W, bias, P, M, N, K, gm, gn, grid);
    else
        hipLaunchKernelGGL(proj_mfma_bf16_big_kernel<32>, dim3(blocks), dim3(512), lds, s, X, ldx, W, bias, P, M, N, K, gm, gn, grid);
    return hipGetLastError();
}

template <int TM, int TN, int BK = 16>
static hipError_t launch_f32(const float* X, int ldx, const float* W, const float* bias, float* P, const float* W1,
                             const float* bias1, float* P1, int M, int N, int K, hipStream_t s)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    const int gm = (M + BM - 1) / BM, gn = (N + BN - 1) / BN;
    const int grid = ((gm * gn + kXcds - 1) / kXcds) * kXcds;
    const size_t lds = 2 * (size_t)(BM + BN) * (BK + 4) * sizeof(float);
    if (lds > 64 * 1024) {
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute((const void*)proj_mfma_f32_kernel<TM, TN, BK>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
    }
    hipLaunchKernelGGL((proj_mfma_f32_kernel<TM, TN, BK>), dim3(grid, W1 ? 2 : 1), dim3(256), lds, s, X, ldx, W, bias, P, W1,
                       bias1, P1, M, N, K, gm, gn);
    return hipGetLastError();
}

// Tile choice of the fp32 kernel.  The product is bound by the matrix instruction, so its time is the work of the
// busiest compute unit: (tiles it receives) x (tile area).  128 x 128 tiles are the more efficient ones, but a grid of
// a few hundred leaves most compute units with one tile while some have two; 64 x 64 tiles spread evenly.  The
// smaller tile is taken when it shortens that estimate by more than a tenth.
static bool f32_small_tiles(int M, int N, int ndir)
{
    if (M <= 64) return true;
    const long cus = device_num_cus();
    const long big = (long)((M + 127) / 128) * ((N + 127) / 128) * ndir;
    const long small = (long)((M + 63) / 64) * ((N + 63) / 64) * ndir;
    const long t_big = ((big + cus - 1) / cus) * 4, t_small = (small + cus - 1) / cus;
    return t_small * 10 < t_big * 9;
}

// fp32, two directions of one layer (same X) in one launch
hipError_t launch_proj_mfma_f32_pair(const float* X, int ldx, const float* W0, const float* bias0, float* P0,
                                     const float* W1, const float* bias1, float* P1, int M, int N, int K, hipStream_t s)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    if (!proj_mfma_supported(false, K, ldx)) return hipErrorInvalidValue;
    if (f32_small_tiles(M, N, W1 ? 2 : 1)) return launch_f32<1, 1, 32>(X, ldx, W0, bias0, P0, W1, bias1, P1, M, N, K, s);
    return launch_f32<2, 2, 32>(X, ldx, W0, bias0, P0, W1, bias1, P1, M, N, K, s);
}

bool proj_mfma_supported(bool w_bf16, int K, int ldx)
{
    return w_bf16 ? (K % 8 == 0 && ldx % 8 == 0) : (K % 4 == 0 && ldx % 4 == 0);
}

hipError_t launch_proj_mfma(const void* X, bool x_bf16, int ldx, const void* W, bool w_bf16, const float* bias, float* P,
                            int M, int N, int K, hipStream_t s, const float* W_frag16)
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
    if (M <= 64 && K % 4 == 0 && ldx % 4 == 0 && W_frag16 != nullptr) {
        switch ((M + 15) / 16) {
            case 1: return launch_skinny<1>((const float*)X, ldx, W_frag16, bias, P, M, N, K, s);
            case 2: return launch_skinny<2>((const float*)X, ldx, W_frag16, bias, P, M, N, K, s);
            case 3: return launch_skinny<3>((const float*)X, ldx, W_frag16, bias, P, M, N, K, s);
            default: return launch_skinny<4>((const float*)X, ldx, W_frag16, bias, P, M, N, K, s);
        }
    }
    if (f32_small_tiles(M, N, 1)) return launch_f32<1, 1, 32>((const float*)X, ldx, (const float*)W, bias, P, nullptr, nullptr, nullptr, M, N, K, s);
    return launch_f32<2, 2, 32>((const float*)X, ldx, (const float*)W, bias, P, nullptr, nullptr, nullptr, M, N, K, s);
}

}  // namespace l355

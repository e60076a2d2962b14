// Measurement kernels that give the achievable peaks quoted next to the spec-sheet ones: a streaming copy, a
// matrix-instruction issue loop (bf16 32x32x16 and fp32 32x32x2, operands and accumulators in registers), and a
// device-wide barrier with no data (one tagged slot per workgroup).
#include "common.h"
#include "exchange.h"

namespace l355 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---- streaming copy: four 16-byte loads in flight per thread, stores marked non-temporal (they are not read again)
__global__ __launch_bounds__(256) void copy_stream_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const f32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                    c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
        __builtin_nontemporal_store(c, dst + i + 2 * stride);
        __builtin_nontemporal_store(d, dst + i + 3 * stride);
    }
    for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

hipError_t launch_copy_stream(void* dst, const void* src, size_t bytes, hipStream_t s)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t g = (n16 + 4 * 256 - 1) / (4 * 256);
    const size_t cap = (size_t)device_num_cus() * 8;     // eight workgroups per compute unit
    if (g > cap) g = cap;
    hipLaunchKernelGGL(copy_stream_kernel, dim3((unsigned)g), dim3(256), 0, s, (f32x4*)dst, (const f32x4*)src, n16);
    return hipGetLastError();
}

// ---- matrix-instruction issue loop -------------------------------------------------------------------------------
// Every wave keeps eight independent accumulator tiles and issues `reps` rounds of eight matrix instructions on
// operands it holds in registers: nothing but the matrix pipe (and the power it draws) limits it.  RANDOM = false:
// one constant operand pair (registers that never toggle: the highest clock the device holds under matrix load);
// RANDOM = true: eight A and four B fragments of random sign and mantissa, rotated every round, as a product of
// real data presents them (the device then settles at a lower clock).  The shader clock is read around the loop.
constexpr int kMfmaChains = 8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4y;

__device__ __forceinline__ unsigned lcg(unsigned& s) { s = s * 1664525u + 1013904223u; return s; }
// two bf16 values in (-2, 2) of magnitude >= 1/128: random sign and mantissa, exponents in a narrow range
__device__ __forceinline__ unsigned random_bf16_pair(unsigned& s, bool random)
{
    const unsigned hi = (random ? (lcg(s) & 0x807F0000u) : 0u) | 0x3C000000u;
    const unsigned lo = ((random ? (lcg(s) & 0x807F0000u) : 0u) | 0x3C000000u) >> 16;
    return hi | lo;
}

template <bool BF16, bool RANDOM>
__global__ __launch_bounds__(256) void mfma_issue_kernel(float* __restrict__ sink, int reps, long long* __restrict__ clocks)
{
    u32x4y a[8], b[4];
    unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j) a[i][j] = random_bf16_pair(s, RANDOM);
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) b[i][j] = random_bf16_pair(s, RANDOM);
    f32x16 acc[kMfmaChains];
    for (int c = 0; c < kMfmaChains; ++c)
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int r = 0; r < reps; ++r) {
#pragma unroll
        for (int c = 0; c < kMfmaChains; ++c) {
            const u32x4y& fa = a[RANDOM ? c : 0];
            const u32x4y& fb = b[RANDOM ? (c & 3) : 0];
            if (BF16)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa), __builtin_bit_cast(bf16x8, fb),
                                                                acc[c], 0, 0, 0);
            else   // fp32: the first register of each fragment, read as a float of small magnitude
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[0] & 0xBFFFFFFFu), __uint_as_float(fb[0] & 0xBFFFFFFFu),
                                                             acc[c], 0, 0, 0);
        }
        if (RANDOM) {   // rotate the B fragments: operands differ from round to round (four moves under 256 pipe cycles)
            const u32x4y t = b[0];
            b[0] = b[1]; b[1] = b[2]; b[2] = b[3]; b[3] = t;
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float t = 0.f;
    for (int c = 0; c < kMfmaChains; ++c)
        for (int i = 0; i < 16; ++i) t += acc[c][i];
    if (t == 123.456f) sink[blockIdx.x * blockDim.x + threadIdx.x] = t;
    if (threadIdx.x == 0) {
        clocks[2 * blockIdx.x] = c1 - c0;
        clocks[2 * blockIdx.x + 1] = w1 - w0;   // 100 MHz
    }
}

// two workgroups of four waves per compute unit: two waves per SIMD.  *flops receives the operations of one launch.
// clocks: 2 x blocks 64-bit counters (shader cycles, 100 MHz ticks) per workgroup.
int mfma_issue_blocks() { return device_num_cus() * 2; }
hipError_t launch_mfma_issue(bool bf16, bool random, float* sink, long long* clocks, int reps, double* flops, hipStream_t s)
{
    const int blocks = mfma_issue_blocks();
    if (bf16 && random) hipLaunchKernelGGL((mfma_issue_kernel<true, true>), dim3(blocks), dim3(256), 0, s, sink, reps, clocks);
    else if (bf16) hipLaunchKernelGGL((mfma_issue_kernel<true, false>), dim3(blocks), dim3(256), 0, s, sink, reps, clocks);
    else if (random) hipLaunchKernelGGL((mfma_issue_kernel<false, true>), dim3(blocks), dim3(256), 0, s, sink, reps, clocks);
    else hipLaunchKernelGGL((mfma_issue_kernel<false, false>), dim3(blocks), dim3(256), 0, s, sink, reps, clocks);
    const double per_instruction = 2.0 * 32 * 32 * (bf16 ? 16 : 2);
    if (flops) *flops = per_instruction * kMfmaChains * (double)reps * 4.0 * blocks;
    return hipGetLastError();
}
size_t mfma_issue_sink_floats() { return (size_t)mfma_issue_blocks() * 256; }

// ---- device-wide barrier with no data ------------------------------------------------------------------------------
// `steps` rounds in which every workgroup raises its own tagged slot and waits until it has seen the slots of all
// workgroups: the same tagged-slot protocol as the recurrence kernels, carrying nothing.  One slot per workgroup, two
// arrays alternating by round parity.
__global__ __launch_bounds__(1024) void barrier_only_kernel(u64* slots, unsigned tag_base, int groups, int steps,
                                                            int* timeout_flag, unsigned spin_limit, int poll_pace)
{
    __shared__ float seen[256];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    for (int s = 0; s < steps; ++s) {
        if (s > 0) {
            pace_poll(poll_pace);
            gather_tagged(slots + (size_t)(s & 1) * groups, groups, tag_base + (unsigned)s, seen, tid, nthreads,
                          timeout_flag, spin_limit);
        }
        __syncthreads();
        if (s + 1 < steps && tid == 0)
            __hip_atomic_store(slots + (size_t)((s + 1) & 1) * groups + blockIdx.x,
                               pack_slot(0.f, tag_base + (unsigned)s + 1u), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
}

hipError_t launch_barrier_only(u64* slots, unsigned tag_base, int groups, int waves, int steps, int* timeout_flag,
                               unsigned spin_limit, int poll_pace, int cooperative, hipStream_t s)
{
    if (groups < 1 || groups > 256 || groups > device_num_cus() || waves < 1 || waves > 16 || steps < 2)
        return hipErrorInvalidValue;
    void* args[] = {(void*)&slots, (void*)&tag_base, (void*)&groups, (void*)&steps, (void*)&timeout_flag, (void*)&spin_limit, (void*)&poll_pace};
    if (cooperative) return hipLaunchCooperativeKernel((const void*)barrier_only_kernel, dim3(groups), dim3(waves * 64), args, 0, s);
    return hipLaunchKernel((const void*)barrier_only_kernel, dim3(groups), dim3(waves * 64), args, 0, s);
}

}  // namespace l355

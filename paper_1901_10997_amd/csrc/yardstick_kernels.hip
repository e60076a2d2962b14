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
// Every wave keeps four independent accumulator tiles and issues `reps` rounds of four matrix instructions on
// operands it never reloads: nothing but the matrix pipe limits it.  The sink store keeps the loop alive.
constexpr int kMfmaChains = 4;

__global__ __launch_bounds__(256) void mfma_issue_bf16_kernel(float* __restrict__ sink, int reps)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
    }
    f32x16 acc[kMfmaChains];
    for (int c = 0; c < kMfmaChains; ++c)
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    for (int r = 0; r < reps; ++r) {
#pragma unroll
        for (int c = 0; c < kMfmaChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float t = 0.f;
    for (int c = 0; c < kMfmaChains; ++c)
        for (int i = 0; i < 16; ++i) t += acc[c][i];
    if (t == 123.456f) sink[blockIdx.x * blockDim.x + threadIdx.x] = t;
}

__global__ __launch_bounds__(256) void mfma_issue_f32_kernel(float* __restrict__ sink, int reps)
{
    const float a = 0.001f * (float)(threadIdx.x & 7), b = 0.002f * (float)((threadIdx.x * 3) & 7);
    f32x16 acc[kMfmaChains];
    for (int c = 0; c < kMfmaChains; ++c)
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    for (int r = 0; r < reps; ++r) {
#pragma unroll
        for (int c = 0; c < kMfmaChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float t = 0.f;
    for (int c = 0; c < kMfmaChains; ++c)
        for (int i = 0; i < 16; ++i) t += acc[c][i];
    if (t == 123.456f) sink[blockIdx.x * blockDim.x + threadIdx.x] = t;
}

// two workgroups of four waves per compute unit: two waves per SIMD.  *flops receives the operations of one launch.
hipError_t launch_mfma_issue(bool bf16, float* sink, int reps, double* flops, hipStream_t s)
{
    const int blocks = device_num_cus() * 2;
    if (bf16) hipLaunchKernelGGL(mfma_issue_bf16_kernel, dim3(blocks), dim3(256), 0, s, sink, reps);
    else hipLaunchKernelGGL(mfma_issue_f32_kernel, dim3(blocks), dim3(256), 0, s, sink, reps);
    const double per_instruction = 2.0 * 32 * 32 * (bf16 ? 16 : 2);
    if (flops) *flops = per_instruction * kMfmaChains * (double)reps * 4.0 * blocks;
    return hipGetLastError();
}
size_t mfma_issue_sink_floats() { return (size_t)device_num_cus() * 2 * 256; }

// ---- device-wide barrier with no data ------------------------------------------------------------------------------
// `steps` rounds in which every workgroup raises its own tagged slot and waits until it has seen the slots of all
// workgroups: the same tagged-slot protocol as the recurrence kernels, carrying nothing.  One slot per workgroup, two
// arrays alternating by round parity.
__global__ __launch_bounds__(1024) void barrier_only_kernel(u64* slots, unsigned tag_base, int groups, int steps,
                                                            int* timeout_flag, unsigned spin_limit)
{
    __shared__ float seen[256];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    for (int s = 0; s < steps; ++s) {
        if (s > 0) gather_tagged(slots + (size_t)(s & 1) * groups, groups, tag_base + (unsigned)s, seen, tid, nthreads,
                                 timeout_flag, spin_limit);
        __syncthreads();
        if (s + 1 < steps && tid == 0)
            __hip_atomic_store(slots + (size_t)((s + 1) & 1) * groups + blockIdx.x,
                               pack_slot(0.f, tag_base + (unsigned)s + 1u), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
}

hipError_t launch_barrier_only(u64* slots, unsigned tag_base, int groups, int waves, int steps, int* timeout_flag,
                               unsigned spin_limit, int cooperative, hipStream_t s)
{
    if (groups < 1 || groups > 256 || groups > device_num_cus() || waves < 1 || waves > 16 || steps < 2)
        return hipErrorInvalidValue;
    void* args[] = {(void*)&slots, (void*)&tag_base, (void*)&groups, (void*)&steps, (void*)&timeout_flag, (void*)&spin_limit};
    if (cooperative) return hipLaunchCooperativeKernel((const void*)barrier_only_kernel, dim3(groups), dim3(waves * 64), args, 0, s);
    return hipLaunchKernel((const void*)barrier_only_kernel, dim3(groups), dim3(waves * 64), args, 0, s);
}

}  // namespace l355

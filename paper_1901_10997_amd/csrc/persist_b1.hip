// Batch-1 recurrence with the time loop on the device (one launch per layer and direction).
//
// Per timestep (paper Section 4, cell equations): a = P[t] + W_h.h_{t-1}; f,i,o = sigmoid, g = tanh;
// c_t = f*c_{t-1} + i*g; h_t = o*tanh(c_t).
//
// Design: every wavefront owns one hidden unit j (packed rows 4j..4j+3) and keeps that slice of W_h in
// registers for the whole sequence, so after the first step no weight is read from memory again.
// The only cross-workgroup traffic is h_t itself.  It is exchanged through a small library-owned buffer of
// 64-bit slots (low word: h value, high word: a step tag).  A slot is written with ONE 8-byte store, so the
// tag and the value arrive together; consumers poll the slots they need until the tag equals the step
// they are waiting for.  There is no separate grid barrier: data arrival is the synchronisation.
// Two slot arrays alternate by step parity; a producer can only overwrite array p two steps later, after it
// has consumed every value of the step in between, which every other wave had to finish reading array p to
// produce -- so no slot is overwritten while still needed.
// Tags grow monotonically over the life of the handle (the host advances tag_base by T per launch), so
// leftovers from earlier launches never match.
//
// All waits are bounded: on expiry a device flag is raised, every wave stops waiting and the kernel drains.
#include "common.h"
#include "device_math.h"

namespace l355 {

__device__ __forceinline__ unsigned long long pack_slot(float v, unsigned tag)
{
    return ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v);
}

// Fetch h (tagged `want`) for elements tid, tid+nthreads, ... < H into dst[].  Up to four slots are polled
// together so their memory latencies overlap.
__device__ __forceinline__ void gather_tagged(const unsigned long long* slots, int H, unsigned want, float* dst,
                                              int tid, int nthreads, int* timeout_flag, unsigned spin_limit)
{
    for (int e0 = tid; e0 < H; e0 += 4 * nthreads) {
        unsigned long long v[4];
        unsigned spins = 0;
        bool ok;
        do {
            ok = true;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * nthreads;
                v[u] = (e < H) ? __hip_atomic_load(slots + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                               : ((unsigned long long)want << 32);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) ok = ok && ((unsigned)(v[u] >> 32) == want);
            if (!ok) {
                ++spins;
                if (spins > spin_limit) {
                    __hip_atomic_store(timeout_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                if ((spins & 63u) == 0 &&
                    __hip_atomic_load(timeout_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                    break;
            }
        } while (!ok);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * nthreads;
            if (e < H) dst[e] = __uint_as_float((unsigned)v[u]);
        }
    }
}

// Shared tail of a step: nonlinearities, state update, outputs, publication of h_t.
__device__ __forceinline__ void finish_step(const PersistB1Args& a, int j, int t, int s, bool active, int lane,
                                            const float r[4], const float4& p, float& c)
{
    const float f = sigmoidf_fast(r[0] + p.x);
    const float i = sigmoidf_fast(r[1] + p.y);
    const float o = sigmoidf_fast(r[2] + p.z);
    const float g = tanhf_fast(r[3] + p.w);
    c = f * c + i * g;
    const float h = o * tanhf_fast(c);
    if (active && lane == 0) {
        a.y[(size_t)t * a.y_ld + j] = h;
        if (s + 1 < a.T) {
            const float hx = a.round_h_bf16 ? round_bf16(h) : h;
            __hip_atomic_store(a.xchg + (size_t)((s + 1) & 1) * a.H + j, pack_slot(hx, a.tag_base + (unsigned)s + 1u),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            if (a.hT) a.hT[j] = h;
            if (a.cT) a.cT[j] = c;
        }
    }
}

// Stage h_{s-1} into LDS buffer `dst` (step 0: from h0 / zeros; later: from the tagged slots).
__device__ __forceinline__ void stage_h(const PersistB1Args& a, int s, float* dst, int tid, int nthreads)
{
    if (s == 0) {
        for (int e = tid; e < a.H; e += nthreads) {
            float v = a.h0 ? a.h0[e] : 0.f;
            if (a.round_h_bf16) v = round_bf16(v);
            dst[e] = v;
        }
    } else {
        gather_tagged(a.xchg + (size_t)(s & 1) * a.H, a.H, a.tag_base + (unsigned)s, dst, tid, nthreads,
                      a.timeout_flag, a.spin_limit);
    }
}

template <int KI, int MAXT>
__global__ __launch_bounds__(MAXT) void persist_b1_dense_kernel(PersistB1Args a, const void* __restrict__ Wh, int w_bf16)
{
    extern __shared__ float hs[];  // [2][KI*64]
    constexpr int HP = KI * 64;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = blockIdx.x * (nthreads >> 6) + wave;
    const bool active = j < a.H;

    float w[4][KI];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const int k = lane + 64 * i;
            float v = 0.f;
            if (active && k < a.H) {
                const size_t idx = (size_t)(4 * j + q) * a.H + k;
                v = w_bf16 ? bf16_bits_to_f32(((const uint16_t*)Wh)[idx]) : ((const float*)Wh)[idx];
            }
            w[q][i] = v;
        }
    for (int e = tid; e < 2 * HP; e += nthreads) hs[e] = 0.f;  // padding beyond H must be finite
    float c = (active && a.c0) ? a.c0[j] : 0.f;
    __syncthreads();

    for (int s = 0; s < a.T; ++s) {
        const int t = a.reverse ? (a.T - 1 - s) : s;
        float* hb = hs + (s & 1) * HP;
        float4 p = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active) p = *reinterpret_cast<const float4*>(a.P + (size_t)t * 4 * a.H + 4 * j);
        stage_h(a, s, hb, tid, nthreads);
        __syncthreads();
        float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const float hv = hb[lane + 64 * i];
            acc0 = fmaf(w[0][i], hv, acc0);
            acc1 = fmaf(w[1][i], hv, acc1);
            acc2 = fmaf(w[2][i], hv, acc2);
            acc3 = fmaf(w[3][i], hv, acc3);
        }
        float r[4];
        wave_sum4(acc0, acc1, acc2, acc3, r);
        finish_step(a, j, t, s, active, lane, r, p, c);
    }
}

template <int NZ>
__global__ __launch_bounds__(1024) void persist_b1_sparse_kernel(PersistB1Args a, const float* __restrict__ ell_val,
                                                                 const uint16_t* __restrict__ ell_col)
{
    extern __shared__ float hs[];  // [2][H]
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = blockIdx.x * (nthreads >> 6) + wave;
    const bool active = j < a.H;

    float wv[4][NZ];
    int wc[4][NZ];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < NZ; ++i) {
            float v = 0.f;
            int k = 0;
            if (active) {
                const size_t idx = ((size_t)(4 * j + q) * NZ + i) * 64 + lane;
                v = ell_val[idx];
                k = ell_col[idx];
            }
            wv[q][i] = v;
            wc[q][i] = k;
        }
    float c = (active && a.c0) ? a.c0[j] : 0.f;

    for (int s = 0; s < a.T; ++s) {
        const int t = a.reverse ? (a.T - 1 - s) : s;
        float* hb = hs + (size_t)(s & 1) * a.H;
        float4 p = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active) p = *reinterpret_cast<const float4*>(a.P + (size_t)t * 4 * a.H + 4 * j);
        stage_h(a, s, hb, tid, nthreads);
        __syncthreads();
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NZ; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = fmaf(wv[q][i], hb[wc[q][i]], acc[q]);
        float r[4];
        wave_sum4(acc[0], acc[1], acc[2], acc[3], r);
        finish_step(a, j, t, s, active, lane, r, p, c);
    }
}

// Exchange with no arithmetic: the yardstick for the per-step cost of the persistent kernels.
__global__ __launch_bounds__(1024) void exchange_only_kernel(unsigned long long* xchg, unsigned tag_base, int H,
                                                             int steps, int* timeout_flag, unsigned spin_limit)
{
    extern __shared__ float hs[];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63;
    const int j = blockIdx.x * (nthreads >> 6) + (tid >> 6);
    float acc = 0.f;
    for (int s = 0; s < steps; ++s) {
        float* hb = hs + (size_t)(s & 1) * H;
        if (s > 0)
            gather_tagged(xchg + (size_t)(s & 1) * H, H, tag_base + (unsigned)s, hb, tid, nthreads, timeout_flag,
                          spin_limit);
        __syncthreads();
        if (s > 0) acc += hb[j < H ? j : 0];
        if (j < H && lane == 0 && s + 1 < steps)
            __hip_atomic_store(xchg + (size_t)((s + 1) & 1) * H + j, pack_slot(acc * 1e-30f, tag_base + (unsigned)s + 1u),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------------------------------------ launchers
static int g_num_cu = 0;
static int num_cu()
{
    if (g_num_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            g_num_cu = prop.multiProcessorCount;
        if (g_num_cu <= 0) g_num_cu = 256;
    }
    return g_num_cu;
}

static int pick_waves(int H, int requested, int max_waves)
{
    int w = requested;
    if (w <= 0) {
        w = 4;
        while (w < max_waves && (H + w - 1) / w > num_cu()) w *= 2;
    }
    if (w > max_waves) w = max_waves;
    if (w < 1) w = 1;
    return w;
}

template <typename K>
static hipError_t coop_launch(K kernel, int blocks, int threads, size_t lds, void** args, hipStream_t s)
{
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, lds);
    if (e != hipSuccess) return e;
    if ((long long)per_cu * num_cu() < blocks) return hipErrorCooperativeLaunchTooLarge;
    return hipLaunchCooperativeKernel((const void*)kernel, dim3(blocks), dim3(threads), args, (unsigned)lds, s);
}

bool persist_b1_dense_supported(int H) { return H >= 1 && H <= 2048; }
bool persist_b1_sparse_supported(int H, int slots) { return H >= 1 && H <= 16384 && slots >= 1 && slots <= 8; }

template <int KI>
static hipError_t launch_dense_ki(PersistB1Args a, const void* Wh, int w_bf16, int wpg_req, hipStream_t s)
{
    constexpr int MAXT = (KI <= 16) ? 1024 : 512;
    const int wpg = pick_waves(a.H, wpg_req, MAXT / 64);
    const int blocks = (a.H + wpg - 1) / wpg;
    const size_t lds = 2 * (size_t)KI * 64 * sizeof(float);
    void* args[] = {(void*)&a, (void*)&Wh, (void*)&w_bf16};
    return coop_launch(persist_b1_dense_kernel<KI, MAXT>, blocks, wpg * 64, lds, args, s);
}

hipError_t launch_persist_b1_dense(const PersistB1Args& a, const void* Wh, bool w_bf16, int wpg, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    if (!persist_b1_dense_supported(a.H)) return hipErrorInvalidValue;
    const int KI = (a.H + 63) / 64;
    const int wb = w_bf16 ? 1 : 0;
    switch (KI) {
#define CASE_KI(n) \
    case n: return launch_dense_ki<n>(a, Wh, wb, wpg, s);
        CASE_KI(1) CASE_KI(2) CASE_KI(3) CASE_KI(4) CASE_KI(5) CASE_KI(6) CASE_KI(7) CASE_KI(8)
        CASE_KI(9) CASE_KI(10) CASE_KI(11) CASE_KI(12) CASE_KI(13) CASE_KI(14) CASE_KI(15) CASE_KI(16)
        CASE_KI(17) CASE_KI(18) CASE_KI(19) CASE_KI(20) CASE_KI(21) CASE_KI(22) CASE_KI(23) CASE_KI(24)
        CASE_KI(25) CASE_KI(26) CASE_KI(27) CASE_KI(28) CASE_KI(29) CASE_KI(30) CASE_KI(31) CASE_KI(32)
#undef CASE_KI
    }
    return hipErrorInvalidValue;
}

template <int NZ>
static hipError_t launch_sparse_nz(PersistB1Args a, const float* ev, const uint16_t* ec, int wpg_req, hipStream_t s)
{
    const int wpg = pick_waves(a.H, wpg_req, 16);
    const int blocks = (a.H + wpg - 1) / wpg;
    const size_t lds = 2 * (size_t)a.H * sizeof(float);
    void* args[] = {(void*)&a, (void*)&ev, (void*)&ec};
    return coop_launch(persist_b1_sparse_kernel<NZ>, blocks, wpg * 64, lds, args, s);
}

hipError_t launch_persist_b1_sparse(const PersistB1Args& a, const float* ell_val, const uint16_t* ell_col, int slots,
                                    int wpg, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    if (!persist_b1_sparse_supported(a.H, slots)) return hipErrorInvalidValue;
    if (2 * (size_t)a.H * sizeof(float) > 64 * 1024) return hipErrorInvalidValue;
    switch (slots) {
        case 1: return launch_sparse_nz<1>(a, ell_val, ell_col, wpg, s);
        case 2: return launch_sparse_nz<2>(a, ell_val, ell_col, wpg, s);
        case 3: return launch_sparse_nz<3>(a, ell_val, ell_col, wpg, s);
        case 4: return launch_sparse_nz<4>(a, ell_val, ell_col, wpg, s);
        case 5: return launch_sparse_nz<5>(a, ell_val, ell_col, wpg, s);
        case 6: return launch_sparse_nz<6>(a, ell_val, ell_col, wpg, s);
        case 7: return launch_sparse_nz<7>(a, ell_val, ell_col, wpg, s);
        case 8: return launch_sparse_nz<8>(a, ell_val, ell_col, wpg, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_exchange_only(unsigned long long* xchg, unsigned tag_base, int H, int waves, int steps,
                                int* timeout_flag, unsigned spin_limit, hipStream_t s)
{
    if (H <= 0 || steps <= 0) return hipSuccess;
    const int wpg = pick_waves(H, waves, 16);
    const int blocks = (H + wpg - 1) / wpg;
    const size_t lds = 2 * (size_t)H * sizeof(float);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    void* args[] = {(void*)&xchg, (void*)&tag_base, (void*)&H, (void*)&steps, (void*)&timeout_flag, (void*)&spin_limit};
    return coop_launch(exchange_only_kernel, blocks, wpg * 64, lds, args, s);
}

}  // namespace l355

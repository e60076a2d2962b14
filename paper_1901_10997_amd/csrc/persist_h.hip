// Batch-1 H-LSTM recurrence with the time loop on the device, row-compressed weights in registers
// (paper Section 4: cell equations with one hidden layer inside each gate; ReLU hidden activation).
//
// Per timestep, for the gates q in {f, i, o, g}:
//     u_q = relu( b1_q + W1x_q . x_t + W1h_q . h_{t-1} )      hidden layer of gate q, G units
//     a_q = b2_q + W2_q . u_q;   f,i,o = sigmoid, g = tanh;   c_t = f*c_{t-1} + i*g;   h_t = o*tanh(c_t)
//
// A step is two dependent products, and each needs a vector the whole device has produced (h_{t-1}: H values,
// u_t: 4G values), so a step costs two exchanges.  Wave w of the grid owns hidden-layer unit g = w (packed rows
// 4g..4g+3 of W1x and W1h: the unit's row in each of the four gates) in the first half of a step and output unit
// j = w (packed rows 4j..4j+3 of W2) in the second half; its slices of all three matrices stay in registers as
// 64-lane slices of (value, 16-bit column) pairs for the whole sequence, its cell state in a register.
// h travels through tagged 8-byte slots (low word: value, high word: step tag; one store publishes both, consumers
// poll until the tag matches, no fence and no separate barrier).  u has four times as many values and every
// workgroup needs all of them, which made its exchange a matter of volume (6000 slots: 48 KB per workgroup and step);
// but u >= 0 (ReLU), so its sign bit is free and carries the stamp instead: a 4-byte word per value, sign bit = parity
// of the number of steps the array has seen.  One bit is enough: a reader of step s has itself received every word
// of step s-1, so what it can find in a word is step s-1 (other parity: ask again) or step s.  The count runs on over
// the launches that use the array (u_epoch), so that what a launch finds from the one before has the other parity
// than its first step.  u is laid out gate-major ([q][G]), so row q of W2 gathers from one contiguous block of LDS
// with its stored column indices, and a workgroup publishes one contiguous run of words per gate.
// One array per vector is enough: u_{t+1} is published only after its producer has received every h_t, and
// each h_t was published only after its producer had finished reading u_t (and the same with the roles swapped).
// The input row x_{t+2} is requested at the top of step t, parked in LDS at the top of step t+1 (before the wait), and
// its products are accumulated after h_{t+1} has been published, off the critical path.
// All waits are bounded: on expiry a device flag is raised, every wave stops waiting and the kernel drains.
#include "common.h"
#include "device_math.h"
#include "exchange.h"

namespace l355 {

namespace {

constexpr int hl_maxt(int nz) { return nz <= 2 ? 1024 : nz <= 4 ? 768 : 512; }

// Fetch `npairs` pairs of stamped words into LDS (sign bits cleared): a pair is accepted when both sign bits equal
// `stamp`.  Each word was published by a store of its own, so each half of a pair is checked by its own bit.
// Bounded like the tagged polls.
template <int NF>
__device__ __forceinline__ void gather_stamped_pairs(const u64* src, int npairs, unsigned stamp, u64* dst, int tid,
                                                     int nthreads, int* timeout_flag, unsigned spin_limit)
{
    constexpr u64 kSigns = 0x8000000080000000ull;
    const u64 want = stamp ? kSigns : 0ull;
    for (int e0 = tid; e0 < npairs; e0 += NF * nthreads) {
        u64 v[NF];
        unsigned spins = 0;
        bool ok;
        do {
            ok = true;
#pragma unroll
            for (int u = 0; u < NF; ++u) {
                const int e = e0 + u * nthreads;
                v[u] = (e < npairs) ? __hip_atomic_load(src + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : want;
                ok = ok && ((v[u] & kSigns) == want);
            }
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
        for (int u = 0; u < NF; ++u) {
            const int e = e0 + u * nthreads;
            if (e < npairs) dst[e] = v[u] & ~kSigns;
        }
    }
}

}  // namespace

template <int NZ, int MAXT>
__global__ __launch_bounds__(MAXT) void persist_b1_hlstm_kernel(PersistHArgs a)
{
    extern __shared__ float lds[];  // hbuf[H (+1: ubuf is copied in 8-byte pairs)] | ubuf[4G] | xbuf[2][D] | pub[4 * waves]
    const int H = a.H, G = a.G, D = a.D;
    float* hbuf = lds;
    float* ubuf = hbuf + ((H + 1) & ~1);
    float* xbuf = ubuf + 4 * (size_t)G;
    float* pub = xbuf + 2 * (size_t)D;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    const int unit = blockIdx.x * nwaves + wave;    // hidden-layer unit g in stage 1, output unit j in stage 2
    const bool act1 = unit < G, act2 = unit < H;

    constexpr int NZP = (NZ + 1) / 2;
    float v1x[4][NZ], v1h[4][NZ], v2[4][NZ];
    unsigned c1x[4][NZP], c1h[4][NZP], c2[4][NZP];
    // Every load of a matrix is issued whatever the shape (idle waves and slices past the slot count read a valid element
    // and are zeroed afterwards), one matrix at a time: with a branch per element the loads went out one by one, each
    // waiting for the one before it.
    auto load_matrix = [&](const float* val, const uint16_t* col, int slots, int rows, bool act, float (&v)[4][NZ],
                           unsigned (&c)[4][NZP]) {
        const int un = act ? unit : rows - 1;
        float tv[4][NZ];
        unsigned tk[4][NZ];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < NZ; ++i) {
                const size_t idx = ((size_t)(4 * un + q) * slots + (i < slots ? i : slots - 1)) * 64 + lane;
                tv[q][i] = val[idx];
                tk[q][i] = col[idx];
            }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int i = 0; i < NZP; ++i) c[q][i] = 0u;
#pragma unroll
            for (int i = 0; i < NZ; ++i) {
                const bool live = act && i < slots;
                v[q][i] = live ? tv[q][i] : 0.f;
                c[q][i >> 1] |= (live ? tk[q][i] : 0u) << (16 * (i & 1));
            }
        }
    };
    load_matrix(a.ell_val_1x, a.ell_col_1x, a.slots_1x, G, act1, v1x, c1x);
    load_matrix(a.ell_val_1h, a.ell_col_1h, a.slots_1h, G, act1, v1h, c1h);
    load_matrix(a.ell_val_2, a.ell_col_2, a.slots_2, H, act2, v2, c2);
#define HCOL(arr, q, i) ((arr[q][(i) >> 1] >> (16 * ((i) & 1))) & 0xFFFFu)
    const int row = lane >> 4;                       // gate held by this lane after the reduction
    const float bias1 = act1 ? a.bias1[4 * unit + row] : 0.f;
    const float bias2 = act2 ? a.bias2[4 * unit + row] : 0.f;
    float c = (act2 && a.c0) ? a.c0[unit] : 0.f;

    constexpr int XPT = 2;  // x elements per thread held in registers
    float xr[XPT];
    auto request_x = [&](int s_) {
        const size_t xrow = (size_t)(a.reverse ? (a.T - 1 - s_) : s_) * a.x_ld;
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
            const int e = tid + u * nthreads;
            xr[u] = (e < D) ? a.x[xrow + e] : 0.f;
        }
    };
    auto park_x = [&](int s_) {
        const size_t xrow = (size_t)(a.reverse ? (a.T - 1 - s_) : s_) * a.x_ld;
        float* xb = xbuf + (size_t)(s_ & 1) * D;
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
            const int e = tid + u * nthreads;
            if (e < D) xb[e] = xr[u];
        }
        for (int e = tid + XPT * nthreads; e < D; e += nthreads) xb[e] = a.x[xrow + e];  // wider inputs: the rest
    };
    float xacc[4] = {0.f, 0.f, 0.f, 0.f};
    auto x_products = [&](int s_) {
        const float* xb = xbuf + (size_t)(s_ & 1) * D;
#pragma unroll
        for (int q = 0; q < 4; ++q) xacc[q] = 0.f;
#pragma unroll
        for (int i = 0; i < NZ; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) xacc[q] = fmaf(v1x[q][i], xb[HCOL(c1x, q, i)], xacc[q]);
    };
    request_x(0);
    park_x(0);
    __syncthreads();
    x_products(0);
    if (1 < a.T) request_x(1);

    for (int s = 0; s < a.T; ++s) {
        const int t = a.reverse ? (a.T - 1 - s) : s;
        const unsigned tag = a.tag_base + (unsigned)s + 1u;
        const unsigned stamp = (a.u_epoch + (unsigned)s + 1u) & 1u;
        const bool more_x = s + 1 < a.T;
        if (more_x) park_x(s + 1);                   // requested a whole step ago: nothing to wait for
        if (s + 2 < a.T) request_x(s + 2);           // in flight during this step
        // ---- stage 1: hidden layers from h_{t-1}
        if (s == 0) {
            for (int e = tid; e < H; e += nthreads) hbuf[e] = a.h0 ? a.h0[e] : 0.f;
        } else {
            gather_tagged(a.xchg_h, H, tag - 1u, hbuf, tid, nthreads, a.timeout_flag, a.spin_limit);
        }
        __syncthreads();
        {
            float acc[4] = {xacc[0], xacc[1], xacc[2], xacc[3]};
#pragma unroll
            for (int i = 0; i < NZ; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = fmaf(v1h[q][i], hbuf[HCOL(c1h, q, i)], acc[q]);
            const float pre = wave_sum4_rows(acc[0], acc[1], acc[2], acc[3]) + bias1;
            if ((lane & 15) == 0) pub[4 * wave + row] = pre > 0.f ? pre : 0.f;
        }
        __syncthreads();
        if (tid < 4 * nwaves) {
            // thread (q, w) publishes the hidden activation of gate q that wave w produced: one contiguous run of
            // slots per gate and workgroup
            const int q = tid / nwaves, w = tid - q * nwaves;
            const int g = blockIdx.x * nwaves + w;
            if (g < G)   // pub holds +0 or a positive value: the sign bit is the stamp's
                __hip_atomic_store(a.xchg_u + (size_t)q * G + g, __float_as_uint(pub[4 * w + q]) | (stamp << 31),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // ---- stage 2: gate outputs from u_t, cell update
        // (nothing of this wave's own stands between its publication and this poll, so the poll is paced: exchange.h.  The
        // poll of h at the top of the step comes after the outputs and the next step's input products and needs none.)
        pace_poll(a.poll_pace_u);
        gather_stamped_pairs<4>(reinterpret_cast<const u64*>(a.xchg_u), 2 * G, stamp, reinterpret_cast<u64*>(ubuf), tid,
                                nthreads, a.timeout_flag, a.spin_limit);
        __syncthreads();
        float h = 0.f;
        {
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < NZ; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = fmaf(v2[q][i], ubuf[q * G + HCOL(c2, q, i)], acc[q]);
            const float pre = wave_sum4_rows(acc[0], acc[1], acc[2], acc[3]) + bias2;
            h = lstm_cell_rows(pre, lane, c);
        }
        // pub is free again: every thread passed the barrier after the stage-1 publication read it
        if (lane == 0) pub[wave] = h;
        __syncthreads();
        if (tid < nwaves && more_x) {
            const int j = blockIdx.x * nwaves + tid;
            if (j < H)
                __hip_atomic_store(a.xchg_h + j, pack_slot(pub[tid], tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // outputs after the publication: nothing on the way of h_t
        if (lane == 0 && act2) {
            a.y[(size_t)t * a.y_ld + unit] = h;
            if (s + 1 == a.T) {
                if (a.hT) a.hT[unit] = h;
                if (a.cT) a.cT[unit] = c;
            }
        }
        if (more_x) x_products(s + 1);               // input side of step s+1, off the critical path
    }
#undef HCOL
}

bool persist_b1_hlstm_supported(int H, int G, int D, int slots_1x, int slots_1h, int slots_2)
{
    if (H < 1 || G < 1 || D < 1) return false;
    const int nz = std::max(slots_1x, std::max(slots_1h, slots_2));
    if (slots_1x < 1 || slots_1h < 1 || slots_2 < 1 || nz > 7) return false;
    const int waves = hl_maxt(nz) / 64;
    if (((size_t)H + 1 + 4 * (size_t)G + 2 * (size_t)D + 4 * waves) * sizeof(float) > 64 * 1024) return false;
    const int units = std::max(H, G);
    return (units + waves - 1) / waves <= device_num_cus();
}

template <int NZ>
static hipError_t launch_hl_nz(PersistHArgs a, bool coop, hipStream_t s)
{
    constexpr int MAXT = hl_maxt(NZ);
    const int waves = MAXT / 64;
    const int units = std::max(a.H, a.G);
    const int blocks = (units + waves - 1) / waves;
    if (blocks > device_num_cus()) return hipErrorCooperativeLaunchTooLarge;
    const size_t lds = ((size_t)a.H + 1 + 4 * (size_t)a.G + 2 * (size_t)a.D + 4 * waves) * sizeof(float);
    void* args[] = {(void*)&a};
    const void* kern = (const void*)persist_b1_hlstm_kernel<NZ, MAXT>;
    // every workgroup must be resident at the same time: at most one per compute unit
    if (coop) return hipLaunchCooperativeKernel(kern, dim3(blocks), dim3(MAXT), args, (unsigned)lds, s);
    return hipLaunchKernel(kern, dim3(blocks), dim3(MAXT), args, lds, s);
}

hipError_t launch_persist_b1_hlstm(const PersistHArgs& a, int cooperative, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    if (!persist_b1_hlstm_supported(a.H, a.G, a.D, a.slots_1x, a.slots_1h, a.slots_2)) return hipErrorInvalidValue;
    const int nz = std::max(a.slots_1x, std::max(a.slots_1h, a.slots_2));
    switch (nz) {
        case 1: return launch_hl_nz<1>(a, cooperative != 0, s);
        case 2: return launch_hl_nz<2>(a, cooperative != 0, s);
        case 3: return launch_hl_nz<3>(a, cooperative != 0, s);
        case 4: return launch_hl_nz<4>(a, cooperative != 0, s);
        case 5: return launch_hl_nz<5>(a, cooperative != 0, s);
        case 6: return launch_hl_nz<6>(a, cooperative != 0, s);
        case 7: return launch_hl_nz<7>(a, cooperative != 0, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace l355

// Batch-1 recurrence with the time loop on the device.
//
// Per timestep (paper Section 4, cell equations): a = b + W_x.x_t + W_h.h_{t-1}; f,i,o = sigmoid, g = tanh;
// c_t = f*c_{t-1} + i*g; h_t = o*tanh(c_t).
//
// Design: every wavefront owns one hidden unit j of one layer (packed rows 4j..4j+3) and keeps its slices of
// the weight matrices in registers for the whole sequence, so after the prologue no weight is read from
// memory again.  The only cross-workgroup traffic is h_t itself.  It is exchanged through a small
// library-owned buffer of 64-bit slots (low word: h value, high word: a step tag).  A slot is written with ONE
// 8-byte store, so tag and value arrive together; consumers poll the slots until the tag equals the step they
// wait for.  There is no separate grid barrier: data arrival is the synchronisation, which costs one memory
// round trip per step instead of two.  A workgroup collects the h values of its units in LDS and publishes
// them with one coalesced store.
// Two slot arrays per layer alternate by time parity.  h_t overwrites h_{t-2}; whoever publishes h_t has
// received every value of h_{t-1}, and each of those was published only after its workgroup had finished
// reading h_{t-2} -- so no slot is overwritten while still needed.
// Tags grow monotonically over the life of the handle (the host advances tag_base by T per launch), so
// leftovers of earlier launches never match.
//
// Where the input-side product W_x.x_t fits in registers too it is computed inside the same kernel, before
// the wait for h_{t-1} (x_t does not depend on the recurrence), which removes the separate projection launch.
// The row-compressed kernel can host two stacked layers in one launch: the waves of layer 1 consume h of
// layer 0 one step behind it (a diagonal wavefront over layers and time), which halves the number of
// sequential exchanges of a 2-layer stack.
//
// All waits are bounded: on expiry a device flag is raised, every wave stops waiting and the kernel drains.
#include "common.h"
#include "device_math.h"
#include "exchange.h"

namespace l355 {

__device__ __forceinline__ float uniform_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}

__device__ __forceinline__ void stage_initial(const float* h0, int H, float* dst, int tid, int nthreads, int round_bf)
{
    for (int e = tid; e < H; e += nthreads) {
        float v = h0 ? h0[e] : 0.f;
        if (round_bf) v = round_bf16(v);
        dst[e] = v;
    }
}

__device__ __forceinline__ float load_x(const void* x, int x_bf16, size_t idx)
{
    return x_bf16 ? bf16_bits_to_f32(((const uint16_t*)x)[idx]) : ((const float*)x)[idx];
}

// widest layer whose waves publish for themselves when the grid sits on one XCD (measured, 35 steps: H = 256 49.8 -> 46.7 us, 320 54.3 ->
// 49.6, 384 57.3 -> 57.0, 448 62.6 -> 68.1: beyond some 350 stores per step the one coalesced store per workgroup wins)
constexpr int kDenseDirectMaxH = 352;

// ------------------------------------------------------------------------------------------------------------
// Dense: W_h (and, when FUSEX, W_x) slices in registers.  One cell (layer, direction) per launch.
// ------------------------------------------------------------------------------------------------------------
template <int KI, bool FUSEX, int MAXT, bool DIRECT>
__global__ __launch_bounds__(MAXT) void persist_b1_dense_kernel(PersistB1Args a)
{
    extern __shared__ float lds[];  // hbuf[DIRECT ? 2 : 1][KI*64] | pub[16] | xbuf[2][KI*64] (fused only)
    constexpr int HP = KI * 64;
    constexpr int HB = DIRECT ? 2 : 1;
    float* hbuf = lds;
    float* pub = lds + HB * HP;
    float* xbuf = pub + 16;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, upb = nthreads >> 6;
    // Workgroups are dealt to the eight XCDs in turn.  A grid small enough for one XCD is launched eight times as
    // large and only the ids of residue 0 work, so that all of them can meet in one L2 (checked below).
    int bid = blockIdx.x;
    if (a.one_xcd) {
        if (blockIdx.x & 7) return;
        bid = blockIdx.x >> 3;
    }
    const int j = bid * upb + wave;
    const bool active = j < a.H;

    float wh[4][KI];
    float wx[FUSEX ? 4 : 1][FUSEX ? KI : 1];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const int k = lane + 64 * i;
            float v = 0.f;
            if (active && k < a.H) {
                const size_t idx = (size_t)(4 * j + q) * a.H + k;
                v = a.w_bf16 ? bf16_bits_to_f32(((const uint16_t*)a.Wh)[idx]) : ((const float*)a.Wh)[idx];
            }
            wh[q][i] = v;
            if (FUSEX) {
                float u = 0.f;
                if (active && k < a.D) {
                    const size_t idx = (size_t)(4 * j + q) * a.D + k;
                    u = a.w_bf16 ? bf16_bits_to_f32(((const uint16_t*)a.Wx)[idx]) : ((const float*)a.Wx)[idx];
                }
                wx[q][i] = u;
            }
        }
    const int row = lane >> 4;                       // gate handled by this lane after the reduction
    float bias_l = 0.f;                              // fused: bias of gate `row`
    if (FUSEX && active) bias_l = a.bias[4 * j + row];
    for (int e = tid; e < HB * HP; e += nthreads) hbuf[e] = 0.f;  // padding beyond H must stay finite
    float c = (active && a.c0) ? a.c0[j] : 0.f;
    __syncthreads();
    bool same_xcd = false;
    if (a.one_xcd)
        same_xcd = group_shares_xcd(a.xcc_ids, (int)(gridDim.x >> 3), bid, a.tag_base + 1u, hbuf, tid, nthreads,
                                    a.timeout_flag, a.spin_limit) && !a.device_scope_only;

    // Input side: x_t does not depend on the recurrence.  The workgroup requests row s+2 with coalesced loads at
    // the top of step s, parks it in LDS at the top of step s+1 (before the wait, so that nothing but h stands
    // between the arrival of h and the products), and each wave accumulates its products for step s+1 after h_s
    // has been published -- the time in which the wave would otherwise idle until that h has travelled.
    constexpr int XPT = (HP + MAXT - 1) / MAXT > 4 ? (HP + MAXT - 1) / MAXT : 4;
    float xr[FUSEX ? XPT : 1];
    float xa0 = 0.f, xa1 = 0.f, xa2 = 0.f, xa3 = 0.f;
    auto request_x = [&](int s_) {
        const size_t xrow = (size_t)(a.reverse ? (a.T - 1 - s_) : s_) * a.D;
        if (a.x_bf16) {
#pragma unroll
            for (int u = 0; u < XPT; ++u) {
                const int e = tid + u * nthreads;
                xr[FUSEX ? u : 0] = (e < a.D) ? bf16_bits_to_f32(((const uint16_t*)a.x)[xrow + e]) : 0.f;
            }
        } else {
#pragma unroll
            for (int u = 0; u < XPT; ++u) {
                const int e = tid + u * nthreads;
                xr[FUSEX ? u : 0] = (e < a.D) ? ((const float*)a.x)[xrow + e] : 0.f;
            }
        }
    };
    auto park_x = [&](int s_) {
        float* xb = xbuf + (s_ & 1) * HP;
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
            const int e = tid + u * nthreads;
            if (e < HP) xb[e] = a.round_x_bf16 ? round_bf16(xr[FUSEX ? u : 0]) : xr[FUSEX ? u : 0];
        }
    };
    auto x_products = [&](int s_) {
        const float* xb = xbuf + (s_ & 1) * HP;
        xa0 = xa1 = xa2 = xa3 = 0.f;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const float v = xb[lane + 64 * i];
            xa0 = fmaf(wx[FUSEX ? 0 : 0][FUSEX ? i : 0], v, xa0);
            xa1 = fmaf(wx[FUSEX ? 1 : 0][FUSEX ? i : 0], v, xa1);
            xa2 = fmaf(wx[FUSEX ? 2 : 0][FUSEX ? i : 0], v, xa2);
            xa3 = fmaf(wx[FUSEX ? 3 : 0][FUSEX ? i : 0], v, xa3);
        }
    };
    if (FUSEX) {
        request_x(0);
        park_x(0);
        __syncthreads();
        x_products(0);
        if (1 < a.T) request_x(1);
    }

    for (int s = 0; s < a.T; ++s) {
        const int t = a.reverse ? (a.T - 1 - s) : s;
        float pl = bias_l;
        const bool more_x = FUSEX && s + 1 < a.T;
        if (FUSEX) {
            if (more_x) park_x(s + 1);               // requested a whole step ago: nothing to wait for
            if (s + 2 < a.T) request_x(s + 2);       // in flight during this step
        } else if (active) {
            pl = a.P[(size_t)t * 4 * a.H + 4 * j + row];
        }
        // DIRECT: the copy of h alternates between two buffers, so that the barrier behind the poll is the only one a step
        // needs when every wave publishes for itself (below): a wave that runs ahead writes the other buffer, and cannot
        // get two steps ahead without the slowest wave passing a barrier in between.
        float* const hb = DIRECT ? hbuf + (s & 1) * HP : hbuf;
        if (s == 0)
            stage_initial(a.h0, a.H, hb, tid, nthreads, a.round_h_bf16);
        else
            gather_tagged(a.xchg + (size_t)(s & 1) * a.H, a.H, a.tag_base + (unsigned)s, hb, tid, nthreads,
                          a.timeout_flag, a.spin_limit);
        __syncthreads();
        float acc0 = xa0, acc1 = xa1, acc2 = xa2, acc3 = xa3;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const float hv = hb[lane + 64 * i];
            acc0 = fmaf(wh[0][i], hv, acc0);
            acc1 = fmaf(wh[1][i], hv, acc1);
            acc2 = fmaf(wh[2][i], hv, acc2);
            acc3 = fmaf(wh[3][i], hv, acc3);
        }
        const float pre = wave_sum4_rows(acc0, acc1, acc2, acc3) + pl;
        const float h = lstm_cell_rows(pre, lane, c);
        if constexpr (DIRECT) {
            // A narrow layer on one XCD: every wave stores its own slot (through to the shared L2) -- no hand-over through
            // LDS and no second barrier.  (On the whole device one coalesced store per workgroup is the faster form: 1.6-1.9
            // against 2.5-3.3 us per step on 256 compute units.)  The slot overwritten held h_{s-2}; every workgroup
            // finished reading that before any of its waves published h_{s-1}, all of which this workgroup has received.
            if (lane == 0 && active && s + 1 < a.T)
                exchange_store(a.xchg + (size_t)((s + 1) & 1) * a.H + j,
                               pack_slot(a.round_h_bf16 ? round_bf16(h) : h, a.tag_base + (unsigned)s + 1u), same_xcd);
        } else {
            if (lane == 0) pub[wave] = a.round_h_bf16 ? round_bf16(h) : h;
            __syncthreads();
            if (s + 1 < a.T && tid < upb) {
                const int ju = bid * upb + tid;
                if (ju < a.H)
                    exchange_store(a.xchg + (size_t)((s + 1) & 1) * a.H + ju, pack_slot(pub[tid], a.tag_base + (unsigned)s + 1u),
                                   same_xcd);
            }
        }
        // outputs after the publication: nothing on the way of h_t
        if (lane == 0 && active) {
            a.y[(size_t)t * a.y_ld + j] = h;
            if (s + 1 == a.T) {
                if (a.hT) a.hT[j] = h;
                if (a.cT) a.cT[j] = c;
            }
        }
        if (more_x) x_products(s + 1);               // for step s+1, off the critical path
    }
}

// ------------------------------------------------------------------------------------------------------------
// Dense, fused, grid on one XCD: every wave on its own.  A dense row multiplies h in the order it is stored, so
// the wave can poll the slots straight into the registers its products read (lane l: h[l + 64 i]), load its part
// of x_t the same way, and publish its h_t with one store from lane 0: no copy of h in LDS, no workgroup barrier
// (the step of the kernel above spends more time in its two barriers and the LDS round trips between them than in
// the hand-over through the L2).  Each wave polls all H slots itself, which only the L2 of one XCD serves fast
// enough, and only for small H (figures below); everything else keeps the kernel above.  The slot ring needs no barrier either: the wave
// that publishes h_t has received every value of h_{t-1}, and each of those was published by a wave that had
// received all of h_{t-2}.
// ------------------------------------------------------------------------------------------------------------
template <int KI>
__global__ __launch_bounds__(1024) void persist_b1_dense_wave_kernel(PersistB1Args a)
{
    __shared__ float tmp[64];
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, upb = nthreads >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (blockIdx.x & 7) return;                      // the ids of residue 0 are dealt to one XCD (checked below)
    const int bid = blockIdx.x >> 3;
    const int j = bid * upb + wave;
    const bool active = j < a.H;
    const int jj = active ? j : a.H - 1;

    float wh[4][KI], wx[4][KI];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const int k = lane + 64 * i;
            float v = 0.f, u = 0.f;
            if (k < a.H) {
                const size_t idx = (size_t)(4 * jj + q) * a.H + k;
                v = a.w_bf16 ? bf16_bits_to_f32(((const uint16_t*)a.Wh)[idx]) : ((const float*)a.Wh)[idx];
            }
            if (k < a.D) {
                const size_t idx = (size_t)(4 * jj + q) * a.D + k;
                u = a.w_bf16 ? bf16_bits_to_f32(((const uint16_t*)a.Wx)[idx]) : ((const float*)a.Wx)[idx];
            }
            wh[q][i] = v;
            wx[q][i] = u;
        }
    const int row = lane >> 4;                       // gate handled by this lane after the reduction
    const float bias_l = a.bias[4 * jj + row];
    float c = (active && a.c0) ? a.c0[j] : 0.f;
    const bool same_xcd = group_shares_xcd(a.xcc_ids, (int)(gridDim.x >> 3), bid, a.tag_base + 1u, tmp, tid, nthreads,
                                           a.timeout_flag, a.spin_limit) && !a.device_scope_only;
    if (!active) return;                             // (after the workgroup's barriers)

    // x_t in the lanes' registers; the row of the next step is requested once h_t is out
    float xr[KI];
    auto request_x = [&](int s_) {
        const size_t xrow = (size_t)(a.reverse ? (a.T - 1 - s_) : s_) * a.D;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const int k = lane + 64 * i;
            xr[i] = (k < a.D) ? load_x(a.x, a.x_bf16, xrow + k) : 0.f;
        }
    };
    float xa[4];
    auto x_products = [&]() {
#pragma unroll
        for (int q = 0; q < 4; ++q) xa[q] = 0.f;
#pragma unroll
        for (int i = 0; i < KI; ++i) {
            const float v = a.round_x_bf16 ? round_bf16(xr[i]) : xr[i];
#pragma unroll
            for (int q = 0; q < 4; ++q) xa[q] = fmaf(wx[q][i], v, xa[q]);
        }
    };
    request_x(0);
    x_products();
    if (1 < a.T) request_x(1);

    for (int s = 0; s < a.T; ++s) {
        const int t = a.reverse ? (a.T - 1 - s) : s;
        float hv[KI];
        if (s == 0) {
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int k = lane + 64 * i;
                float v = (a.h0 && k < a.H) ? a.h0[k] : 0.f;
                hv[i] = a.round_h_bf16 ? round_bf16(v) : v;
            }
        } else {
            const u64* slots = a.xchg + (size_t)(s & 1) * a.H;
            const unsigned want = a.tag_base + (unsigned)s;
            u64 v[KI];
            unsigned spins = 0;
            bool ok;
            do {
                ok = true;
#pragma unroll
                for (int i = 0; i < KI; ++i) {
                    const int k = lane + 64 * i;
                    v[i] = (k < a.H) ? __hip_atomic_load(slots + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ((u64)want << 32);
                    ok = ok && ((unsigned)(v[i] >> 32) == want);
                }
                if (!ok) {
                    ++spins;
                    if (spins > a.spin_limit) {
                        __hip_atomic_store(a.timeout_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    if ((spins & 63u) == 0 && __hip_atomic_load(a.timeout_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                        break;
                }
            } while (!ok);
#pragma unroll
            for (int i = 0; i < KI; ++i) hv[i] = (lane + 64 * i < a.H) ? __uint_as_float((unsigned)v[i]) : 0.f;
        }
        float acc[4] = {xa[0], xa[1], xa[2], xa[3]};
#pragma unroll
        for (int i = 0; i < KI; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = fmaf(wh[q][i], hv[i], acc[q]);
        const float pre = wave_sum4_rows(acc[0], acc[1], acc[2], acc[3]) + bias_l;
        const float h = lstm_cell_rows(pre, lane, c);
        if (lane == 0) {
            if (s + 1 < a.T)
                exchange_store(a.xchg + (size_t)((s + 1) & 1) * a.H + j,
                               pack_slot(a.round_h_bf16 ? round_bf16(h) : h, a.tag_base + (unsigned)s + 1u), same_xcd);
            // outputs after the publication: nothing on the way of h_t
            a.y[(size_t)t * a.y_ld + j] = h;
            if (s + 1 == a.T) {
                if (a.hT) a.hT[j] = h;
                if (a.cT) a.cT[j] = c;
            }
        }
        if (s + 1 < a.T) {
            x_products();                            // for step s+1, off the critical path
            if (s + 2 < a.T) request_x(s + 2);
        }
    }
}
// Every wave polls all H slots, so the polled volume grows with H squared and all of it hits the same few lines of
// the L2: measured against the kernel above (35 steps), H = 64: 37.7 against 45.8 us, 128: 43.6 against 47.2,
// 192: 50.0 against 47.8, 256: 57.1 against 50.0, 448: 102.6 against 63.2.  Used up to H = 128.
constexpr int kDenseWaveMaxKI = 2;

// ------------------------------------------------------------------------------------------------------------
// Row-compressed: (value, column) slices of W_x and W_h in registers; NL stacked layers per launch.
// Wave w of a workgroup serves layer w / upb, unit blockIdx*upb + w % upb.  Global step s advances layer l
// at time index s - l.
// ------------------------------------------------------------------------------------------------------------
template <int NZ, int NL, int MAXT>
__global__ __launch_bounds__(MAXT) void persist_b1_sparse_kernel(SparseStackArgs a)
{
    extern __shared__ float lds[];  // hbuf[NL][H] | xbuf[2][D0] | pub[waves]
    const int H = a.H;
    float* xbuf = lds + (size_t)NL * H;
    float* pub = xbuf + 2 * (size_t)a.D0;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    // the wave index as a scalar: everything derived from it (layer, unit, liveness) is then wave-uniform for the compiler
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = nthreads >> 6;
    const int upb = nwaves / NL;
    const int l = wave / upb;                       // layer served by this wave
    const int j = blockIdx.x * upb + (wave % upb);  // hidden unit
    const bool active = j < H;
    const SparseLayerArgs& L = a.layer[l];

    // values in fp32 registers; the 16-bit column indices two to a register (slot i in half i&1 of word i/2)
    constexpr int NZP = (NZ + 1) / 2;
    constexpr int XPT = 2;  // x elements per thread held in registers
    float xr[XPT];
    auto request_x = [&](int s_) {
        const size_t xrow = (size_t)(a.reverse ? (a.T - 1 - s_) : s_) * a.D0;
        if (a.x_bf16) {
#pragma unroll
            for (int u = 0; u < XPT; ++u) {
                const int e = tid + u * nthreads;
                xr[u] = (e < a.D0) ? bf16_bits_to_f32(((const uint16_t*)a.x)[xrow + e]) : 0.f;
            }
        } else {
#pragma unroll
            for (int u = 0; u < XPT; ++u) {
                const int e = tid + u * nthreads;
                xr[u] = (e < a.D0) ? ((const float*)a.x)[xrow + e] : 0.f;
            }
        }
    };
    request_x(0);   // first of everything: the row is in flight while the weights are fetched
    // copies of the layer's remaining fields, taken together with the ones below (one round trip for all of them)
    const int32_t* const opx = L.ovf_ptr_x;
    const int32_t* const oph = L.ovf_ptr_h;
    const uint32_t* const oenx = L.ovf_ent_x;
    const uint32_t* const oenh = L.ovf_ent_h;
    const float* const ovlx = L.ovf_val_x;
    const float* const ovlh = L.ovf_val_h;
    const float* const pbias = L.bias;
    const float* const pc0 = L.c0;
    const int jj = active ? j : H - 1;
    // first entry and count of this unit's overflow lists, requested ahead of the weights
    int obx = 0, obh = 0, nox = 0, noh = 0;
    if (opx) { obx = opx[jj]; nox = opx[jj + 1]; }
    if (oph) { obh = oph[jj]; noh = oph[jj + 1]; }
    float vx[4][NZ], vh[4][NZ];
    unsigned cxp[4][NZP], chp[4][NZP];
    {
        // The layer's fields are copied once (the layer is chosen by the wave index, so `L` lives in memory), and every
        // load is issued whatever the shape -- idle waves and slices past the slot count read a valid element and are
        // zeroed afterwards.  With a reload of the fields and a branch per element the loads went out one at a time,
        // each behind two dependent round trips.
        const float* const pvx = L.ell_val_x;
        const float* const pvh = L.ell_val_h;
        const uint16_t* const pcx = L.ell_col_x;
        const uint16_t* const pch = L.ell_col_h;
        const int sx = L.slots_x, sh = L.slots_h;
        float tu[4][NZ], tv[4][NZ];
        unsigned tku[4][NZ], tkv[4][NZ];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int i = 0; i < NZ; ++i) {
                const size_t ix = ((size_t)(4 * jj + q) * sx + (i < sx ? i : sx - 1)) * 64 + lane;
                const size_t ih = ((size_t)(4 * jj + q) * sh + (i < sh ? i : sh - 1)) * 64 + lane;
                tu[q][i] = pvx[ix];
                tku[q][i] = pcx[ix];
                tv[q][i] = pvh[ih];
                tkv[q][i] = pch[ih];
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int i = 0; i < NZP; ++i) cxp[q][i] = chp[q][i] = 0u;
#pragma unroll
            for (int i = 0; i < NZ; ++i) {
                const bool lx = active && i < sx, lh = active && i < sh;
                vx[q][i] = lx ? tu[q][i] : 0.f;
                vh[q][i] = lh ? tv[q][i] : 0.f;
                cxp[q][i >> 1] |= (lx ? tku[q][i] : 0u) << (16 * (i & 1));
                chp[q][i >> 1] |= (lh ? tkv[q][i] : 0u) << (16 * (i & 1));
            }
        }
    }
    // overflow entries of this unit's rows (rows longer than 64*slots; rare): lane e holds entry e
    unsigned oex = 0u, oeh = 0u;
    float ovx = 0.f, ovh = 0.f;
    nox = active ? nox - obx : 0;
    noh = active ? noh - obh : 0;
    if (lane < nox) { oex = oenx[obx + lane]; ovx = ovlx[obx + lane]; }
    if (lane < noh) { oeh = oenh[obh + lane]; ovh = ovlh[obh + lane]; }
    nox = __builtin_amdgcn_readfirstlane(nox);
    noh = __builtin_amdgcn_readfirstlane(noh);
    // lane e adds its overflow product to the partial sum of the gate its entry belongs to: the value is kept once per
    // gate (zero for the other three), so that a step needs neither a comparison nor a lane mask for it; lanes without
    // an entry hold value 0 and column 0.  The branch is wave-uniform (n is a scalar) and most waves skip it.
    float ovxq[4], ovhq[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        ovxq[g] = (oex >> 16) == (unsigned)g ? ovx : 0.f;
        ovhq[g] = (oeh >> 16) == (unsigned)g ? ovh : 0.f;
    }
    const unsigned ocx = oex & 0xFFFFu, och = oeh & 0xFFFFu;
    auto add_overflow = [&](float (&acc)[4], int n, unsigned col, const float (&valq)[4], const float* vec) {
        if (n > 0) {
            const float x = vec[col];
#pragma unroll
            for (int g = 0; g < 4; ++g) acc[g] = fmaf(valq[g], x, acc[g]);
        }
    };
#define COLX(q, i) ((cxp[q][(i) >> 1] >> (16 * ((i) & 1))) & 0xFFFFu)
#define COLH(q, i) ((chp[q][(i) >> 1] >> (16 * ((i) & 1))) & 0xFFFFu)
    const int row = lane >> 4;                       // gate handled by this lane after the reduction
    const float bias_l = active ? pbias[4 * j + row] : 0.f;
    float c = (active && pc0) ? pc0[j] : 0.f;
    const int total_steps = a.T + NL - 1;
    // The layer is chosen by the wave index, so the compiler addresses `L` through memory; taken inside the time loop
    // these fields cost a load and a wait on the critical path of every step.  Copies made once:
    float* const out_y = (active && L.y) ? L.y + j : nullptr;
    const size_t out_ld = (size_t)L.y_ld;
    float* const out_hT = (active && L.hT) ? L.hT + j : nullptr;
    float* const out_cT = (active && L.cT) ? L.cT + j : nullptr;

    // The input vector of the first layer comes from the external sequence and does not depend on the
    // recurrence.  The whole workgroup requests row s+2 with coalesced loads at the top of step s, parks it in LDS
    // at the top of step s+1 (before the wait, so that nothing but h stands between the arrival of h and the
    // products), and the first layer's waves gather their products for step s+1 after h_s has been published --
    // the time in which they would otherwise idle until that h has travelled.
    auto park_x = [&](int s_) {
        const size_t xrow = (size_t)(a.reverse ? (a.T - 1 - s_) : s_) * a.D0;
        float* xb = xbuf + (size_t)(s_ & 1) * a.D0;
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
            const int e = tid + u * nthreads;
            if (e < a.D0) xb[e] = a.round_x_bf16 ? round_bf16(xr[u]) : xr[u];
        }
        for (int e = tid + XPT * nthreads; e < a.D0; e += nthreads) {  // wider inputs: the rest, directly
            const float v = load_x(a.x, a.x_bf16, xrow + e);
            xb[e] = a.round_x_bf16 ? round_bf16(v) : v;
        }
    };
    float xacc[4] = {0.f, 0.f, 0.f, 0.f};
    auto x_products = [&](int s_) {
        const float* xb = xbuf + (size_t)(s_ & 1) * a.D0;
#pragma unroll
        for (int q = 0; q < 4; ++q) xacc[q] = 0.f;
        if (l == 0) {
#pragma unroll
            for (int i = 0; i < NZ; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) xacc[q] = fmaf(vx[q][i], xb[COLX(q, i)], xacc[q]);
            add_overflow(xacc, nox, ocx, ovxq, xb);
        }
    };
    park_x(0);
    __syncthreads();
    x_products(0);
    if (1 < a.T) request_x(1);

    for (int s = 0; s < total_steps; ++s) {
        const int ts = s - l;                        // time index this wave's layer works on
        const bool live = ts >= 0 && ts < a.T;
        const int t = a.reverse ? (a.T - 1 - ts) : ts;  // position in the sequence
        const bool more_x = s + 1 < a.T;
        if (more_x) park_x(s + 1);                   // requested a whole step ago: nothing to wait for
        if (s + 2 < a.T) request_x(s + 2);           // in flight during this step
        // stage, for every layer m, h^m at time index s-m-1 (the operand of layer m's recurrence at time s-m
        // and of layer m+1's input side at time s-m-1)
        PollSrc src[2] = {{nullptr, nullptr, 0u, 0}, {nullptr, nullptr, 0u, 0}};
#pragma unroll
        for (int m = 0; m < NL; ++m) {
            const int tm = s - m - 1;
            float* dst = lds + (size_t)m * H;
            if (tm == -1)
                stage_initial(a.layer[m].h0, H, dst, tid, nthreads, a.round_h_bf16);
            else if (tm >= 0 && tm < a.T - 1 + (m + 1 < NL ? 1 : 0))
                src[m] = PollSrc{a.xchg + ((size_t)m * 2 + ((tm + 1) & 1)) * H, dst, a.tag_base + (unsigned)tm + 1u, H};
        }
        gather_tagged2(src[0], src[1], tid, nthreads, a.timeout_flag, a.spin_limit);
        __syncthreads();
        float h = 0.f;
        if (live) {
            float acc[4] = {xacc[0], xacc[1], xacc[2], xacc[3]};
            const float* hrec = lds + (size_t)l * H;
            if (l > 0) {
                const float* hin = lds + (size_t)(l - 1) * H;
#pragma unroll
                for (int i = 0; i < NZ; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[q] = fmaf(vx[q][i], hin[COLX(q, i)], acc[q]);
                add_overflow(acc, nox, ocx, ovxq, hin);
            }
#pragma unroll
            for (int i = 0; i < NZ; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = fmaf(vh[q][i], hrec[COLH(q, i)], acc[q]);
            add_overflow(acc, noh, och, ovhq, hrec);
            const float pre = wave_sum4_rows(acc[0], acc[1], acc[2], acc[3]) + bias_l;
            h = lstm_cell_rows(pre, lane, c);
        }
        if (lane == 0) pub[wave] = a.round_h_bf16 ? round_bf16(h) : h;
        __syncthreads();
        if (tid < nwaves) {
            // thread `tid` publishes the value wave `tid` produced
            const int lm = tid / upb, ju = blockIdx.x * upb + (tid % upb);
            const int tsm = s - lm;
            // the last time index of the last layer has no consumer
            const bool wanted = tsm >= 0 && tsm < a.T && !(tsm == a.T - 1 && lm == NL - 1);
            if (wanted && ju < H)
                __hip_atomic_store(a.xchg + ((size_t)lm * 2 + ((tsm + 1) & 1)) * H + ju,
                                   pack_slot(pub[tid], a.tag_base + (unsigned)tsm + 1u), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        // outputs after the publication: nothing on the way of h_t
        if (live && lane == 0) {
            if (out_y) out_y[(size_t)t * out_ld] = h;
            if (ts + 1 == a.T) {
                if (out_hT) *out_hT = h;
                if (out_cT) *out_cT = c;
            }
        }
        if (more_x) x_products(s + 1);               // input side of step s+1, off the critical path
    }
}

#undef COLX
#undef COLH

// Exchange with no arithmetic: the yardstick for the per-step cost of the persistent kernels.
__global__ __launch_bounds__(1024) void exchange_only_kernel(u64* xchg, unsigned tag_base, int H, int steps,
                                                             int* timeout_flag, unsigned spin_limit, int poll_pace)
{
    extern __shared__ float lds[];  // hbuf[H] | pub[waves]
    float* pub = lds + H;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, upb = nthreads >> 6;
    const int j = blockIdx.x * upb + wave;
    float acc = 0.f;
    for (int s = 0; s < steps; ++s) {
        if (s > 0) {
            pace_poll(poll_pace);
            gather_tagged(xchg + (size_t)(s & 1) * H, H, tag_base + (unsigned)s, lds, tid, nthreads, timeout_flag,
                          spin_limit);
        }
        __syncthreads();
        if (s > 0) acc += lds[j < H ? j : 0];
        if (lane == 0) pub[wave] = acc * 1e-30f;
        __syncthreads();
        if (s + 1 < steps && tid < upb) {
            const int ju = blockIdx.x * upb + tid;
            if (ju < H)
                __hip_atomic_store(xchg + (size_t)((s + 1) & 1) * H + ju, pack_slot(pub[tid], tag_base + (unsigned)s + 1u),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ------------------------------------------------------------------------------------------------ launchers
// Every workgroup of these kernels must be resident at the same time.  A cooperative launch makes the runtime
// guarantee it; the ordinary launch relies on at most one workgroup per compute unit on an otherwise idle
// device (the waits inside the kernels are bounded either way).
template <typename K>
static hipError_t coop_launch(K kernel, int blocks, int threads, size_t lds, void** args, bool cooperative, hipStream_t s)
{
    if (blocks > device_num_cus()) return hipErrorCooperativeLaunchTooLarge;
    if (cooperative)
        return hipLaunchCooperativeKernel((const void*)kernel, dim3(blocks), dim3(threads), args, (unsigned)lds, s);
    return hipLaunchKernel((const void*)kernel, dim3(blocks), dim3(threads), args, lds, s);
}

// waves per workgroup: the largest allowed that still leaves at most one workgroup per compute unit
static int pick_waves(int H, int requested, int max_waves, int divisor)
{
    int w = requested > 0 ? requested : max_waves;
    if (w > max_waves) w = max_waves;
    w -= w % divisor;
    if (w < divisor) w = divisor;
    // never more workgroups than compute units: every workgroup must be resident for the exchange to progress
    while (w + divisor <= max_waves && (H + w / divisor - 1) / (w / divisor) > device_num_cus()) w += divisor;
    return w;
}

// threads per workgroup allowed by the register budget: the weight slices take (fused ? 8 : 4)*KI registers
// per lane, the rest of the kernel about 60; a compute unit gives 512 registers per lane and SIMD.
constexpr int dense_maxt(int KI, bool fusex)
{
    return fusex ? (8 * KI <= 56 ? 1024 : 8 * KI <= 88 ? 768 : 512) : (4 * KI <= 64 ? 1024 : 4 * KI <= 96 ? 768 : 512);
}
constexpr int kDenseFuseMaxKI = 20;
constexpr int sparse_maxt(int NZ) { return NZ <= 1 ? 1024 : NZ <= 4 ? 768 : 512; }

bool persist_b1_dense_supported(int H) { return H >= 1 && H <= 2048; }
bool persist_b1_dense_fusable(int H, int D)
{
    const int KI = (H + 63) / 64;
    return persist_b1_dense_supported(H) && D <= 64 * KI && KI <= kDenseFuseMaxKI;
}

template <int KI, bool FUSEX>
static hipError_t launch_dense_ki(PersistB1Args a, int wpg_req, bool coop, hipStream_t s)
{
    constexpr int MAXT = dense_maxt(KI, FUSEX);
    const int wpg = pick_waves(a.H, wpg_req, MAXT / 64, 1);
    int blocks = (a.H + wpg - 1) / wpg;
    // a grid that fits one XCD (an eighth of the compute units) is placed on one
    a.one_xcd = (a.xcc_ids != nullptr && blocks > 1 && blocks <= device_num_cus() / 8) ? 1 : 0;
    if (a.one_xcd) blocks *= 8;
    void* args[] = {(void*)&a};
    if constexpr (FUSEX && KI <= kDenseWaveMaxKI) {
        // on one XCD every wave works on its own (no LDS, no barriers); x and h must both fit the KI register slices
        if (a.one_xcd && a.D <= 64 * KI) return coop_launch(persist_b1_dense_wave_kernel<KI>, blocks, wpg * 64, 0, args, coop, s);
    }
    if constexpr (64 * (KI - 1) < kDenseDirectMaxH) {
        if (a.one_xcd && a.H <= kDenseDirectMaxH) {
            const size_t lds2 = ((size_t)KI * 64 * (FUSEX ? 4 : 2) + 16) * sizeof(float);
            return coop_launch(persist_b1_dense_kernel<KI, FUSEX, MAXT, true>, blocks, wpg * 64, lds2, args, coop, s);
        }
    }
    const size_t lds = ((size_t)KI * 64 * (FUSEX ? 3 : 1) + 16) * sizeof(float);
    return coop_launch(persist_b1_dense_kernel<KI, FUSEX, MAXT, false>, blocks, wpg * 64, lds, args, coop, s);
}

hipError_t launch_persist_b1_dense(const PersistB1Args& a, int wpg, int cooperative, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    if (!persist_b1_dense_supported(a.H)) return hipErrorInvalidValue;
    const int KI = (a.H + 63) / 64;
    const bool fuse = a.Wx != nullptr;
    if (fuse && !persist_b1_dense_fusable(a.H, a.D)) return hipErrorInvalidValue;
    switch (KI) {
#define CASE_KI(n)                                                     \
    case n:                                                            \
        if (n <= kDenseFuseMaxKI && fuse) return launch_dense_ki<(n <= kDenseFuseMaxKI ? n : 1), true>(a, wpg, cooperative != 0, s); \
        return launch_dense_ki<n, false>(a, wpg, cooperative != 0, s);
        CASE_KI(1) CASE_KI(2) CASE_KI(3) CASE_KI(4) CASE_KI(5) CASE_KI(6) CASE_KI(7) CASE_KI(8)
        CASE_KI(9) CASE_KI(10) CASE_KI(11) CASE_KI(12) CASE_KI(13) CASE_KI(14) CASE_KI(15) CASE_KI(16)
        CASE_KI(17) CASE_KI(18) CASE_KI(19) CASE_KI(20) CASE_KI(21) CASE_KI(22) CASE_KI(23) CASE_KI(24)
        CASE_KI(25) CASE_KI(26) CASE_KI(27) CASE_KI(28) CASE_KI(29) CASE_KI(30) CASE_KI(31) CASE_KI(32)
#undef CASE_KI
    }
    return hipErrorInvalidValue;
}

bool persist_b1_sparse_supported(int H, int D0, int slots_x, int slots_h, int nl)
{
    if (((size_t)nl * H + 2 * (size_t)D0 + 16) * sizeof(float) > 64 * 1024) return false;
    if (H < 1 || nl < 1 || nl > 2 || slots_x < 1 || slots_h < 1 || slots_x > 7 || slots_h > 7) return false;
    const int nz = slots_x > slots_h ? slots_x : slots_h;
    const int maxt = nz <= 1 ? 1024 : nz <= 4 ? 768 : 512;
    const int upb = (maxt / 64) / nl;
    return (H + upb - 1) / upb <= device_num_cus();
}

template <int NZ, int NL>
static hipError_t launch_sparse_nz(SparseStackArgs a, int wpg_req, bool coop, hipStream_t s)
{
    constexpr int MAXT = sparse_maxt(NZ);
    const int wpg = pick_waves(a.H, wpg_req, MAXT / 64, NL);
    const int upb = wpg / NL;
    const int blocks = (a.H + upb - 1) / upb;
    const size_t lds = ((size_t)NL * a.H + 2 * (size_t)a.D0 + wpg) * sizeof(float);
    void* args[] = {(void*)&a};
    return coop_launch(persist_b1_sparse_kernel<NZ, NL, MAXT>, blocks, wpg * 64, lds, args, coop, s);
}

hipError_t launch_persist_b1_sparse(const SparseStackArgs& a, int nl, int wpg, int cooperative, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    int nz = 1;
    for (int l = 0; l < nl; ++l) nz = std::max(nz, std::max(a.layer[l].slots_x, a.layer[l].slots_h));
    if (!persist_b1_sparse_supported(a.H, a.D0, nz, nz, nl)) return hipErrorInvalidValue;
#define CASE_NZ(n)                                               \
    case n:                                                      \
        return nl == 1 ? launch_sparse_nz<n, 1>(a, wpg, cooperative != 0, s) : launch_sparse_nz<n, 2>(a, wpg, cooperative != 0, s);
    switch (nz) {
        CASE_NZ(1) CASE_NZ(2) CASE_NZ(3) CASE_NZ(4) CASE_NZ(5) CASE_NZ(6) CASE_NZ(7)
    }
#undef CASE_NZ
    return hipErrorInvalidValue;
}

hipError_t launch_exchange_only(u64* xchg, unsigned tag_base, int H, int waves, int steps, int* timeout_flag,
                                unsigned spin_limit, int poll_pace, int cooperative, hipStream_t s)
{
    if (H <= 0 || steps <= 0) return hipSuccess;
    const int wpg = pick_waves(H, waves, 16, 1);
    const int blocks = (H + wpg - 1) / wpg;
    const size_t lds = ((size_t)H + wpg) * sizeof(float);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    void* args[] = {(void*)&xchg, (void*)&tag_base, (void*)&H, (void*)&steps, (void*)&timeout_flag, (void*)&spin_limit, (void*)&poll_pace};
    return coop_launch(exchange_only_kernel, blocks, wpg * 64, lds, args, cooperative != 0, s);
}

}  // namespace l355

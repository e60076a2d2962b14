// Small-batch row-compressed recurrence with the time loop on the device: one launch per layer, every
// direction of the layer in the same grid.
//
// Per timestep (paper Section 4, cell equations): a = P[t] + W_h.h_{t-1} (P = input projection with bias);
// f,i,o = sigmoid, g = tanh; c_t = f*c_{t-1} + i*g; h_t = o*tanh(c_t).
//
// The grid is a 2-D partition per direction: unit groups x batch groups.  A workgroup owns UPB hidden units
// and BW batch columns; it needs only the h values of its own batch columns (all H of them), which keeps the
// polled volume per workgroup at BW*H slots however large the batch is.  Each wave keeps the kept weights of
// its UPW units in registers in the quarter-wave form: slot s of a unit is one 64-lane gather that serves all
// four gate rows, gate q on lanes 16q..16q+15, so a lane accumulates BW sums per unit, a row's total is a butterfly
// inside its 16 lanes, and lane 16*gate + pair ends up with a gate total (pair = local unit * BW + column).  One
// exp2 and one reciprocal evaluate all gates of all pairs; c and h are updated in lanes 0..pairs-1.  h travels
// between workgroups through tagged 64-bit slots (value and step tag published by one store; consumers poll until
// the tag matches), laid out per direction as [parity][batch group][k][BW], the order of the LDS copy, so that the
// poll is a straight copy.  Only the workgroups of one (direction, batch group) exchange anything; where the groups
// fit they are placed on one XCD each and, once the launch has verified that from the hardware's XCD ids, publish h
// with workgroup-scope stores that stay in that XCD's L2 (exchange.h).  All waits are bounded.
#include <type_traits>
#include "common.h"
#include "device_math.h"
#include "exchange.h"

namespace l355 {

// S = slots per unit (16 kept entries of each gate per slot).  Configurations with registers to spare for the
// XCD-local hand-over:
constexpr bool persist_batched_q16_xcd_capable(int s, int upw) { return s * upw <= 84; }

template <int S, int UPW, int BW>
__global__ __launch_bounds__(512) void persist_batched_q16_kernel(PersistBatchedArgs a)
{
    extern __shared__ float lds[];  // hbuf[H][BW] (the BW batch values of one k adjacent) | pub[BW][UPB]
    constexpr int PAIRS = UPW * BW;
    static_assert(PAIRS <= 16, "pairs must fit one 16-lane row");
    static_assert(S % 2 == 0, "slots come in pairs (one per bank half)");
    const int H = a.H, B = a.B;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    const int upb = nwaves * UPW;
    float* hbuf = lds;
    float* pub = lds + (size_t)BW * H;
    constexpr bool kXcd = persist_batched_q16_xcd_capable(S, UPW);
    int dir, bgi, ugi;
    if (kXcd && a.xcd_local) {
        const int j = blockIdx.x >> 3;
        const int g = (blockIdx.x & 7) + 8 * (j / a.ug);
        if (g >= a.ndir * a.bg) return;     // padding ids take no part in the exchange
        ugi = j % a.ug; dir = g / a.bg; bgi = g % a.bg;
    } else {
        const int per_dir = a.ug * a.bg;
        dir = blockIdx.x / per_dir;
        const int rem = blockIdx.x % per_dir;
        bgi = rem / a.ug; ugi = rem % a.ug;
    }
    const PersistBatchedDir& D = a.d[dir];
    const int b0 = bgi * BW;
    const int bw = (B - b0) < BW ? (B - b0) : BW;         // columns actually present
    const int u0 = ugi * upb + wave * UPW;                // first unit of this wave
    // slots of this batch group: [parity][batch group][k][BW], i.e. in the order of the LDS copy of h
    u64* const xchg = a.xchg + (size_t)dir * 2 * (B + 3) * H + (size_t)bgi * H * BW;
    const size_t parity_stride = (size_t)a.bg * H * BW;

    // kept weights of this wave's units: values in fp32 registers, columns as 16-bit LDS byte offsets of their h
    // values, two to a register.  Every load is issued whatever the shape (clamped address, zeroed afterwards).
    float wv[UPW][S];
    unsigned wc[UPW][S / 2];
    {
        const int slots = D.q16_slots;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int unit = (u0 + u < H) ? (u0 + u) : (H - 1);
            float tv[S];
            unsigned tk[S];
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const int ii = i < slots ? i : slots - 1;
                const size_t idx = ((size_t)unit * slots + ii) * 64 + lane;
                tv[i] = D.q16_val[idx];
                tk[i] = D.q16_col[idx];
            }
#pragma unroll
            for (int i = 0; i < S / 2; ++i) wc[u][i] = 0u;
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const bool live = (u0 + u < H) && i < slots;
                wv[u][i] = live ? tv[i] : 0.f;
                wc[u][i >> 1] |= ((live ? tk[i] : 0u) * (BW * 4u)) << (16 * (i & 1));
            }
        }
    }
    // The few entries of rows longer than 16 S (at most 6 per wave; most waves have none):
    // lane e holds entry e of the wave's run of lists -- value, LDS byte offset of its column, and the lane that
    // collects its gate's total for batch column 0 (16 * gate + local unit * BW).
    float ovf_v = 0.f;
    unsigned ovf_off = 0u;
    int ovf_lane = 0, ovf_n = 0;
    if (D.q16_ovf_ptr != nullptr && u0 < H) {
        const int first = D.q16_ovf_ptr[u0];
        const int idx = first + lane;
        int pos = first;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int nxt = (u0 + u < H) ? D.q16_ovf_ptr[u0 + u + 1] : pos;
            if (idx >= pos && idx < nxt) {
                const unsigned e = D.q16_ovf_ent[idx];
                ovf_off = (e & 0xFFFFu) * (BW * 4u);
                ovf_lane = 16 * (int)(e >> 16) + u * BW;
                ovf_v = D.q16_ovf_val[idx];
            }
            pos = nxt;
        }
        ovf_n = pos - first;
        ovf_n = ovf_n < 64 ? ovf_n : 64;
    }
    ovf_n = __builtin_amdgcn_readfirstlane(ovf_n);
    // lane 16*gate + pair: pair = local unit * BW + column
    const int lp = lane & 15, row = lane >> 4;
    const int pu = lp / BW, pb = lp % BW;
    const bool pair_ok = lp < PAIRS && pb < bw && (u0 + pu) < H;
    const int unit_l = u0 + pu;
    float c = 0.f;
    if (lane < 16 && pair_ok && D.c0) c = D.c0[(size_t)(b0 + pb) * H + unit_l];

    // The direction is chosen by the block index, so `D` is addressed through memory: its fields are copied once
    // and the outputs are written after the publication.
    const float* const Pd_c = D.P;
    float* const y_c = D.y;
    const size_t y_ld_c = (size_t)D.y_ld;
    float* const hT_c = D.hT;
    float* const cT_c = D.cT;
    const float* const h0_c = D.h0;
    const int reverse = D.reverse;
    bool same_xcd = false;
    if (kXcd && a.xcd_local)
        same_xcd = group_shares_xcd(a.xcc_ids + ((size_t)dir * a.bg + bgi) * 64, a.ug, ugi, a.tag_base + 1u, hbuf, tid,
                                    nthreads, a.timeout_flag, a.spin_limit) && !a.device_scope_only;
    // P comes from memory (never from a cache: every element is read once), and a wave's loads return in order: a
    // load of P issued in front of the poll would hold back the poll's answer by a memory round trip in every step.
    // So the element for step s+1 is requested right after the poll of step s has been answered.
    auto load_p = [&](int s_) {
        const int t_ = reverse ? (a.T - 1 - s_) : s_;
        return (pair_ok && s_ < a.T) ? Pd_c[((size_t)t_ * a.Bld + b0 + pb) * (4 * (size_t)H) + 4 * unit_l + row] : 0.f;
    };
    float pin_next = load_p(0);
    for (int s = 0; s < a.T; ++s) {
        const int t = reverse ? (a.T - 1 - s) : s;
        if (s == 0) {
            for (int e = tid; e < BW * H; e += nthreads) {
                const int b = e / H, k = e - b * H;
                float v = (h0_c && b < bw) ? h0_c[(size_t)(b0 + b) * H + k] : 0.f;
                if (a.round_h_bf16) v = round_bf16(v);
                hbuf[k * BW + b] = v;
            }
        } else {
            pace_poll(a.poll_pace);   // device-wide exchange only (exchange.h); inside one XCD any wait costs what it lasts
            if (BW * H > 4 * nthreads && S * UPW <= 84)
                gather_tagged_cols<8, BW>(xchg + (size_t)(s & 1) * parity_stride, BW * H, bw, a.tag_base + (unsigned)s, hbuf, tid,
                                          nthreads, a.timeout_flag, a.spin_limit);
            else
                gather_tagged_cols<4, BW>(xchg + (size_t)(s & 1) * parity_stride, BW * H, bw, a.tag_base + (unsigned)s, hbuf, tid,
                                          nthreads, a.timeout_flag, a.spin_limit);
        }
        // (the value is taken over here, behind the poll's own wait, and not at the top of the loop, where waiting for
        // it would also wait for the acknowledgement of the stores just issued, in front of the poll)
        constexpr bool kTight = S * UPW >= 84 || (BW == 4 && S * UPW >= 72);   // near the register limit
        if constexpr (!kTight) asm volatile("" : "+v"(pin_next));   // (near the register limit the pin costs more than it saves)
        const float pin = pin_next;
        pin_next = load_p(s + 1);
        __syncthreads();
        if constexpr (kTight) {
            // near the register limit the offsets stay packed two to a register: the compiler must not unpack all
            // of them ahead of the time loop
#pragma unroll
            for (int u = 0; u < UPW; ++u)
#pragma unroll
                for (int i = 0; i < S / 2; ++i) asm volatile("" : "+v"(wc[u][i]));
        }
        float G = 0.f;
        {
            // The wave's UPW * S gathers as one software-pipelined sequence: PD reads are in flight ahead of the
            // multiply-adds that consume them, whatever unit they belong to.
            using VT = typename std::conditional<BW == 2, float2, float4>::type;
            constexpr int NS = UPW * S;
            constexpr int PDMAX = kTight ? 8 : 12;
            constexpr int PD = NS < PDMAX ? NS : PDMAX;
            auto read_slot = [&](int n) {
                const int u = n / S, i = n % S;
                const unsigned off = (wc[u][i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                return *reinterpret_cast<const VT*>(reinterpret_cast<const char*>(hbuf) + off);
            };
            VT ring[PD];
#pragma unroll
            for (int n = 0; n < PD; ++n) ring[n] = read_slot(n);
            float acc[2][BW];   // two chains per column
            float tot[16];      // per-lane partial sums of the wave's (unit, column) pairs, pair p = BW u + b
#pragma unroll
            for (int p = PAIRS; p < 16; ++p) tot[p] = 0.f;
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int u = n / S, i = n % S;
                if (i == 0) {
#pragma unroll
                    for (int b = 0; b < BW; ++b) acc[0][b] = acc[1][b] = 0.f;
                }
                const float w = wv[u][i];
                const VT x = ring[n % PD];
                acc[i & 1][0] = fmaf(w, x.x, acc[i & 1][0]);
                acc[i & 1][1] = fmaf(w, x.y, acc[i & 1][1]);
                if constexpr (BW == 4) {
                    acc[i & 1][2] = fmaf(w, x.z, acc[i & 1][2]);
                    acc[i & 1][3] = fmaf(w, x.w, acc[i & 1][3]);
                }
                if (n + PD < NS) ring[n % PD] = read_slot(n + PD);
                __builtin_amdgcn_sched_barrier(0);
                if (i == S - 1) {
#pragma unroll
                    for (int b = 0; b < BW; ++b) tot[u * BW + b] = acc[0][b] + acc[1][b];
                }
            }
            // all the sums over the 16 lanes of a row at once: lane p of row q ends up with gate q's total of pair p
            G = row16_transpose_sum(tot, lp);
        }
        if (ovf_n > 0) {   // wave-uniform; false in almost every wave
            // every lane multiplies its own entry (one gather for all of them); the products are then handed to the lanes
            // that collect their gates' totals, one entry at a time, without further memory accesses
            using VT = typename std::conditional<BW == 2, float2, float4>::type;
            const VT x = *reinterpret_cast<const VT*>(reinterpret_cast<const char*>(hbuf) + ovf_off);
            float pr[BW];
            pr[0] = ovf_v * x.x; pr[1] = ovf_v * x.y;
            if constexpr (BW == 4) { pr[2] = ovf_v * x.z; pr[3] = ovf_v * x.w; }
            for (int e = 0; e < ovf_n; ++e) {
                const int tgt = __builtin_amdgcn_readlane(ovf_lane, e);
#pragma unroll
                for (int b = 0; b < BW; ++b) {
                    const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr[b]), e));
                    G += (lane == tgt + b) ? v : 0.f;
                }
            }
        }
        G += pin;
        const bool cand = row == 3;
        const float sc = cand ? 2.8853900817779268f : -1.4426950408889634f;
        const float rr = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc * G));
        const float gate = cand ? fmaf(-2.0f, rr, 1.0f) : rr;
        const float gi = __shfl(gate, 16 + lp, 64), go = __shfl(gate, 32 + lp, 64), gg = __shfl(gate, 48 + lp, 64);
        float h_keep = 0.f;
        if (lane < 16) {
            c = fmaf(gate, c, gi * gg);
            const float h = go * tanhf_fast(c);
            if (lp < PAIRS) pub[(wave * UPW + pu) * BW + pb] = a.round_h_bf16 ? round_bf16(h) : h;
            h_keep = h;
        }
        __syncthreads();
        if (s + 1 < a.T) {
            u64* const out = xchg + (size_t)((s + 1) & 1) * parity_stride + (size_t)ugi * upb * BW;
            for (int e = tid; e < BW * upb; e += nthreads) {
                const int b = e & (BW - 1), unit = ugi * upb + e / BW;
                if (b < bw && unit < H)
                    exchange_store(out + e, pack_slot(pub[e], a.tag_base + (unsigned)s + 1u), kXcd && same_xcd);
            }
        }
        // outputs after the publication: nothing on the way of h_t
        if (lane < 16 && pair_ok) {
            y_c[((size_t)t * a.Bld + b0 + pb) * y_ld_c + unit_l] = h_keep;
            if (s + 1 == a.T) {
                const size_t ci = (size_t)(b0 + pb) * H + unit_l;
                if (hT_c) hT_c[ci] = h_keep;
                if (cT_c) cT_c[ci] = c;
            }
        }
    }
}

constexpr int kWaves = 8;

// ------------------------------------------------------------------------------------------------ planning
// Choose (UPW, BW): the most workgroups that still fit one per compute unit, within the register budget (1.5
// registers per unit and slot; 512-thread workgroups leave 256 registers per lane) and PAIRS <= 16.
constexpr int kQ16WeightRegs = 156;
bool persist_batched_q16_plan(int B, int H, int slots, int ndir, int* upw_out, int* bw_out, int* ug_out, int* bg_out)
{
    if (B < 2 || slots < 2 || slots > 24 || (slots & 1) || H < 1 || H > 4096) return false;
    // Two rounds.  The first takes the shape with the most workgroups.  The second prefers a shape whose batch groups fit
    // one XCD each (their exchange then stays in that XCD's L2, which is worth more than the extra workgroups: H = 512
    // at batch 20, 2.09 -> 1.80 us per step; two directions of 256 at batch 20, 1.94 -> 1.64), as long as a wave gets at
    // most twice the units (1500 wide at batch 2: six units per wave inside one XCD ran at 2.82 us against 2.41 with two
    // units per wave across the device).
    int best = -1, upw0 = 0;
    for (int round = 0; round < 2; ++round)
        for (int bw = 2; bw <= 4; bw *= 2) {
            for (int upw = 2; upw <= 8; ++upw) {
                if (upw * bw > 16 || 3 * slots * upw > 2 * kQ16WeightRegs) continue;
                if (((size_t)bw * H + (size_t)bw * kWaves * upw) * sizeof(float) > 64 * 1024) continue;
                const int ug = (H + kWaves * upw - 1) / (kWaves * upw), bg = (B + bw - 1) / bw;
                const int blocks = ug * bg * ndir;
                if (blocks > device_num_cus()) continue;
                const bool local = ((ndir * bg + 7) / 8) * ug <= device_num_cus() / 8;
                if (round == 1 && (!local || upw > 2 * upw0)) continue;
                const int score = blocks + (round == 1 ? 100000 : 0);
                if (score > best) {
                    best = score;
                    *upw_out = upw; *bw_out = bw; *ug_out = ug; *bg_out = bg;
                }
            }
            if (round == 0 && bw == 4) upw0 = best > 0 ? *upw_out : 0;
        }
    return best > 0;
}

template <int S, int UPW, int BW>
static hipError_t launch_q16_cfg(PersistBatchedArgs& a, int blocks, bool cooperative, hipStream_t s)
{
    const size_t lds = ((size_t)BW * a.H + (size_t)BW * kWaves * UPW) * sizeof(float);
    void* args[] = {(void*)&a};
    auto kern = persist_batched_q16_kernel<S, UPW, BW>;
    if (cooperative) return hipLaunchCooperativeKernel((const void*)kern, dim3(blocks), dim3(64 * kWaves), args, (unsigned)lds, s);
    return hipLaunchKernel((const void*)kern, dim3(blocks), dim3(64 * kWaves), args, lds, s);
}

template <int S>
static hipError_t launch_q16_s(PersistBatchedArgs& a, int upw, int bw, int blocks, bool coop, hipStream_t s)
{
#define CFG(U, W) if constexpr (3 * S * U <= 2 * kQ16WeightRegs) { if (upw == U && bw == W) return launch_q16_cfg<S, U, W>(a, blocks, coop, s); }
    CFG(2, 2) CFG(3, 2) CFG(4, 2) CFG(5, 2) CFG(6, 2) CFG(7, 2) CFG(8, 2) CFG(2, 4) CFG(3, 4) CFG(4, 4)
#undef CFG
    return hipErrorInvalidValue;
}

hipError_t launch_persist_batched_q16(PersistBatchedArgs& a, int ndir, int slots, int cooperative, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    int upw, bw, ug, bg;
    if (!persist_batched_q16_plan(a.B, a.H, slots, ndir, &upw, &bw, &ug, &bg)) return hipErrorInvalidValue;
    a.ug = ug;
    a.bg = bg;
    const int per_xcd = (ndir * bg + 7) / 8;
    a.ndir = ndir;
    a.xcd_local = (persist_batched_q16_xcd_capable(slots, upw) && ug <= 64 && per_xcd * ug <= device_num_cus() / 8) ? 1 : 0;
    const int blocks = a.xcd_local ? 8 * per_xcd * ug : ug * bg * ndir;
    if (a.xcd_local) a.poll_pace = 0;
    switch (slots) {
        case 2: return launch_q16_s<2>(a, upw, bw, blocks, cooperative != 0, s);
        case 4: return launch_q16_s<4>(a, upw, bw, blocks, cooperative != 0, s);
        case 6: return launch_q16_s<6>(a, upw, bw, blocks, cooperative != 0, s);
        case 8: return launch_q16_s<8>(a, upw, bw, blocks, cooperative != 0, s);
        case 10: return launch_q16_s<10>(a, upw, bw, blocks, cooperative != 0, s);
        case 12: return launch_q16_s<12>(a, upw, bw, blocks, cooperative != 0, s);
        case 14: return launch_q16_s<14>(a, upw, bw, blocks, cooperative != 0, s);
        case 16: return launch_q16_s<16>(a, upw, bw, blocks, cooperative != 0, s);
        case 18: return launch_q16_s<18>(a, upw, bw, blocks, cooperative != 0, s);
        case 20: return launch_q16_s<20>(a, upw, bw, blocks, cooperative != 0, s);
        case 22: return launch_q16_s<22>(a, upw, bw, blocks, cooperative != 0, s);
        case 24: return launch_q16_s<24>(a, upw, bw, blocks, cooperative != 0, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace l355

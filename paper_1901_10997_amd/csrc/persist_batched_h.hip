// Small-batch H-LSTM recurrence with the time loop on the device, row-compressed weights in registers: one launch
// per layer, every direction of the layer in the same grid (paper Section 4: cell equations with one hidden layer
// inside each gate; ReLU hidden activation).
//
// Per timestep, for the gates q in {f, i, o, g}:
//     u_q = relu( P1_q[t] + W1h_q . h_{t-1} )       P1 = b1 + W1x . x_t, computed for all t before the launch
//     a_q = b2_q + W2_q . u_q;   f,i,o = sigmoid, g = tanh;   c_t = f*c_{t-1} + i*g;   h_t = o*tanh(c_t)
//
// The grid is a 2-D partition per direction: unit groups x batch groups.  A workgroup owns UPB units (hidden-layer
// units g in the first half of a step, output units j in the second) and BW batch columns for the whole sequence;
// each wave keeps the kept weights of its UPW units of W1h and of W2 in registers in the quarter-wave form (slot s of a
// unit is one 64-lane gather that serves all four gate rows, gate q on lanes 16q..16q+15; value and 16-bit LDS offset)
// and the cell state of its (unit, column) pairs in lanes 0..15.  A product gathers from an LDS copy of the vector
// ([k][BW]: the BW batch values of one k adjacent, one 8- or 16-byte read per kept weight), a lane accumulates BW sums
// per unit, all (unit, column) sums of a wave are reduced together inside the 16-lane rows so that lane 16*gate + pair
// holds a gate total (pair = local unit * BW + column), and one exp2 and one reciprocal evaluate all gates of all pairs.
//
// A step needs two vectors the whole batch group has produced.  They travel differently:
//   h_t   (H values per column) through tagged 8-byte slots (value and step tag in one store; consumers poll until
//         the tag matches), laid out [k][BW] per batch group so that the poll is a straight copy into LDS;
//   u_t   (4G values per column, four times as many) as plain fp32 in the same [k][BW] layout (k = q*G + g), written
//         with device-scope write-through stores; when a workgroup's stores have been acknowledged it raises its
//         flag to the step tag.  A consumer's first wave polls the flags of its batch group; after a barrier the
//         workgroup copies the vector with device-scope 8-byte loads, all of a thread's loads in flight at once.
//         (An acquire fence followed by ordinary cached loads measured three times slower for these 50 KB.)
// One array per vector is enough: u_{t+1} is written only after its producer has received every h_t of the batch
// group, and each of those was published after its producer had finished reading u_t (and the same with the roles
// swapped).  Where the batch groups fit one XCD each and the launch has verified the placement from the hardware's
// XCD ids, h, u and the flags are stored at workgroup scope and meet in that XCD's L2 (exchange.h).
// All waits are bounded: on expiry a device flag is raised, every wave stops waiting, the kernel drains.
#include <type_traits>
#include "common.h"
#include "device_math.h"
#include "exchange.h"

namespace l355 {

namespace {
constexpr int kWaves = 8;
constexpr int kWeightRegs = 150;   // registers per lane for the weights of both matrices (3 per unit and slot)
constexpr int kMaxLds = 160 * 1024;
// hbuf (padded to whole 16-byte units) + ubuf
size_t lds_bytes(int H, int G, int bw) { return ((((size_t)bw * H + 3) & ~(size_t)3) + 4 * (size_t)G * bw) * sizeof(float); }
}  // namespace

template <int S, int UPW, int BW>   // S: slots per unit of the quarter-wave form (16 kept entries of each gate per slot)
__global__ __launch_bounds__(512) void persist_batched_hlstm_kernel(PersistBatchedHArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];  // hbuf[H][BW] | ubuf[4G][BW]
    constexpr int PAIRS = UPW * BW;
    static_assert(PAIRS <= 16 && S % 2 == 0, "pairs must fit one 16-lane row; slots come in pairs");
    const int H = a.H, G = a.G, B = a.B;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6;
    constexpr int upb = kWaves * UPW;
    float* hbuf = lds;
    float* ubuf = lds + (((size_t)BW * H + 3) & ~(size_t)3);   // 16-byte aligned for the row copy
    // block -> (direction, batch group, unit group).  Workgroups are dealt to the eight XCDs in turn; when the
    // groups fit, all workgroups of one (direction, batch group) -- the only ones that exchange data -- take ids of
    // one residue modulo 8 and so share an L2: a vector is then fetched from memory once per step instead of once per
    // XCD.  (Only speed depends on that dealing order.)
    int dir, bgi, ugi;
    if (a.xcd_local) {
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
    const PersistBatchedHDir& D = a.d[dir];
    const int b0 = bgi * BW;
    const int bw = (B - b0) < BW ? (B - b0) : BW;         // columns actually present
    const int u0 = ugi * upb + wave * UPW;                // first unit of this wave
    const size_t grp = (size_t)dir * a.bg + bgi;
    u64* xh = a.xchg_h + grp * a.h_stride;                // [H][BW] slots
    float* xu = a.xchg_u + grp * a.u_stride;              // [4G][BW]
    unsigned* flags = a.flags + grp * 64;                 // one per unit group

    // kept weights of this wave's units in the quarter-wave form (slot s of a unit is one 64-lane gather that serves
    // all four gate rows, gate q on lanes 16q..16q+15); the column is kept as the 16-bit LDS offset, in floats, of its BW
    // values (W2's columns are stored with their gate's offset q * G into the hidden-layer vector)
    float w1[UPW][S], w2[UPW][S];
    unsigned o1[UPW][S / 2], o2[UPW][S / 2];
    {
        // Every load is issued whatever the shape (units past the width and slots past a matrix's slot count read a
        // valid element and are zeroed afterwards): with a branch per element the loads went out one at a time.
        const int s1 = D.slots_1h, s2 = D.slots_2;
        float t1[S], t2[S];
        unsigned k1[S], k2[S];
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int g1 = (u0 + u < G) ? (u0 + u) : (G - 1), j2 = (u0 + u < H) ? (u0 + u) : (H - 1);
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const size_t i1 = ((size_t)g1 * s1 + (i < s1 ? i : s1 - 1)) * 64 + lane;
                const size_t i2 = ((size_t)j2 * s2 + (i < s2 ? i : s2 - 1)) * 64 + lane;
                t1[i] = D.q16_val_1h[i1];
                k1[i] = D.q16_col_1h[i1];
                t2[i] = D.q16_val_2[i2];
                k2[i] = D.q16_col_2[i2];
            }
#pragma unroll
            for (int i = 0; i < S / 2; ++i) o1[u][i] = o2[u][i] = 0u;
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const bool l1 = (u0 + u < G) && i < s1, l2 = (u0 + u < H) && i < s2;
                w1[u][i] = l1 ? t1[i] : 0.f;
                w2[u][i] = l2 ? t2[i] : 0.f;
                o1[u][i >> 1] |= ((l1 ? k1[i] : 0u) * (unsigned)BW) << (16 * (i & 1));   // h[k][0]
                o2[u][i >> 1] |= ((l2 ? k2[i] : 0u) * (unsigned)BW) << (16 * (i & 1));   // u[q*G + k][0]
            }
        }
    }
    // lane 16*gate + pair: pair = local unit * BW + column
    const int lp = lane & 15, row = lane >> 4;
    const int pu = lp / BW, pb = lp % BW;
    const int unit_l = u0 + pu;
    const bool in_pairs = lp < PAIRS;
    const bool ok1 = in_pairs && pb < bw && unit_l < G;
    const bool ok2 = in_pairs && pb < bw && unit_l < H;
    const float bias2 = (in_pairs && unit_l < H) ? D.bias2[4 * unit_l + row] : 0.f;
    float c = 0.f;
    if (lane < 16 && ok2 && D.c0) c = D.c0[(size_t)(b0 + pb) * H + unit_l];
    const int poll_i = lane < a.ug ? lane : a.ug - 1;

    // The few entries of rows longer than 16 S (at most 6 per wave; most waves have none): lane e holds entry e of the
    // wave's run of per-unit lists -- value, LDS byte offset of its column, and the lane that collects its gate's total
    // for batch column 0 (16 * gate + local unit * BW).
    struct Extra { float v; unsigned off; int lane0; int n; };
    auto load_extra = [&](const int32_t* ptr, const uint32_t* ent, const float* val, int units, int gate_stride) {
        Extra x{0.f, 0u, 0, 0};
        if (ptr != nullptr && u0 < units) {
            const int first = ptr[u0];
            const int idx = first + lane;
            int pos = first;
#pragma unroll
            for (int u = 0; u < UPW; ++u) {
                const int nxt = (u0 + u < units) ? ptr[u0 + u + 1] : pos;
                if (idx >= pos && idx < nxt) {
                    const unsigned e = ent[idx];
                    const unsigned g = e >> 16;
                    x.off = (g * (unsigned)gate_stride + (e & 0xFFFFu)) * (BW * 4u);
                    x.lane0 = 16 * (int)g + u * BW;
                    x.v = val[idx];
                }
                pos = nxt;
            }
            x.n = pos - first;
            x.n = x.n < 64 ? x.n : 64;
        }
        x.n = __builtin_amdgcn_readfirstlane(x.n);
        return x;
    };
    const Extra x1 = load_extra(D.ovf_ptr_1h, D.ovf_ent_1h, D.ovf_val_1h, G, 0);
    const Extra x2 = load_extra(D.ovf_ptr_2, D.ovf_ent_2, D.ovf_val_2, H, G);

    // One product: the wave's UPW * S gathers as one software-pipelined sequence (PD reads in flight ahead of the
    // multiply-adds that consume them), the UPW * BW sums reduced together by the transposing 16-lane reduction, so that
    // lane 16*gate + pair holds the gate's total of the pair; then the rare entries outside the slots.
    using VT = typename std::conditional<BW == 2, float2, float4>::type;
    auto products = [&](const float (&wv)[UPW][S], const unsigned (&wo)[UPW][S / 2], const Extra& xt, const float* vec) -> float {
        constexpr int NS = UPW * S;
        constexpr int PDMAX = (3 * S * UPW > 128) ? 8 : 12;
        constexpr int PD = NS < PDMAX ? NS : PDMAX;
        auto read_slot = [&](int n) {
            const int u = n / S, i = n % S;
            const unsigned off = (wo[u][i >> 1] >> (16 * (i & 1))) & 0xFFFFu;   // in floats: shift and add are one instruction
            return *reinterpret_cast<const VT*>(vec + off);
        };
        VT ring[PD];
#pragma unroll
        for (int n = 0; n < PD; ++n) ring[n] = read_slot(n);
        float acc[2][BW];
        float tot[16];
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
        float Gv = row16_transpose_sum(tot, lp);
        if (xt.n > 0) {   // wave-uniform; false in almost every wave
            const VT x = *reinterpret_cast<const VT*>(reinterpret_cast<const char*>(vec) + xt.off);
            float pr[BW];
            pr[0] = xt.v * x.x; pr[1] = xt.v * x.y;
            if constexpr (BW == 4) { pr[2] = xt.v * x.z; pr[3] = xt.v * x.w; }
            for (int e = 0; e < xt.n; ++e) {
                const int tgt = __builtin_amdgcn_readlane(xt.lane0, e);
#pragma unroll
                for (int b = 0; b < BW; ++b) {
                    const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr[b]), e));
                    Gv += (lane == tgt + b) ? v : 0.f;
                }
            }
        }
        return Gv;
    };

    // The direction is chosen by the block index, so `D` is addressed through memory: taken inside the time loop its
    // fields cost a load and a wait per step.  Where registers allow (kCopy) they are copied once.
    constexpr bool kCopy = S * UPW < 40;
    const float* P1_c = nullptr;
    float *y_c = nullptr, *hT_c = nullptr, *cT_c = nullptr;
    size_t y_ld_c = 0;
    if constexpr (kCopy) {
        P1_c = D.P1; y_c = D.y; y_ld_c = (size_t)D.y_ld; hT_c = D.hT; cT_c = D.cT;
    }
    // With the group's workgroups placed on one XCD (checked here, per launch, from the hardware's own id) the vectors
    // are handed over through that XCD's L2.
    bool same_xcd = false;
    if (a.xcd_local)
        same_xcd = group_shares_xcd(a.xcc_ids + grp * 64, a.ug, ugi, a.tag_base + 1u, hbuf, tid, nthreads, a.timeout_flag,
                                    a.spin_limit) && !a.device_scope_only;
    for (int s = 0; s < a.T; ++s) {
        const int t = D.reverse ? (a.T - 1 - s) : s;
        const unsigned tag = a.tag_base + (unsigned)s + 1u;
        // keep the packed offsets packed: without this the compiler unpacks all of them ahead of the loop, two
        // registers for every one saved
#pragma unroll
        for (int u = 0; u < UPW; ++u)
#pragma unroll
            for (int i = 0; i < S / 2; ++i) {
                asm volatile("" : "+v"(o1[u][i]));
                asm volatile("" : "+v"(o2[u][i]));
            }
        float pin = 0.f;
        if (ok1) pin = (kCopy ? P1_c : D.P1)[((size_t)t * a.Bld + b0 + pb) * (4 * (size_t)G) + 4 * unit_l + row];
        // ---- stage 1: hidden layers from h_{t-1}
        if (s == 0) {
            for (int e = tid; e < BW * H; e += nthreads) {
                const int k = e / BW, b = e - k * BW;
                hbuf[e] = (D.h0 && b < bw) ? D.h0[(size_t)(b0 + b) * H + k] : 0.f;
            }
        } else {
            gather_tagged_wide(xh, BW * H, tag - 1u, hbuf, tid, nthreads, a.timeout_flag, a.spin_limit);
        }
        __syncthreads();
        {
            const float pre = products(w1, o1, x1, hbuf) + pin;
            // dead columns of a ragged batch group are written as zeros: the consumers copy whole rows
            const float uval = (pb < bw && pre > 0.f) ? pre : 0.f;
            if (in_pairs && unit_l < G)
                exchange_store(xu + ((size_t)row * G + unit_l) * BW + pb, uval, same_xcd);
        }
        // stores acknowledged by every wave, then the workgroup's flag
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        if (tid == 0) exchange_store(flags + ugi, tag, same_xcd);
        // ---- stage 2: gate outputs from u_t, cell update
        if (wave == 0) {
            unsigned spins = 0;
            while (__hip_atomic_load(flags + poll_i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != tag) {
                if (++spins > a.spin_limit) {
                    __hip_atomic_store(a.timeout_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                if ((spins & 255u) == 0 && __hip_atomic_load(a.timeout_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                    break;
            }
        }
        __syncthreads();
        {
            // the flags say every producer's stores have reached memory: device-scope loads (which do not hit stale
            // lines of this compute unit's vector cache or this XCD's L2) fetch them, sixteen 8-byte loads per thread in
            // flight at once
            const u64* src = reinterpret_cast<const u64*>(xu);
            u64* dst = reinterpret_cast<u64*>(ubuf);
            const int nw = 2 * G * BW;   // 4G*BW floats, two to a load
            for (int e0 = tid; e0 < nw; e0 += 16 * nthreads) {
                u64 v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int e = e0 + u * nthreads;
                    v[u] = e < nw ? __hip_atomic_load(src + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int e = e0 + u * nthreads;
                    if (e < nw) dst[e] = v[u];
                }
            }
        }
        __syncthreads();
        {
            const float pre = products(w2, o2, x2, ubuf) + bias2;
            const bool cand = row == 3;
            const float sc = cand ? 2.8853900817779268f : -1.4426950408889634f;
            const float rr = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc * pre));
            const float gate = cand ? fmaf(-2.0f, rr, 1.0f) : rr;
            const float gi = __shfl(gate, 16 + lp, 64), go = __shfl(gate, 32 + lp, 64), gg = __shfl(gate, 48 + lp, 64);
            if (lane < 16) {
                c = fmaf(gate, c, gi * gg);
                const float h = go * tanhf_fast(c);
                if (in_pairs && unit_l < H && s + 1 < a.T)
                    exchange_store(xh + (size_t)unit_l * BW + pb, pack_slot(pb < bw ? h : 0.f, tag), same_xcd);
                if (ok2) {
                    (kCopy ? y_c : D.y)[((size_t)t * a.Bld + b0 + pb) * (kCopy ? y_ld_c : (size_t)D.y_ld) + unit_l] = h;
                    if (s + 1 == a.T) {
                        const size_t ci = (size_t)(b0 + pb) * H + unit_l;
                        float* const hT_out = kCopy ? hT_c : D.hT;
                        float* const cT_out = kCopy ? cT_c : D.cT;
                        if (hT_out) hT_out[ci] = h;
                        if (cT_out) cT_out[ci] = c;
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------ planning
// Choose (UPW, BW): batch groups that fit one XCD each first, then the most workgroups that still fit one per compute
// unit, within the register budget, with
// PAIRS <= 16, 16-bit LDS offsets, and at most 64 unit groups (one flag per polling lane).
bool persist_batched_h_plan(int B, int H, int G, int slots, int ndir, int* upw_out, int* bw_out, int* ug_out, int* bg_out)
{
    if (B < 2 || slots < 2 || slots > 24 || (slots & 1) || H < 1 || G < 1) return false;
    const int units = std::max(H, G);
    int best = -1;
    for (int bw = 2; bw <= 4; bw *= 2) {
        if ((size_t)H * bw > 65535 || (size_t)4 * G * bw > 65535) continue;      // 16-bit offsets, in floats
        if (lds_bytes(H, G, bw) > (size_t)kMaxLds) continue;
        for (int upw = 2; upw <= 4; ++upw) {
            if (upw * bw > 16 || 3 * slots * upw > kWeightRegs) continue;   // 1.5 registers per (unit, slot) and matrix
            const int ug = (units + kWaves * upw - 1) / (kWaves * upw), bg = (B + bw - 1) / bw;
            if (ug > 64) continue;
            const int blocks = ug * bg * ndir;
            if (blocks > device_num_cus()) continue;
            // a shape whose batch groups fit one XCD each goes first: both exchanges of a step then stay in that XCD's
            // L2 (800/800 at batch 2 to 8: 5.9-6.6 us per step with two units per wave across the device, 3.95 with four
            // inside one XCD; 1024/1024 at batch 20: 8.5 -> 5.8)
            const bool local = ((ndir * bg + 7) / 8) * ug <= device_num_cus() / 8;
            const int score = blocks + (local ? 100000 : 0);
            if (score > best) {
                best = score;
                *upw_out = upw; *bw_out = bw; *ug_out = ug; *bg_out = bg;
            }
        }
    }
    return best > 0;
}

// exchange storage per (direction, batch group), in elements of the respective array, padded to whole 256-byte blocks
size_t persist_batched_h_hstride(int H, int bw) { return (((size_t)H * bw * 8 + 255) / 256) * 256 / 8; }
size_t persist_batched_h_ustride(int G, int bw) { return (((size_t)4 * G * bw * 4 + 255) / 256) * 256 / 4; }

template <int S, int UPW, int BW>
static hipError_t launch_cfg(PersistBatchedHArgs& a, int blocks, bool cooperative, hipStream_t s)
{
    const size_t lds = lds_bytes(a.H, a.G, BW);
    auto kern = persist_batched_hlstm_kernel<S, UPW, BW>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    void* args[] = {(void*)&a};
    if (cooperative) return hipLaunchCooperativeKernel((const void*)kern, dim3(blocks), dim3(64 * kWaves), args, (unsigned)lds, s);
    return hipLaunchKernel((const void*)kern, dim3(blocks), dim3(64 * kWaves), args, lds, s);
}

template <int S>
static hipError_t launch_s(PersistBatchedHArgs& a, int upw, int bw, int blocks, bool coop, hipStream_t s)
{
#define CFG(U, W) if constexpr (3 * S * U <= kWeightRegs) { if (upw == U && bw == W) return launch_cfg<S, U, W>(a, blocks, coop, s); }
    CFG(2, 2) CFG(2, 4) CFG(3, 2) CFG(3, 4) CFG(4, 2) CFG(4, 4)
#undef CFG
    return hipErrorInvalidValue;
}

hipError_t launch_persist_batched_h(PersistBatchedHArgs& a, int ndir, int slots, int cooperative, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    int upw, bw, ug, bg;
    if (!persist_batched_h_plan(a.B, a.H, a.G, slots, ndir, &upw, &bw, &ug, &bg)) return hipErrorInvalidValue;
    a.ug = ug;
    a.bg = bg;
    a.h_stride = persist_batched_h_hstride(a.H, bw);
    a.u_stride = persist_batched_h_ustride(a.G, bw);
    // one XCD holds an eighth of the compute units; its share of the groups must fit there
    const int per_xcd = (ndir * bg + 7) / 8;
    a.ndir = ndir;
    a.xcd_local = per_xcd * ug <= device_num_cus() / 8;
    const int blocks = a.xcd_local ? 8 * per_xcd * ug : ug * bg * ndir;
    switch (slots) {
        case 2: return launch_s<2>(a, upw, bw, blocks, cooperative != 0, s);
        case 4: return launch_s<4>(a, upw, bw, blocks, cooperative != 0, s);
        case 6: return launch_s<6>(a, upw, bw, blocks, cooperative != 0, s);
        case 8: return launch_s<8>(a, upw, bw, blocks, cooperative != 0, s);
        case 10: return launch_s<10>(a, upw, bw, blocks, cooperative != 0, s);
        case 12: return launch_s<12>(a, upw, bw, blocks, cooperative != 0, s);
        case 14: return launch_s<14>(a, upw, bw, blocks, cooperative != 0, s);
        case 16: return launch_s<16>(a, upw, bw, blocks, cooperative != 0, s);
        case 18: return launch_s<18>(a, upw, bw, blocks, cooperative != 0, s);
        case 20: return launch_s<20>(a, upw, bw, blocks, cooperative != 0, s);
        case 22: return launch_s<22>(a, upw, bw, blocks, cooperative != 0, s);
        case 24: return launch_s<24>(a, upw, bw, blocks, cooperative != 0, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace l355

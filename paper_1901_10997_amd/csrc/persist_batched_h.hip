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
// each wave keeps the kept weights of its UPW units of W1h and of W2 in registers (64-lane slices of value and
// 16-bit LDS offset) and the cell state of its (unit, column) pairs in lanes 0..15.  A product gathers from an LDS
// copy of the vector ([k][BW]: the BW batch values of one k adjacent, one 8- or 16-byte read per kept weight), the
// 4 x BW partial sums of a unit are reduced with the lane-swap reduction so that lane 16*gate + pair holds a gate
// total (pair = local unit * BW + column), and one exp2 and one reciprocal evaluate all gates of all pairs.
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
constexpr int kWeightRegs = 150;   // registers per lane for the weights of both matrices (12*NZ per unit)
constexpr int kMaxLds = 160 * 1024;
// hbuf (padded to whole 16-byte units) + ubuf
size_t lds_bytes(int H, int G, int bw) { return ((((size_t)bw * H + 3) & ~(size_t)3) + 4 * (size_t)G * bw) * sizeof(float); }
}  // namespace

template <int NZ, int UPW, int BW>
__global__ __launch_bounds__(512) void persist_batched_hlstm_kernel(PersistBatchedHArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];  // hbuf[H][BW] | ubuf[4G][BW]
    constexpr int NZP = (4 * NZ + 1) / 2;   // packed 16-bit offsets of a unit's 4*NZ slices, two to a register
    constexpr int PAIRS = UPW * BW;
    static_assert(PAIRS <= 16, "pairs must fit one 16-lane row");
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

    // kept weights of this wave's units; the column is kept as the 16-bit LDS byte offset of its BW values
    float w1[UPW][4][NZ], w2[UPW][4][NZ];
    unsigned o1[UPW][NZP], o2[UPW][NZP];
    {
        // Every load is issued whatever the shape (units past the width and slices past a matrix's slot count read a
        // valid element and are zeroed afterwards): with a branch per element the loads went out one at a time, each
        // waiting for the one before it.
        const int s1 = D.slots_1h, s2 = D.slots_2;
        float t1[4 * NZ], t2[4 * NZ];
        unsigned k1[4 * NZ], k2[4 * NZ];
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int g1 = (u0 + u < G) ? (u0 + u) : (G - 1), j2 = (u0 + u < H) ? (u0 + u) : (H - 1);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int i = 0; i < NZ; ++i) {
                    const size_t i1 = ((size_t)(4 * g1 + q) * s1 + (i < s1 ? i : s1 - 1)) * 64 + lane;
                    const size_t i2 = ((size_t)(4 * j2 + q) * s2 + (i < s2 ? i : s2 - 1)) * 64 + lane;
                    t1[q * NZ + i] = D.ell_val_1h[i1];
                    k1[q * NZ + i] = D.ell_col_1h[i1];
                    t2[q * NZ + i] = D.ell_val_2[i2];
                    k2[q * NZ + i] = D.ell_col_2[i2];
                }
            }
#pragma unroll
            for (int i = 0; i < NZP; ++i) o1[u][i] = o2[u][i] = 0u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int i = 0; i < NZ; ++i) {
                    const bool l1 = (u0 + u < G) && i < s1, l2 = (u0 + u < H) && i < s2;
                    const int n = q * NZ + i;
                    w1[u][q][i] = l1 ? t1[n] : 0.f;
                    w2[u][q][i] = l2 ? t2[n] : 0.f;
                    o1[u][n >> 1] |= ((l1 ? k1[n] : 0u) * (BW * 4u)) << (16 * (n & 1));                       // h[k][0]
                    o2[u][n >> 1] |= (((unsigned)q * G + (l2 ? k2[n] : 0u)) * (BW * 4u)) << (16 * (n & 1));   // u[q*G + k][0]
                }
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

    // Overflow entries of this wave's units (rows longer than 64*slots; rare): the lists of consecutive units are
    // adjacent, lane e holds entry e of the wave's run, packed as LDS byte offset | gate << 16 | local unit << 18
    // (local unit 15: no entry).  The per-unit counts are wave-uniform.
    unsigned e1 = 15u << 18, e2 = 15u << 18;
    float ev1 = 0.f, ev2 = 0.f;
    int n1[UPW], n2[UPW];
    auto load_overflow = [&](const int32_t* ptr, const uint32_t* ent, const float* val, int units, bool gate_major,
                             unsigned& eo, float& evv, int (&cnt)[UPW]) {
#pragma unroll
        for (int u = 0; u < UPW; ++u) cnt[u] = 0;
        if (ptr == nullptr || u0 >= units) return;
        const int first = ptr[u0];
        int pos = first;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            const int nxt = (u0 + u < units) ? ptr[u0 + u + 1] : pos;
            cnt[u] = __builtin_amdgcn_readfirstlane(nxt - pos);
            const int idx = first + lane;
            if (idx >= pos && idx < nxt) {
                const unsigned e = ent[idx];
                const unsigned g = e >> 16, col = e & 0xFFFFu;
                eo = ((gate_major ? g * (unsigned)G + col : col) * (BW * 4u)) | (g << 16) | ((unsigned)u << 18);
                evv = val[idx];
            }
            pos = nxt;
        }
    };
    load_overflow(D.ovf_ptr_1h, D.ovf_ent_1h, D.ovf_val_1h, G, false, e1, ev1, n1);
    load_overflow(D.ovf_ptr_2, D.ovf_ent_2, D.ovf_val_2, H, true, e2, ev2, n2);

    // gathers of one stage: acc over the NZ slices of every unit, reduced into lane 16*gate + pair
    // The gathers are software-pipelined by hand in groups of GS (gates q0..q0+GS-1 of slice i of one unit): the next
    // group's reads are issued before the current group's multiply-adds, so that LDS latency overlaps arithmetic (left
    // to itself the compiler waits for every read on its own).  Two groups of read results are live at a time; the
    // configurations with the most weight registers take the smaller group.
    using VT = typename std::conditional<BW == 2, float2, float4>::type;
    constexpr int GS = (12 * NZ * UPW > 128 && BW == 4) ? 2 : 4;
    auto products = [&](const float (&wv)[UPW][4][NZ], const unsigned (&wo)[UPW][NZP], const int (&cnt)[UPW], unsigned eo,
                        float evv, const float* vec) -> float {
        constexpr int GPS = 4 / GS;            // groups per slice
        constexpr int NG = UPW * NZ * GPS;
        auto read_group = [&](int g, VT (&dst)[GS]) {
            const int u = g / (NZ * GPS), i = (g / GPS) % NZ, q0 = (g % GPS) * GS;
#pragma unroll
            for (int k = 0; k < GS; ++k) {
                const int n = (q0 + k) * NZ + i;
                const unsigned off = (wo[u][n >> 1] >> (16 * (n & 1))) & 0xFFFFu;
                dst[k] = *reinterpret_cast<const VT*>(reinterpret_cast<const char*>(vec) + off);
            }
        };
        float Gv = 0.f;
        VT hv[2][GS];
        float acc[4][BW];
        read_group(0, hv[0]);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int u = g / (NZ * GPS), i = (g / GPS) % NZ, q0 = (g % GPS) * GS;
            if (g + 1 < NG) read_group(g + 1, hv[(g + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            if (i == 0 && q0 == 0) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int b = 0; b < BW; ++b) acc[q][b] = 0.f;
            }
#pragma unroll
            for (int k = 0; k < GS; ++k) {
                const int q = q0 + k;
                const float w = wv[u][q][i];
                const VT& x = hv[g & 1][k];
                acc[q][0] = fmaf(w, x.x, acc[q][0]);
                acc[q][1] = fmaf(w, x.y, acc[q][1]);
                if constexpr (BW == 4) {
                    acc[q][2] = fmaf(w, x.z, acc[q][2]);
                    acc[q][3] = fmaf(w, x.w, acc[q][3]);
                }
            }
            if (i == NZ - 1 && q0 + GS == 4) {
                if (cnt[u] > 0) {
                    // this unit's overflow entries, one per lane, into the partial sum of the gate each belongs to
                    const float v = ((eo >> 18) & 15u) == (unsigned)u ? evv : 0.f;
                    const unsigned gq = (eo >> 16) & 3u;
                    const VT t = *reinterpret_cast<const VT*>(reinterpret_cast<const char*>(vec) + (eo & 0xFFFFu));
                    float xv[BW];
                    xv[0] = t.x; xv[1] = t.y;
                    if constexpr (BW == 4) { xv[2] = t.z; xv[3] = t.w; }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float vq = (gq == (unsigned)q) ? v : 0.f;
#pragma unroll
                        for (int b = 0; b < BW; ++b) acc[q][b] = fmaf(vq, xv[b], acc[q][b]);
                    }
                }
#pragma unroll
                for (int b = 0; b < BW; ++b) {
                    const float r = wave_sum4_rows(acc[0][b], acc[1][b], acc[2][b], acc[3][b]);
                    Gv = (lp == u * BW + b) ? r : Gv;
                }
            }
        }
        return Gv;
    };

    // The direction is chosen by the block index, so `D` is addressed through memory: taken inside the time loop its
    // fields cost a load and a wait per step.  Where registers allow (kCopy) they are copied once.
    constexpr bool kCopy = NZ * UPW < 12;
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
            for (int i = 0; i < NZP; ++i) {
                asm volatile("" : "+v"(o1[u][i]));
                asm volatile("" : "+v"(o2[u][i]));
            }
        asm volatile("" : "+v"(e1), "+v"(e2));   // likewise the per-gate selections of the overflow entry
        float pin = 0.f;
        if (ok1) pin = (kCopy ? P1_c : D.P1)[((size_t)t * B + b0 + pb) * (4 * (size_t)G) + 4 * unit_l + row];
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
            const float pre = products(w1, o1, n1, e1, ev1, hbuf) + pin;
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
            const float pre = products(w2, o2, n2, e2, ev2, ubuf) + bias2;
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
                    (kCopy ? y_c : D.y)[((size_t)t * B + b0 + pb) * (kCopy ? y_ld_c : (size_t)D.y_ld) + unit_l] = h;
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
// Choose (UPW, BW): the most workgroups that still fit one per compute unit, within the register budget, with
// PAIRS <= 16, 16-bit LDS offsets, and at most 64 unit groups (one flag per polling lane).
bool persist_batched_h_plan(int B, int H, int G, int nz, int ndir, int* upw_out, int* bw_out, int* ug_out, int* bg_out)
{
    if (B < 2 || nz < 1 || nz > 4 || H < 1 || G < 1) return false;
    const int units = std::max(H, G);
    int best = -1;
    for (int bw = 2; bw <= 4; bw *= 2) {
        if ((size_t)H * bw * 4 > 65536 || (size_t)4 * G * bw * 4 > 65536) continue;
        if (lds_bytes(H, G, bw) > (size_t)kMaxLds) continue;
        for (int upw = 2; upw <= 4; ++upw) {
            if (upw * bw > 16 || 12 * nz * upw > kWeightRegs) continue;
            const int ug = (units + kWaves * upw - 1) / (kWaves * upw), bg = (B + bw - 1) / bw;
            if (ug > 64) continue;
            const int blocks = ug * bg * ndir;
            if (blocks > device_num_cus()) continue;
            if (blocks > best) {
                best = blocks;
                *upw_out = upw; *bw_out = bw; *ug_out = ug; *bg_out = bg;
            }
        }
    }
    return best > 0;
}

// exchange storage per (direction, batch group), in elements of the respective array, padded to whole 256-byte blocks
size_t persist_batched_h_hstride(int H, int bw) { return (((size_t)H * bw * 8 + 255) / 256) * 256 / 8; }
size_t persist_batched_h_ustride(int G, int bw) { return (((size_t)4 * G * bw * 4 + 255) / 256) * 256 / 4; }

template <int NZ, int UPW, int BW>
static hipError_t launch_cfg(PersistBatchedHArgs& a, int blocks, bool cooperative, hipStream_t s)
{
    const size_t lds = lds_bytes(a.H, a.G, BW);
    auto kern = persist_batched_hlstm_kernel<NZ, UPW, BW>;
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

template <int NZ>
static hipError_t launch_nz(PersistBatchedHArgs& a, int upw, int bw, int blocks, bool coop, hipStream_t s)
{
#define CFG(U, W) if (upw == U && bw == W) return launch_cfg<NZ, U, W>(a, blocks, coop, s);
    CFG(2, 2) CFG(2, 4)
    if constexpr (12 * NZ * 3 <= kWeightRegs) { CFG(3, 2) CFG(3, 4) }
    if constexpr (12 * NZ * 4 <= kWeightRegs) { CFG(4, 2) CFG(4, 4) }
#undef CFG
    return hipErrorInvalidValue;
}

hipError_t launch_persist_batched_h(PersistBatchedHArgs& a, int ndir, int nz, int cooperative, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    int upw, bw, ug, bg;
    if (!persist_batched_h_plan(a.B, a.H, a.G, nz, ndir, &upw, &bw, &ug, &bg)) return hipErrorInvalidValue;
    a.ug = ug;
    a.bg = bg;
    a.h_stride = persist_batched_h_hstride(a.H, bw);
    a.u_stride = persist_batched_h_ustride(a.G, bw);
    // one XCD holds an eighth of the compute units; its share of the groups must fit there
    const int per_xcd = (ndir * bg + 7) / 8;
    a.ndir = ndir;
    a.xcd_local = per_xcd * ug <= device_num_cus() / 8;
    const int blocks = a.xcd_local ? 8 * per_xcd * ug : ug * bg * ndir;
    switch (nz) {
        case 1: return launch_nz<1>(a, upw, bw, blocks, cooperative != 0, s);
        case 2: return launch_nz<2>(a, upw, bw, blocks, cooperative != 0, s);
        case 3: return launch_nz<3>(a, upw, bw, blocks, cooperative != 0, s);
        case 4: return launch_nz<4>(a, upw, bw, blocks, cooperative != 0, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace l355

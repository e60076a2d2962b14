// Recurrence of a dense fp32 layer at small and medium batch with the time loop on the device (paper Section 4, cell
// equations): the form an unpruned model takes, and the form a row/column-pruned model takes once it has been compacted
// to its smaller dimensions (Section 4, row/column pruning; Section 5.1 step (b)).  One launch per layer, every direction
// of the layer in the same grid.
//
//   R[b][n] = sum_k h_{t-1}[b][k] * W_h[n][k]          (W_h packed rows n = 4 * unit + gate)
//   a = P[t][b][n] + R[b][n];  f,i,o = sigmoid, g = tanh;  c <- f*c + i*g;  h = o*tanh(c)
//
// A 512-thread workgroup owns 16 MT batch rows x 32 packed rows (8 hidden units) of one direction for the whole sequence.
// Its eight waves split K in blocks of 16; each wave's slice of W_h stays in registers as operand fragments of the
// 16x16x4 fp32 matrix instruction for all T steps, each of the first 128 MT threads keeps the cell state of one (batch
// row, unit) pair.  Per step a wave reads its slice of h_{t-1} (16 MT rows x its k) as operand fragments, the eight
// partial tiles are summed through LDS in a fixed order, and the gates are evaluated from the sums.
//
// Hidden-state exchange: B x H fp32 values per direction and step, every workgroup of a block of batch rows needing all
// of them.  The values carry their own readiness: |h| <= 1, so bit 30 of the fp32 pattern (the top exponent bit) is free
// and holds one bit of the step count.  A workgroup stores its 16 MT x 8 block of h_t into a [K blocks][rows][16] buffer
// with device-scope stores, each word stamped; a wave reads its operand fragments of h_{t-1} with device-scope loads and
// repeats the read until every word carries the stamp of step t-1 (bounded).  No flag, no wait for the stores'
// acknowledgement, no second round trip.  Two buffers alternate, step tag g (g = 2 for the first step of a launch) going
// to buffer g & 1 with stamp (g >> 1) & 1, so consecutive uses of a buffer alternate the stamp; the launcher clears the
// buffers in front of every launch (all stamps 0), and h0, if given, is placed by a kernel of its own where step 0 reads
// it (buffer 1, unstamped, taken as it is).  A workgroup writes h_t only after all of its waves have read h_{t-1}
// (barrier), whose producers each stored it after all of their waves had read h_{t-2} from the buffer h_t goes to.
// The first read of a step is paced (exchange.h): issued right behind the workgroup's own stores it would come back
// unstamped and cost a second round.  Every wait is bounded.
#include "common.h"
#include "device_math.h"
#include "exchange.h"

namespace l355 {

namespace {
typedef __attribute__((ext_vector_type(4))) float f32x4;
constexpr int kRN = 32, kUT = 8, kLDP = kRN + 4, kNW = 8, kNTH = 512;
constexpr unsigned kStampBit = 0x40000000u;   // top exponent bit of an fp32 pattern: clear in every |value| < 2
}  // namespace

// MT: 16-row blocks of batch rows per workgroup; KPW: k-blocks of 16 a wave holds at most
template <int MT, int KPW>
__global__ __launch_bounds__(512) void persist_dense_f32_kernel(PersistDenseArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float part[];   // [8][16 MT][36]
    constexpr int RM = 16 * MT;
    const int H = a.H, B = a.B, gm = a.gm, gn = a.gn;
    // Workgroups are dealt to the eight XCDs in turn.  The gn workgroups of one (direction, row block) are the only ones
    // that exchange h among themselves; where those groups fit, each takes block ids of one residue modulo 8, so that
    // it can hand h over through one XCD's L2 (checked below).
    int dir, tile_m, tile_n;
    if (a.xcd_local) {
        const int jj = blockIdx.x >> 3;
        const int grp = (blockIdx.x & 7) + 8 * (jj / gn);
        if (grp >= a.ndir * gm) return;                        // padding ids take no part in the exchange
        tile_n = jj % gn; dir = grp / gm; tile_m = grp - dir * gm;
    } else {
        const int per_dir = gm * gn;
        dir = blockIdx.x / per_dir;
        const int rem = blockIdx.x - dir * per_dir;
        tile_m = rem / gn; tile_n = rem - tile_m * gn;
    }
    const int m0 = tile_m * RM, n0 = tile_n * kRN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, lk = lane >> 4;
    const int Bp = gm * RM;
    const int KB = (H + 15) >> 4;
    const int per = (KB + kNW - 1) / kNW;                      // <= KPW (checked by the launcher)
    const int kb_beg = wave * per;
    const int kb_end = (kb_beg + per) < KB ? (kb_beg + per) : KB;
    const int nkb = kb_end > kb_beg ? kb_end - kb_beg : 0;     // wave-uniform

    // the direction is chosen by the block index, so its argument block lives in memory: fields copied once
    const PersistDenseDir& D = a.d[dir];
    const float* const Pd = D.P;
    const float* const Wh = D.Wh;
    float* const y_c = D.y;
    const size_t y_ld = (size_t)D.y_ld;
    float* const hT_c = D.hT;
    float* const cT_c = D.cT;
    const int reverse = D.reverse;
    const int has_h0 = D.has_h0;

    // W_h fragments of this wave: tile j, k-block q: lane l holds W_h[n0 + 16 j + l % 16][16 (kb_beg + q) + 4 (l / 16) .. + 3]
    float4 fb[2][KPW];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < KPW; ++q) {
            const int row = n0 + 16 * j + lr, k = 16 * (kb_beg + q) + 4 * lk;
            float v[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = (q < nkb && row < 4 * H && k + c < H) ? Wh[(size_t)row * H + k + c] : 0.f;
            fb[j][q] = make_float4(v[0], v[1], v[2], v[3]);
        }

    // exchange buffers of this direction: [2][KB][Bp][16] words
    const size_t xbuf = (size_t)KB * Bp * 16;
    unsigned* const hx = reinterpret_cast<unsigned*>(a.hx) + (size_t)dir * 2 * xbuf;

    // this thread's (batch row, unit) pair
    const int pr = tid >> 3, pu = tid & 7;                     // row inside the tile, unit inside the tile
    const int pb = m0 + pr, unit = (n0 >> 2) + pu;
    const bool in_tile = tid < RM * kUT;
    const bool live = in_tile && pb < B && unit < H;
    float c = (live && D.c0) ? D.c0[(size_t)pb * H + unit] : 0.f;

    bool same_xcd = false;
    if (a.xcd_local)
        same_xcd = group_shares_xcd(a.xcc_ids + (size_t)(dir * gm + tile_m) * 64, gn, tile_n, a.tag_base + 1u, part, tid, kNTH,
                                    a.timeout_flag, a.spin_limit) && !a.device_scope_only;

    for (int s = 0; s < a.T; ++s) {
        const int t = reverse ? a.T - 1 - s : s;
        // epilogue operand, requested first
        float4 pre = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live) pre = *reinterpret_cast<const float4*>(Pd + ((size_t)t * a.Bld + pb) * (4 * (size_t)H) + n0 + 4 * pu);
        f32x4 acc[MT][2];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

        if ((s > 0 || has_h0) && nkb > 0) {
            // h_{t-1} carries step tag s + 1: buffer (s + 1) & 1, stamp ((s + 1) >> 1) & 1 (h0: buffer 1, taken as it is)
            const unsigned g = (unsigned)s + 1u;
            const unsigned* hxs = hx + (size_t)(g & 1u) * xbuf;
            const unsigned long long kBits = ((unsigned long long)kStampBit << 32) | kStampBit;
            const unsigned long long want = (s > 0 && ((g >> 1) & 1u)) ? kBits : 0ull;
            const unsigned long long strip = s > 0 ? ~kBits : ~0ull;
            // Only the last k-block of the layer can reach beyond H; what lies there was never written.  Masks of a lane's
            // four words in that block, for the two 8-byte halves:
            const int klast = 16 * (KB - 1) + 4 * lk;
            const unsigned long long mlo_last = (klast + 0 < H ? 0xFFFFFFFFull : 0ull) | (klast + 1 < H ? 0xFFFFFFFF00000000ull : 0ull);
            const unsigned long long mhi_last = (klast + 2 < H ? 0xFFFFFFFFull : 0ull) | (klast + 3 < H ? 0xFFFFFFFF00000000ull : 0ull);
            if (s > 0) pace_poll(a.poll_pace);
            // the fragments as they are loaded (two 8-byte halves per lane, block and row tile): checked, then cleaned in place
            unsigned long long fr[MT][KPW][2];
            unsigned spins = 0;
            for (;;) {
                bool ok = true;
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int q = 0; q < KPW; ++q) {
                        fr[i][q][0] = fr[i][q][1] = 0ull;
                        if (q < nkb) {
                            // device-scope loads: never served from a stale line of this compute unit's cache or this XCD's L2
                            const unsigned long long* p8 = reinterpret_cast<const unsigned long long*>(
                                hxs + ((size_t)(kb_beg + q) * Bp + m0 + 16 * i + lr) * 16 + 4 * lk);
                            fr[i][q][0] = __hip_atomic_load(p8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            fr[i][q][1] = __hip_atomic_load(p8 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int q = 0; q < KPW; ++q) {
                        const bool tail = (kb_beg + q == KB - 1);                   // wave-uniform
                        const unsigned long long ml = tail ? mlo_last : ~0ull, mh = tail ? mhi_last : ~0ull;
                        if (q < nkb && s > 0)
                            ok = ok && (((fr[i][q][0] ^ want) & kBits & ml) == 0ull) && (((fr[i][q][1] ^ want) & kBits & mh) == 0ull);
                        fr[i][q][0] &= strip & ml;
                        fr[i][q][1] &= strip & mh;
                    }
                if (!__builtin_amdgcn_ballot_w64(!ok)) break;
                if (++spins > a.spin_limit) {
                    __hip_atomic_store(a.timeout_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                if ((spins & 63u) == 0 &&
                    __hip_atomic_load(a.timeout_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                    break;
            }
#pragma unroll
            for (int q = 0; q < KPW; ++q) {
                if (q < nkb) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
#pragma unroll
                        for (int i = 0; i < MT; ++i) {
                            const float av = __uint_as_float((unsigned)(fr[i][q][c >> 1] >> (32 * (c & 1))));
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const float bv = c == 0 ? fb[j][q].x : c == 1 ? fb[j][q].y : c == 2 ? fb[j][q].z : fb[j][q].w;
                                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[i][j], 0, 0, 0);
                            }
                        }
                    }
                }
            }
        }
        // partial tiles -> LDS.  Lane l of an accumulator tile holds rows 4 (l / 16) .. + 3 of column l % 16.
        float* mine = part + (size_t)wave * RM * kLDP;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) mine[(16 * i + 4 * lk + v) * kLDP + 16 * j + lr] = acc[i][j][v];
        __syncthreads();
        const bool last = (s == a.T - 1);
        float hn = 0.f;
        if (in_tile) {
            float4 sum = pre;
#pragma unroll
            for (int w = 0; w < kNW; ++w) {
                const float4 q = *reinterpret_cast<const float4*>(part + ((size_t)w * RM + pr) * kLDP + 4 * pu);
                sum.x += q.x;
                sum.y += q.y;
                sum.z += q.z;
                sum.w += q.w;
            }
            const float f = sigmoidf_fast(sum.x), ig = sigmoidf_fast(sum.y), o = sigmoidf_fast(sum.z), g = tanhf_fast(sum.w);
            const float cn = fmaf(f, c, ig * g);
            hn = o * tanhf_fast(cn);
            c = cn;
            // h_t carries step tag s + 2.  Rows beyond the batch are stored too (readers wait for every row's stamp; what
            // such a row holds is only ever multiplied into accumulator rows that are never used): their magnitude is
            // brought below 2 by clearing the exponent's top bit first.
            if (!last && unit < H) {
                const unsigned gw = (unsigned)s + 2u;
                exchange_store(hx + (size_t)(gw & 1u) * xbuf + ((size_t)(unit >> 4) * Bp + pb) * 16 + (unit & 15),
                               (__float_as_uint(hn) & ~kStampBit) | (((gw >> 1) & 1u) << 30), same_xcd);
            }
        }
        // keeps the next step's partial tiles out of LDS until every thread has read this step's
        if (!last) __syncthreads();
        // outputs after the publication: nothing on the way of h_t
        if (live) {
            y_c[((size_t)t * a.Bld + pb) * y_ld + unit] = hn;
            if (last) {
                if (hT_c) hT_c[(size_t)pb * H + unit] = hn;
                if (cT_c) cT_c[(size_t)pb * H + unit] = c;
            }
        }
    }
}

// h0 (fp32 [B][H]) -> the exchange buffer step 0 reads (buffer 1 of a direction) in the [K blocks][rows][16] layout
__global__ void h0_to_exchange_f32_kernel(const float* __restrict__ h0, float* __restrict__ hx, int B, int H, int Bp)
{
    const size_t n = (size_t)B * H;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t b = i / H, k = i % H;
        hx[((k >> 4) * Bp + b) * 16 + (k & 15)] = h0[i];
    }
}

// ------------------------------------------------------------------------------------------------ shapes and launch
namespace {
// k-blocks a wave must hold, rounded up to an instantiated count
int dense_kpw(int H)
{
    const int per = (((H + 15) / 16) + kNW - 1) / kNW;
    return per <= 4 ? 4 : per <= 8 ? 8 : per <= 12 ? 12 : 0;
}
// the shapes that fit the register file without spilling inside the time loop (16-row blocks per workgroup, k-blocks per wave)
bool dense_shape_built(int mt, int kpw)
{
    return (kpw == 4 && mt <= 4) || (kpw == 8 && mt <= 2) || (kpw == 12 && mt == 1);
}
// 16-row blocks of batch rows per workgroup: the fewest that are built for this width and leave a grid of at most one
// workgroup per compute unit (more, smaller row blocks spread the matrix work over more compute units and exchange less
// per block: H = 1024 at batch 20 takes 11 us per step as one block of 32 rows and half that as blocks of 16 and 4); 0 if
// there is none
int dense_mt(int B, int H, int ndir)
{
    const int kpw = dense_kpw(H);
    const int gn = (4 * H + kRN - 1) / kRN;
    const int most = (B + 15) / 16 > 4 ? 4 : (B + 15) / 16;
    for (int mt = 1; mt <= most; ++mt)
        if (dense_shape_built(mt, kpw) && (long)ndir * ((B + 16 * mt - 1) / (16 * mt)) * gn <= device_num_cus()) return mt;
    return 0;
}
}  // namespace

bool persist_dense_f32_supported(int B, int H, int ndir)
{
    if (B < 2 || H < 1 || ndir < 1 || ndir > 2) return false;
    return dense_mt(B, H, ndir) > 0;
}

// one run of 64 slots per (direction, row block); there are at most as many of those as compute units
size_t persist_dense_f32_ids_count() { return (size_t)device_num_cus() * 64; }

size_t persist_dense_f32_exchange_floats(int B, int H, int ndir)
{
    const int mt = dense_mt(B, H, ndir);
    if (mt == 0) return 0;
    const size_t Bp = (size_t)((B + 16 * mt - 1) / (16 * mt)) * (16 * mt);
    return (size_t)ndir * 2 * ((size_t)(H + 15) / 16) * Bp * 16;
}

template <int MT, int KPW>
static hipError_t launch_dense_shape(PersistDenseArgs& a, const float* const* h0, bool cooperative, hipStream_t s)
{
    constexpr int RM = 16 * MT;
    a.gm = (a.B + RM - 1) / RM;
    a.gn = (4 * a.H + kRN - 1) / kRN;
    // One XCD holds an eighth of the compute units; its share of the groups (gn workgroups each) must fit there: layers of
    // at most 256 units.  (H = 256 at batch 16: 2.31 us per step across the device, 1.89 inside one XCD.  Workgroups of 64
    // packed rows, which would let groups of layers up to 512 wide fit, measured slower than 32 rows across the device:
    // 2.96 against 2.68 us at H = 320, 3.96 against 3.3 at 512 -- twice the partial tiles per workgroup.)
    const int groups_per_xcd = (a.ndir * a.gm + 7) / 8;
    a.xcd_local = (a.xcc_ids != nullptr && a.gn <= 64 && groups_per_xcd * a.gn <= device_num_cus() / 8) ? 1 : 0;
    if (a.xcd_local) a.poll_pace = 0;   // an exchange inside one XCD is visible by the time the first read arrives
    const int grid = a.xcd_local ? 8 * groups_per_xcd * a.gn : a.ndir * a.gm * a.gn;
    const size_t lds = (size_t)kNW * RM * kLDP * sizeof(float);
    const size_t xbuf = (size_t)((a.H + 15) / 16) * a.gm * RM * 16;
    for (int d = 0; d < a.ndir; ++d) {
        a.d[d].has_h0 = h0[d] != nullptr;
        if (h0[d]) {
            const size_t n = (size_t)a.B * a.H;
            int g = (int)((n + 255) / 256);
            if (g > 2048) g = 2048;
            hipLaunchKernelGGL(h0_to_exchange_f32_kernel, dim3(g), dim3(256), 0, s, h0[d], a.hx + ((size_t)d * 2 + 1) * xbuf, a.B,
                               a.H, a.gm * RM);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    const void* kern = (const void*)persist_dense_f32_kernel<MT, KPW>;
    if (lds > 64 * 1024) {
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
    }
    void* kargs[] = {(void*)&a};
    // every workgroup must be resident at the same time: at most one per compute unit
    if (grid > device_num_cus()) return hipErrorCooperativeLaunchTooLarge;
    if (cooperative) return hipLaunchCooperativeKernel(kern, dim3(grid), dim3(kNTH), kargs, (unsigned)lds, s);
    return hipLaunchKernel(kern, dim3(grid), dim3(kNTH), kargs, lds, s);
}

hipError_t launch_persist_dense_f32(PersistDenseArgs& a, const float* const* h0, bool cooperative, hipStream_t s)
{
    if (a.B <= 0 || a.H <= 0 || a.T <= 0) return hipSuccess;
    if (!persist_dense_f32_supported(a.B, a.H, a.ndir)) return hipErrorInvalidValue;
    const int mt = dense_mt(a.B, a.H, a.ndir), kpw = dense_kpw(a.H);
#define SHAPE(M_, K_) if (mt == M_ && kpw == K_) return launch_dense_shape<M_, K_>(a, h0, cooperative, s);
    SHAPE(1, 4) SHAPE(2, 4) SHAPE(3, 4) SHAPE(4, 4)
    SHAPE(1, 8) SHAPE(2, 8)
    SHAPE(1, 12)
#undef SHAPE
    return hipErrorInvalidValue;
}

}  // namespace l355

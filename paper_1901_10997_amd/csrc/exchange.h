// Tagged-slot exchange of hidden-state values between workgroups (device side).
// A slot is 64 bits: low word = fp32 value, high word = step tag.  One 8-byte store publishes both, so a
// consumer that sees the expected tag also has the value; a stale read carries an old tag and is retried.
#pragma once
#include <hip/hip_runtime.h>

namespace l355 {

typedef unsigned long long u64;

__device__ __forceinline__ u64 pack_slot(float v, unsigned tag)
{
    return ((u64)tag << 32) | (u64)__float_as_uint(v);
}

// Pacing of a poll that would otherwise follow the wave's own publication at once.  A device-scope store takes about
// 0.3 us plus half a load round trip to become visible to the other XCDs; a poll round issued before that comes back
// without the value and the next round costs a whole further round trip (about 1 us with a few thousand slots polled by
// every workgroup).  Waiting `units` x 64 clocks first makes the first round the one that succeeds: the bare exchange of
// 3000 slots among 250 workgroups takes 1.83 us per round unpaced and 1.43 us with 10-12 units.  Where a kernel has work
// of its own between publication and poll (outputs, the next step's input products) that work is the pacing.
__device__ __forceinline__ void pace_poll(int units)
{
    for (int i = 0; i < units; ++i) __builtin_amdgcn_s_sleep(1);
}

// One polled slot array: n slots tagged `want` go to dst[0..n).  n = 0 switches the array off.
struct PollSrc {
    const u64* slots;
    float* dst;
    unsigned want;
    int n;
};

// Fetch the tagged values of up to two slot arrays into LDS.  The two arrays are treated as one index space
// so that all outstanding loads of a thread (up to NF) are in flight together, whichever array they hit.
template <int NF = 4>
__device__ __forceinline__ void gather_tagged2(const PollSrc& A, const PollSrc& Bs, int tid, int nthreads,
                                               int* timeout_flag, unsigned spin_limit)
{
    const int total = A.n + Bs.n;
    for (int e0 = tid; e0 < total; e0 += NF * nthreads) {
        u64 v[NF];
        unsigned spins = 0;
        bool ok;
        do {
            ok = true;
#pragma unroll
            for (int u = 0; u < NF; ++u) {
                const int e = e0 + u * nthreads;
                const bool second = e >= A.n;
                const u64* p = second ? (Bs.slots + (e - A.n)) : (A.slots + e);
                const unsigned want = second ? Bs.want : A.want;
                v[u] = (e < total) ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ((u64)want << 32);
                ok = ok && ((unsigned)(v[u] >> 32) == want);
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
            if (e < total) {
                if (e >= A.n) Bs.dst[e - A.n] = __uint_as_float((unsigned)v[u]);
                else A.dst[e] = __uint_as_float((unsigned)v[u]);
            }
        }
    }
}

__device__ __forceinline__ void gather_tagged(const u64* slots, int H, unsigned want, float* dst, int tid,
                                              int nthreads, int* timeout_flag, unsigned spin_limit)
{
    const PollSrc A{slots, dst, want, H}, none{nullptr, nullptr, 0u, 0};
    gather_tagged2<4>(A, none, tid, nthreads, timeout_flag, spin_limit);
}
// For kernels with sixteen registers to spare: a thread with more than four slots to fetch keeps eight loads in
// flight (one polling round less).
__device__ __forceinline__ void gather_tagged_wide(const u64* slots, int H, unsigned want, float* dst, int tid,
                                                   int nthreads, int* timeout_flag, unsigned spin_limit)
{
    const PollSrc A{slots, dst, want, H}, none{nullptr, nullptr, 0u, 0};
    if (H > 4 * nthreads) gather_tagged2<8>(A, none, tid, nthreads, timeout_flag, spin_limit);
    else gather_tagged2<4>(A, none, tid, nthreads, timeout_flag, spin_limit);
}

// As gather_tagged for slots stored in the order of their destination (slot e -> dst[e]), where slot e belongs to
// column e % BW of a batch group that may hold fewer than BW columns: the slots of the missing columns are never
// published and are skipped.
template <int NF, int BW>
__device__ __forceinline__ void gather_tagged_cols(const u64* slots, int n, int bw, unsigned want, float* dst, int tid,
                                                   int nthreads, int* timeout_flag, unsigned spin_limit)
{
    for (int e0 = tid; e0 < n; e0 += NF * nthreads) {
        u64 v[NF];
        unsigned spins = 0;
        bool ok;
        do {
            ok = true;
#pragma unroll
            for (int u = 0; u < NF; ++u) {
                const int e = e0 + u * nthreads;
                const bool live = e < n && (e & (BW - 1)) < bw;
                v[u] = live ? __hip_atomic_load(slots + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ((u64)want << 32);
                ok = ok && ((unsigned)(v[u] >> 32) == want);
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
            if (e < n && (e & (BW - 1)) < bw) dst[e] = __uint_as_float((unsigned)v[u]);
        }
    }
}

// ---- exchange inside one XCD -------------------------------------------------------------------------------------
// The compute units of an XCD share one L2.  A store at workgroup scope is written through the compute unit's vector
// cache into that L2 and stays there; an agent-scope load from any compute unit of the same XCD bypasses its vector
// cache and finds it in the L2.  For workgroups that all run on one XCD this hand-over measured 35-50 % faster than
// agent-scope stores, which travel to memory before anybody sees them (32 workgroups: 1.19 -> 0.78 us per round;
// 16: 1.71 -> 0.86 us).  A workgroup on another XCD would never see such a store, so a group uses it only after it has
// checked, in the launch itself, that its members do share an XCD.  (The loads stay at agent scope: polling loads at
// workgroup scope may be served by the compute unit's own cache and never see anything.)

// id of the XCD this wave runs on (hardware register XCC_ID, bits 3:0)
__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)); }

// publish v at p for the other workgroups of the group
template <class T>
__device__ __forceinline__ void exchange_store(T* p, T v, bool same_xcd)
{
    if (same_xcd) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Do the `members` (<= 64) workgroups of this group all run on one XCD?  Every member publishes its XCD id in
// ids[me] (agent scope, tagged `tag`), polls the whole list and compares; all of them read the same list and so
// agree on the answer.  tmp: LDS, `members` floats, free for other use on return.  Called by the whole workgroup.
__device__ __forceinline__ bool group_shares_xcd(u64* ids, int members, int me, unsigned tag, float* tmp, int tid,
                                                 int nthreads, int* timeout_flag, unsigned spin_limit)
{
    if (tid == 0) __hip_atomic_store(ids + me, pack_slot((float)xcc_id(), tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    gather_tagged(ids, members, tag, tmp, tid, nthreads, timeout_flag, spin_limit);
    __syncthreads();
    bool same = true;
    const float first = tmp[0];
    for (int i = 1; i < members; ++i) same = same && (tmp[i] == first);
    __syncthreads();
    return same;
}

}  // namespace l355

// Measurement kernel: the tagged-slot exchange inside groups of workgroups, with no arithmetic.
#include "common.h"
#include "exchange.h"

namespace l355 {

// Exchange with no arithmetic inside groups of workgroups: `groups` groups of `members` workgroups, each group passing
// `n` tagged slots round among its members (every member publishes its share and polls all n), `steps` rounds.  The
// yardstick for the kernels whose workgroups exchange only inside a (direction, batch group).  placed = 1: a group's
// members take block ids of one residue modulo 8; the group checks from the hardware's XCD ids that it does share an XCD
// and, if `workgroup_stores` is set as well, then publishes with workgroup-scope stores.  verified counts the groups
// whose check succeeded.
__global__ __launch_bounds__(512) void group_exchange_kernel(u64* slots, u64* ids, unsigned tag_base, int n, int members,
                                                             int groups, int placed, int workgroup_stores, int steps,
                                                             int* timeout_flag, unsigned spin_limit, int* verified)
{
    extern __shared__ float lds[];  // [n]
    const int tid = threadIdx.x, nthreads = blockDim.x;
    int grp, mem;
    if (placed) {
        const int jj = blockIdx.x >> 3;
        grp = (blockIdx.x & 7) + 8 * (jj / members);
        mem = jj % members;
        if (grp >= groups) return;
    } else {
        grp = blockIdx.x / members;
        mem = blockIdx.x % members;
    }
    u64* gs = slots + (size_t)grp * 2 * n;
    bool same_xcd = false;
    if (placed) {
        same_xcd = group_shares_xcd(ids + (size_t)grp * 64, members, mem, tag_base + 1u, lds, tid, nthreads, timeout_flag,
                                    spin_limit);
        if (same_xcd && mem == 0 && tid == 0) atomicAdd(verified, 1);
    }
    const bool wg = same_xcd && workgroup_stores != 0;
    const int per = (n + members - 1) / members, e0 = mem * per;
    for (int s = 0; s < steps; ++s) {
        if (s > 0) gather_tagged(gs + (size_t)(s & 1) * n, n, tag_base + (unsigned)s, lds, tid, nthreads, timeout_flag, spin_limit);
        __syncthreads();
        if (s + 1 < steps) {
            u64* out = gs + (size_t)((s + 1) & 1) * n;
            for (int e = e0 + tid; e < e0 + per && e < n; e += nthreads)
                exchange_store(out + e, pack_slot((float)(s + 1), tag_base + (unsigned)s + 1u), wg);
        }
    }
}

hipError_t launch_group_exchange(u64* slots, u64* ids, unsigned tag_base, int n, int members, int groups, int placed,
                                 int workgroup_stores, int steps, int* timeout_flag, unsigned spin_limit, int* verified,
                                 int cooperative, hipStream_t s)
{
    if (n < 1 || n > 16384 || members < 1 || members > 64 || groups < 1 || steps < 2) return hipErrorInvalidValue;
    const int per_xcd = (groups + 7) / 8;
    if (placed && per_xcd * members > device_num_cus() / 8) return hipErrorInvalidValue;
    const int blocks = placed ? 8 * per_xcd * members : groups * members;
    const size_t lds = (size_t)(n > 64 ? n : 64) * sizeof(float);
    void* args[] = {(void*)&slots, (void*)&ids, (void*)&tag_base, (void*)&n, (void*)&members, (void*)&groups, (void*)&placed,
                    (void*)&workgroup_stores, (void*)&steps, (void*)&timeout_flag, (void*)&spin_limit, (void*)&verified};
    if (blocks > device_num_cus()) return hipErrorCooperativeLaunchTooLarge;   // every workgroup must be resident
    if (cooperative) return hipLaunchCooperativeKernel((const void*)group_exchange_kernel, dim3(blocks), dim3(512), args, (unsigned)lds, s);
    return hipLaunchKernel((const void*)group_exchange_kernel, dim3(blocks), dim3(512), args, lds, s);
}

}  // namespace l355

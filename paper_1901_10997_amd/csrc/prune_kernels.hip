// Mask updates of the pruning phases on the device (paper Section 4: magnitude-based weight pruning,
// "Msk(w) = 0 iff |w| <= the (100 p_w)-th percentile of |W|"; row/column pruning algorithm: rows / columns whose
// magnitude sum is at or below an order statistic of the row / column sums are removed).
//
// Both need a k-th smallest value.  Magnitudes and magnitude sums are non-negative floats, whose bit patterns order
// like unsigned integers, so the selection is a four-pass radix select on 32-bit keys: each pass histograms one
// byte of the keys that still match the prefix found so far (LDS histogram per workgroup, then 256 global atomics),
// and a one-thread kernel walks the 256 bins to fix the next byte of the answer.  Nothing returns to the host
// between the passes.  Entries that do not take part (mask byte 0) get the key 0xFFFFFFFF, above every magnitude.
#include "common.h"

namespace l355 {

struct SelectState {
    unsigned prefix;      // bytes of the answer fixed so far (high bytes first)
    unsigned k;           // rank (1-based) still to be found among the keys matching the prefix
    unsigned hist[256];
};

__global__ void weight_keys_kernel(const float* __restrict__ W, const uint8_t* __restrict__ mask, unsigned* __restrict__ keys,
                                   size_t n, unsigned long long* __restrict__ active)
{
    unsigned long long cnt = 0;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const bool on = mask[i] != 0;
        keys[i] = on ? (__float_as_uint(W[i]) & 0x7FFFFFFFu) : 0xFFFFFFFFu;
        cnt += on ? 1u : 0u;
    }
    // one atomic per wave
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
    if ((threadIdx.x & 63) == 0 && cnt) atomicAdd(active, cnt);
}

__global__ void select_init_kernel(SelectState* st, const unsigned long long* count, double ratio, unsigned k_fixed)
{
    // k = ceil(ratio * count) when a count is given, else the fixed rank
    unsigned k = k_fixed;
    if (count) {
        const double c = (double)*count;
        double kk = ceil(ratio * c);
        if (kk > c) kk = c;
        k = (unsigned)kk;
    }
    st->prefix = 0;
    st->k = k;
    for (int b = 0; b < 256; ++b) st->hist[b] = 0;
}

__global__ __launch_bounds__(256) void select_hist_kernel(const unsigned* __restrict__ keys, size_t n, SelectState* st, int shift)
{
    __shared__ unsigned h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const unsigned prefix = st->prefix;
    const unsigned high_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const unsigned key = keys[i];
        if ((key & high_mask) == (prefix & high_mask)) atomicAdd(&h[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&st->hist[threadIdx.x], h[threadIdx.x]);
}

__global__ void select_step_kernel(SelectState* st, int shift)
{
    unsigned k = st->k, cum = 0;
    int b = 0;
    if (k > 0) {
        for (; b < 255; ++b) {
            if (cum + st->hist[b] >= k) break;
            cum += st->hist[b];
        }
        st->prefix |= (unsigned)b << shift;
        st->k = k - cum;
    }
    for (int i = 0; i < 256; ++i) st->hist[i] = 0;
}

// mask[i] = 0 where the entry took part and its key is at or below the selected one (rank 0: nothing)
__global__ void apply_weight_threshold_kernel(const unsigned* __restrict__ keys, uint8_t* __restrict__ mask, size_t n,
                                              const SelectState* st, unsigned long long* __restrict__ kept_after)
{
    const bool any = st->k > 0;
    const unsigned thr = st->prefix;
    unsigned long long cnt = 0;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const unsigned key = keys[i];
        const bool on = key != 0xFFFFFFFFu;
        const bool keep = on && !(any && key <= thr);
        if (on && !keep) mask[i] = 0;
        cnt += keep ? 1u : 0u;
    }
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
    if ((threadIdx.x & 63) == 0 && cnt) atomicAdd(kept_after, cnt);
}

// sums[r] = sum_k mask ? |W[r][k]| : 0, one wave per row, lanes over columns, fp32 accumulation
__global__ __launch_bounds__(256) void row_abs_sum_kernel(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                          int M, int N, float* __restrict__ sums, unsigned* __restrict__ keys)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= M) return;
    float acc = 0.f;
    for (int k = lane; k < N; k += 64) {
        const size_t i = (size_t)r * N + k;
        acc += mask[i] ? fabsf(W[i]) : 0.f;
    }
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
        sums[r] = acc;
        if (keys) keys[r] = __float_as_uint(acc);
    }
}

// sums[c] = sum_r mask ? |W[r][c]| : 0, one thread per column (coalesced across a wave), rows in index order
__global__ void col_abs_sum_kernel(const float* __restrict__ W, const uint8_t* __restrict__ mask, int M, int N,
                                   float* __restrict__ sums, unsigned* __restrict__ keys)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= N) return;
    float acc = 0.f;
    for (int r = 0; r < M; ++r) {
        const size_t i = (size_t)r * N + c;
        acc += mask[i] ? fabsf(W[i]) : 0.f;
    }
    sums[c] = acc;
    if (keys) keys[c] = __float_as_uint(acc);
}

// rows whose sum is at or below the selected row threshold are removed (mask and weights zeroed)
__global__ void apply_row_threshold_kernel(float* __restrict__ W, uint8_t* __restrict__ mask, int M, int N,
                                           const float* __restrict__ sums, const SelectState* st, int* __restrict__ removed)
{
    const int r = blockIdx.x;
    if (st->k == 0 || !(__float_as_uint(sums[r]) <= st->prefix)) return;
    for (int k = threadIdx.x; k < N; k += blockDim.x) {
        mask[(size_t)r * N + k] = 0;
        W[(size_t)r * N + k] = 0.f;
    }
    if (threadIdx.x == 0) atomicAdd(removed, 1);
}

__global__ void apply_col_threshold_kernel(float* __restrict__ W, uint8_t* __restrict__ mask, int M, int N,
                                           const float* __restrict__ sums, const SelectState* st, int* __restrict__ removed)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= N || st->k == 0 || !(__float_as_uint(sums[c]) <= st->prefix)) return;
    for (int r = 0; r < M; ++r) {
        mask[(size_t)r * N + c] = 0;
        W[(size_t)r * N + c] = 0.f;
    }
    atomicAdd(removed, 1);
}

static int grid_for(size_t n)
{
    size_t g = (n + 255) / 256;
    return (int)(g > 2048 ? 2048 : (g < 1 ? 1 : g));
}

// four passes over the keys; leaves the k-th smallest key in st->prefix (st->k == 0 on entry: no selection)
static hipError_t radix_select(const unsigned* keys, size_t n, SelectState* st, hipStream_t s)
{
    for (int shift = 24; shift >= 0; shift -= 8) {
        hipLaunchKernelGGL(select_hist_kernel, dim3(grid_for(n)), dim3(256), 0, s, keys, n, st, shift);
        hipLaunchKernelGGL(select_step_kernel, dim3(1), dim3(1), 0, s, st, shift);
    }
    return hipGetLastError();
}

// scratch: keys [count] u32, state (SelectState), counters 2 x u64
hipError_t launch_prune_weights(const float* W, uint8_t* mask, size_t count, double p_w, unsigned* keys, void* state,
                                unsigned long long* counters, hipStream_t s)
{
    SelectState* st = (SelectState*)state;
    hipError_t e = launch_fill_u64(counters, 2, 0ull, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(weight_keys_kernel, dim3(grid_for(count)), dim3(256), 0, s, W, mask, keys, count, counters);
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(1), 0, s, st, counters, p_w, 0u);
    // a rank of zero (nothing to prune) stays zero through the passes; otherwise the state ends with k >= 1
    e = radix_select(keys, count, st, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(apply_weight_threshold_kernel, dim3(grid_for(count)), dim3(256), 0, s, keys, mask, count, st, counters + 1);
    return hipGetLastError();
}
size_t prune_state_bytes() { return sizeof(SelectState); }

// scratch: sums [max(M,N)] f32, keys [max(M,N)] u32, two states, removed 2 x int
hipError_t launch_prune_rows_cols(float* W, uint8_t* mask, int M, int N, unsigned k_rows, unsigned k_cols, float* sums,
                                  unsigned* keys, void* state_r, void* state_c, int* removed, hipStream_t s)
{
    SelectState* sr = (SelectState*)state_r;
    SelectState* sc = (SelectState*)state_c;
    hipError_t e = launch_fill_u64((unsigned long long*)removed, 1, 0ull, s);   // two ints, 8-byte aligned
    if (e != hipSuccess) return e;
    // both thresholds from the matrix as it came in
    hipLaunchKernelGGL(row_abs_sum_kernel, dim3((M + 3) / 4), dim3(256), 0, s, W, mask, M, N, sums, keys);
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(1), 0, s, sr, (const unsigned long long*)nullptr, 0.0, k_rows);
    e = radix_select(keys, (size_t)M, sr, s);
    if (e != hipSuccess) return e;
    float* csums = sums + M;
    hipLaunchKernelGGL(col_abs_sum_kernel, dim3((N + 255) / 256), dim3(256), 0, s, W, mask, M, N, csums, keys);
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(1), 0, s, sc, (const unsigned long long*)nullptr, 0.0, k_cols);
    e = radix_select(keys, (size_t)N, sc, s);
    if (e != hipSuccess) return e;
    // rows first, then columns judged on what the row pass left
    hipLaunchKernelGGL(apply_row_threshold_kernel, dim3(M), dim3(256), 0, s, W, mask, M, N, sums, sr, removed);
    hipLaunchKernelGGL(col_abs_sum_kernel, dim3((N + 255) / 256), dim3(256), 0, s, W, mask, M, N, csums, (unsigned*)nullptr);
    hipLaunchKernelGGL(apply_col_threshold_kernel, dim3((N + 255) / 256), dim3(256), 0, s, W, mask, M, N, csums, sc, removed + 1);
    return hipGetLastError();
}

}  // namespace l355

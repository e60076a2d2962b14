// Mask updates of the pruning phases on the device (paper Section 4: magnitude-based weight pruning,
// "Msk(w) = 0 iff |w| <= the (100 p_w)-th percentile of |W|"; row/column pruning algorithm: rows / columns whose
// magnitude sum is at or below an order statistic of the row / column sums are removed).
//
// Both need a k-th smallest value of non-negative floating-point numbers, whose bit patterns order like unsigned
// integers, so the selection is a byte-wise radix select.  Weight pruning: 32-bit keys (the magnitudes), four passes,
// each histogramming one byte of the keys that still match the prefix found so far (LDS histogram per workgroup, then
// 256 global atomics), and a one-thread kernel that walks the 256 bins to fix the next byte of the answer; entries that
// do not take part (mask byte 0) get the key 0xFFFFFFFF, above every magnitude.  Row/column pruning: 64-bit keys (fp64
// sums), a few thousand of them, eight passes inside one workgroup.  Nothing returns to the host between the passes.
#include "common.h"

#include <mutex>

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

// ---- row / column pruning -------------------------------------------------------------------------------------
// Importance of a line (row or column) = sum of the magnitudes of its active entries, accumulated in fp64 in index
// order: s = (...((+0 + e_0) + e_1) + ...) + e_last, where e_k = |W| for an active entry and +0 otherwise (adding
// +0 to a non-negative double changes nothing).  The order is part of the definition: an fp64 sum of several
// thousand fp32 magnitudes is not exact in general, and the decision "sum <= threshold" must come out the same on
// every implementation for the masks to be reproducible bit for bit.
//
// Both kernels stage tiles in LDS so that the global reads are coalesced whatever the direction of the sum, and one
// wave then adds a tile's values line by line; the loads of the next tile are in flight meanwhile.
constexpr int kSumTile = 128;   // positions of a line per tile

// sums[c], 64 columns per workgroup; a wave reads 64 consecutive columns of one row per load
__global__ __launch_bounds__(256) void col_abs_sum_f64_kernel(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                              int M, int N, double* __restrict__ sums)
{
    __shared__ float tile[kSumTile][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    const bool col_ok = c < N;
    float v[kSumTile / 4];
    auto fetch = [&](int r0) {
#pragma unroll
        for (int i = 0; i < kSumTile / 4; ++i) {
            const int r = r0 + wave + 4 * i;
            const bool ok = col_ok && r < M;
            const size_t idx = ok ? (size_t)r * N + c : 0;
            const float w = W[idx];
            const uint8_t on = mask[idx];
            v[i] = (ok && on) ? fabsf(w) : 0.f;
        }
    };
    double acc = 0.0;
    fetch(0);
    for (int r0 = 0; r0 < M; r0 += kSumTile) {
#pragma unroll
        for (int i = 0; i < kSumTile / 4; ++i) tile[wave + 4 * i][lane] = v[i];
        __syncthreads();
        if (r0 + kSumTile < M) fetch(r0 + kSumTile);
        if (wave == 0) {
#pragma unroll 16
            for (int i = 0; i < kSumTile; ++i) acc += (double)tile[i][lane];
        }
        __syncthreads();
    }
    if (wave == 0 && col_ok) sums[c] = acc;
}

// sums[r], 64 rows per workgroup; a wave reads 64 consecutive columns of one row per load and parks them transposed
__global__ __launch_bounds__(256) void row_abs_sum_f64_kernel(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                              int M, int N, double* __restrict__ sums)
{
    constexpr int kRowsPerWave = 16, kChunks = kSumTile / 64;
    __shared__ float tile[kSumTile][65];   // [position][row], odd stride: both the parking and the summing are conflict-free
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rbase = blockIdx.x * 64;
    float v[kRowsPerWave * kChunks];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i)
#pragma unroll
            for (int j = 0; j < kChunks; ++j) {
                const int r = rbase + wave * kRowsPerWave + i, k = k0 + 64 * j + lane;
                const bool ok = r < M && k < N;
                const size_t idx = ok ? (size_t)r * N + k : 0;
                const float w = W[idx];
                const uint8_t on = mask[idx];
                v[i * kChunks + j] = (ok && on) ? fabsf(w) : 0.f;
            }
    };
    double acc = 0.0;
    fetch(0);
    for (int k0 = 0; k0 < N; k0 += kSumTile) {
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i)
#pragma unroll
            for (int j = 0; j < kChunks; ++j) tile[64 * j + lane][wave * kRowsPerWave + i] = v[i * kChunks + j];
        __syncthreads();
        if (k0 + kSumTile < N) fetch(k0 + kSumTile);
        if (wave == 0) {
#pragma unroll 16
            for (int i = 0; i < kSumTile; ++i) acc += (double)tile[i][lane];
        }
        __syncthreads();
    }
    const int r = rbase + lane;
    if (wave == 0 && r < M) sums[r] = acc;
}

struct LineThreshold {
    double value;   // the k-th smallest sum
    unsigned any;   // 0: rank 0 was asked for, nothing is removed along this axis
    unsigned pad;
};

// k-th smallest (1-based) of n non-negative doubles, whose bit patterns order like 64-bit unsigned integers: eight
// byte-wide radix passes by one workgroup, histogram in LDS.  n is a row or column count, a few thousand.
__global__ __launch_bounds__(1024) void select_kth_f64_kernel(const double* __restrict__ sums, int n, unsigned k,
                                                              LineThreshold* __restrict__ out)
{
    __shared__ unsigned hist[256];
    __shared__ unsigned long long prefix_s;
    __shared__ unsigned k_s;
    if (threadIdx.x == 0) { prefix_s = 0ull; k_s = k; }
    __syncthreads();
    for (int shift = 56; shift >= 0 && k > 0; shift -= 8) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        const unsigned long long prefix = prefix_s;
        const unsigned long long high_mask = shift == 56 ? 0ull : (~0ull << (shift + 8));
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            const unsigned long long key = (unsigned long long)__double_as_longlong(sums[i]);
            if ((key & high_mask) == prefix) atomicAdd(&hist[(unsigned)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned kk = k_s, cum = 0;
            int b = 0;
            for (; b < 255; ++b) {
                if (cum + hist[b] >= kk) break;
                cum += hist[b];
            }
            prefix_s = prefix | ((unsigned long long)b << shift);
            k_s = kk - cum;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out->value = __longlong_as_double((long long)prefix_s);
        out->any = k > 0 ? 1u : 0u;
        out->pad = 0u;
    }
}

// rows whose sum is at or below the row threshold are removed (mask and weights zeroed)
__global__ void apply_row_threshold_kernel(float* __restrict__ W, uint8_t* __restrict__ mask, int M, int N,
                                           const double* __restrict__ sums, const LineThreshold* __restrict__ th,
                                           int* __restrict__ removed)
{
    const int r = blockIdx.x;
    if (th->any == 0 || !(sums[r] <= th->value)) return;
    for (int k = threadIdx.x; k < N; k += blockDim.x) {
        mask[(size_t)r * N + k] = 0;
        W[(size_t)r * N + k] = 0.f;
    }
    if (threadIdx.x == 0) atomicAdd(removed, 1);
}

// columns likewise; lanes over columns, blockIdx.y over row chunks
__global__ void apply_col_threshold_kernel(float* __restrict__ W, uint8_t* __restrict__ mask, int M, int N,
                                           const double* __restrict__ sums, const LineThreshold* __restrict__ th,
                                           int* __restrict__ removed)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= N || th->any == 0 || !(sums[c] <= th->value)) return;
    const int rows_per = (M + gridDim.y - 1) / gridDim.y;
    const int r0 = blockIdx.y * rows_per, r1 = min(M, r0 + rows_per);
    for (int r = r0; r < r1; ++r) {
        mask[(size_t)r * N + c] = 0;
        W[(size_t)r * N + c] = 0.f;
    }
    if (blockIdx.y == 0) atomicAdd(removed, 1);
}

__global__ void clear_removed_kernel(int* removed)
{
    if (threadIdx.x < 2) removed[threadIdx.x] = 0;
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

// scratch (prune_rows_cols_scratch_bytes): row sums [M] f64 | column sums [N] f64 | two thresholds | removed 2 x int
size_t prune_rows_cols_scratch_bytes(int M, int N)
{
    return ((size_t)M + (size_t)N) * sizeof(double) + 2 * sizeof(LineThreshold) + 2 * sizeof(int);
}

hipError_t launch_prune_rows_cols(float* W, uint8_t* mask, int M, int N, unsigned k_rows, unsigned k_cols, void* scratch,
                                  int** removed_out, hipStream_t s)
{
    double* rsums = (double*)scratch;
    double* csums = rsums + M;
    LineThreshold* th = (LineThreshold*)(csums + N);
    int* removed = (int*)(th + 2);
    if (removed_out) *removed_out = removed;
    hipLaunchKernelGGL(clear_removed_kernel, dim3(1), dim3(64), 0, s, removed);
    // both thresholds from the matrix as it came in
    hipLaunchKernelGGL(row_abs_sum_f64_kernel, dim3((M + 63) / 64), dim3(256), 0, s, W, mask, M, N, rsums);
    hipLaunchKernelGGL(col_abs_sum_f64_kernel, dim3((N + 63) / 64), dim3(256), 0, s, W, mask, M, N, csums);
    hipLaunchKernelGGL(select_kth_f64_kernel, dim3(1), dim3(1024), 0, s, rsums, M, k_rows, th);
    hipLaunchKernelGGL(select_kth_f64_kernel, dim3(1), dim3(1024), 0, s, csums, N, k_cols, th + 1);
    // rows first, then columns judged on what the row pass left
    hipLaunchKernelGGL(apply_row_threshold_kernel, dim3(M), dim3(256), 0, s, W, mask, M, N, rsums, th, removed);
    hipLaunchKernelGGL(col_abs_sum_f64_kernel, dim3((N + 63) / 64), dim3(256), 0, s, W, mask, M, N, csums);
    hipLaunchKernelGGL(apply_col_threshold_kernel, dim3((N + 255) / 256, std::min(64, (M + 63) / 64)), dim3(256), 0, s, W, mask,
                       M, N, csums, th + 1, removed + 1);
    return hipGetLastError();
}

// ---- the same iteration with no allocation: scratch in a file-scope device array ----------------------------------
// Every device that loads the library holds its own copy of the array, at its own address, until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; the address that call returns for the
// current device is what the kernels get.
constexpr int kStaticMaxLines = 16384;   // largest M and largest N accepted
constexpr size_t kStaticScratchBytes = (size_t)2 * kStaticMaxLines * sizeof(double) + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

int prune_rows_cols_static_max_lines() { return kStaticMaxLines; }

// address of this device's copy of the array, looked up once per device with that device current
static hipError_t static_scratch_for_current_device(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

__global__ void copy_removed_kernel(const int* __restrict__ removed, int* __restrict__ out)
{
    if (threadIdx.x < 2) out[threadIdx.x] = removed[threadIdx.x];
}

// the caller has checked M, N <= kStaticMaxLines
hipError_t launch_prune_rows_cols_static(float* W, uint8_t* mask, int M, int N, unsigned k_rows, unsigned k_cols,
                                         int* removed_dev, hipStream_t s)
{
    if (prune_rows_cols_scratch_bytes(M, N) > kStaticScratchBytes) return hipErrorInvalidValue;
    void* ptr = nullptr;
    hipError_t e = static_scratch_for_current_device(&ptr);
    if (e != hipSuccess) return e;
    int* removed = nullptr;
    // the launcher clears the two counters with a fill kernel and overwrites every sum and threshold it reads,
    // so what the previous call left in the array does not matter
    e = launch_prune_rows_cols(W, mask, M, N, k_rows, k_cols, ptr, &removed, s);
    if (e != hipSuccess) return e;
    if (removed_dev) {
        hipLaunchKernelGGL(copy_removed_kernel, dim3(1), dim3(64), 0, s, removed, removed_dev);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace l355

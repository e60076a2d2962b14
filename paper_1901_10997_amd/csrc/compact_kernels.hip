// Dimension compaction after row/column pruning (paper Section 4, row/column growth & pruning: the pruning shrinks the
// dimensions of the weight matrices; Section 5.1 step (b): each control-gate matrix goes from 1500/400 to 1197/317).
// Rows and columns that have no active connection left leave the matrix; what remains is written out as a smaller
// dense matrix together with the lists of the rows and columns that were kept.
//
// Three kernels, nothing returns to the host between them: one pass over the mask sets a flag per row and per column
// that still has a connection; one workgroup turns the flags into ascending index lists (ballot + popcount per wave,
// wave totals through LDS); a gather writes the compacted matrix and mask.
#include "common.h"

namespace l355 {

// a workgroup covers 256 columns x 64 rows of the mask; every writer of a flag writes the same value
__global__ __launch_bounds__(256) void active_flags_kernel(const uint8_t* __restrict__ mask, int M, int N,
                                                           unsigned* __restrict__ rowflag, unsigned* __restrict__ colflag)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r0 = blockIdx.y * 64;
    const int r1 = r0 + 64 < M ? r0 + 64 : M;
    bool col_any = false;
    for (int r = r0; r < r1; ++r) {
        const bool on = c < N && mask[(size_t)r * N + c] != 0;
        col_any |= on;
        const unsigned long long b = __ballot(on);
        if (b != 0ull && (threadIdx.x & 63) == 0) rowflag[r] = 1u;
    }
    if (col_any) colflag[c] = 1u;
}

// out[0 .. total) = the indices i in [0, n) with keep(i), ascending; out[total .. n) = -1; *count = total
template <class Keep>
__device__ void ordered_indices(int n, Keep keep, int* __restrict__ out, int* __restrict__ count, int* wave_tot, int* base)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (threadIdx.x == 0) *base = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n; i0 += 1024) {
        const int i = i0 + (int)threadIdx.x;
        const bool on = i < n && keep(i);
        const unsigned long long b = __ballot(on);
        const int before = __popcll(b & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[wv] = __popcll(b);
        __syncthreads();
        int off = *base;
        for (int k = 0; k < wv; ++k) off += wave_tot[k];
        if (on) out[off + before] = i;
        __syncthreads();
        if (threadIdx.x == 0) {
            int t = 0;
            for (int k = 0; k < 16; ++k) t += wave_tot[k];
            *base += t;
        }
        __syncthreads();
    }
    const int total = *base;
    for (int i = total + (int)threadIdx.x; i < n; i += 1024) out[i] = -1;
    if (threadIdx.x == 0) *count = total;
    __syncthreads();
}

// one workgroup of 1024 threads; a unit is kept when any of its `gates` rows has a flag
__global__ __launch_bounds__(1024) void compact_index_kernel(const unsigned* __restrict__ rowflag, const unsigned* __restrict__ colflag,
                                                             int gates, int R, int N, int* __restrict__ row_index,
                                                             int* __restrict__ col_index, int* __restrict__ counts)
{
    __shared__ int wave_tot[16];
    __shared__ int base;
    ordered_indices(R, [&](int u) {
        unsigned any = 0u;
        for (int q = 0; q < gates; ++q) any |= rowflag[(size_t)q * R + u];
        return any != 0u;
    }, row_index, counts, wave_tot, &base);
    ordered_indices(N, [&](int k) { return colflag[k] != 0u; }, col_index, counts + 1, wave_tot, &base);
}

// Wc[q*Rc + i][j] = the value at (q*R + row_index[i], col_index[j]) where its mask byte is set, +0 otherwise
__global__ void compact_gather_kernel(const float* __restrict__ W, const uint8_t* __restrict__ mask, int gates, int R, int N,
                                      const int* __restrict__ row_index, const int* __restrict__ col_index,
                                      const int* __restrict__ counts, float* __restrict__ Wc, uint8_t* __restrict__ mask_c)
{
    const int Rc = counts[0], Nc = counts[1];
    const size_t total = (size_t)gates * Rc * Nc;
    for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(idx % (size_t)Nc);
        const size_t row = idx / (size_t)Nc;
        const int i = (int)(row % (size_t)Rc);
        const int q = (int)(row / (size_t)Rc);
        const size_t src = ((size_t)q * R + row_index[i]) * N + col_index[j];
        const bool on = mask[src] != 0;
        Wc[idx] = on ? W[src] : 0.f;
        if (mask_c) mask_c[idx] = on ? 1 : 0;
    }
}

// scratch: flags [gates*R + N] u32 (rounded up to an even count), then counts 2 x int
size_t compact_scratch_bytes(int gates, int R, int N)
{
    const size_t flags = ((size_t)gates * R + N + 1) & ~(size_t)1;
    return flags * sizeof(unsigned) + 2 * sizeof(int);
}

hipError_t launch_compact_rows_cols(const float* W, const uint8_t* mask, int gates, int R, int N, int* row_index,
                                    int* col_index, float* Wc, uint8_t* mask_c, void* scratch, int** counts_out, hipStream_t s)
{
    const int M = gates * R;
    const size_t flags = ((size_t)M + N + 1) & ~(size_t)1;
    unsigned* rowflag = (unsigned*)scratch;
    unsigned* colflag = rowflag + M;
    int* counts = (int*)(rowflag + flags);
    *counts_out = counts;
    hipError_t e = launch_fill_u64((unsigned long long*)scratch, flags / 2 + 1, 0ull, s);   // flags and both counts
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(active_flags_kernel, dim3((N + 255) / 256, (M + 63) / 64), dim3(256), 0, s, mask, M, N, rowflag, colflag);
    hipLaunchKernelGGL(compact_index_kernel, dim3(1), dim3(1024), 0, s, rowflag, colflag, gates, R, N, row_index, col_index, counts);
    size_t g = ((size_t)M * N + 255) / 256;
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL(compact_gather_kernel, dim3((unsigned)g), dim3(256), 0, s, W, mask, gates, R, N, row_index, col_index,
                       counts, Wc, mask_c);
    return hipGetLastError();
}

}  // namespace l355

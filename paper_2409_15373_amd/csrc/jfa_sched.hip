// Offsets-driven work scheduler: turns the jagged tensor's offsets array (paper Section 2) into a
// table of (sample, row-block) tiles, longest samples first, so that the persistent attention
// kernels hand out exactly the non-padded work and short samples leave no idle workgroups.
#include "jfa_common.h"

namespace jfa {

constexpr int kSchedThreads = 1024;

// Inclusive scan of one int per thread across the workgroup (kSchedThreads threads).
__device__ inline int block_inclusive_scan(int x, int *wave_sums) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) wave_sums[wave] = x;
    __syncthreads();
    if (wave == 0) {
        int s = lane < kSchedThreads / 64 ? wave_sums[lane] : 0;
        for (int d = 1; d < kSchedThreads / 64; d <<= 1) {
            const int y = __shfl_up(s, d, 64);
            if (lane >= d) s += y;
        }
        if (lane < kSchedThreads / 64) wave_sums[lane] = s;
    }
    __syncthreads();
    const int base = wave > 0 ? wave_sums[wave - 1] : 0;
    __syncthreads();
    return x + base;
}

// offsets_other (cross attention, else nullptr): the offsets of the rows that stream past a block.  Blocks are
// counted over `offsets`, but a block's cost grows with the length of the stream, so samples are ordered by that.
__global__ __launch_bounds__(kSchedThreads) void schedule_kernel(const int64_t *__restrict__ offsets,
                                                                 const int64_t *__restrict__ offsets_other, int B,
                                                                 int block_rows, int32_t *__restrict__ order,
                                                                 int32_t *__restrict__ tile_start,
                                                                 int32_t *__restrict__ counters, int n_counters) {
    __shared__ int hist[kSchedBins];    // samples per bin, then the bin's first position in `order`
    __shared__ int cursor[kSchedBins];  // next free slot of each bin
    __shared__ int wave_sums[kSchedThreads / 64];
    __shared__ int carry;
    const int tid = threadIdx.x;

    for (int i = tid; i < n_counters; i += kSchedThreads) counters[i] = 0;
    for (int i = tid; i < kSchedBins; i += kSchedThreads) { hist[i] = 0; cursor[i] = 0; }
    __syncthreads();

    // 1. histogram of the sort key: the row-block count of the stream (of the sample itself in self attention)
    auto sort_key = [&](int b) {
        const int64_t *o = offsets_other ? offsets_other : offsets;
        const int64_t key = (o[b + 1] - o[b] + block_rows - 1) / block_rows;
        return key < kSchedBins - 1 ? (int)key : kSchedBins - 1;
    };
    for (int b = tid; b < B; b += kSchedThreads) atomicAdd(&hist[sort_key(b)], 1);
    __syncthreads();

    // 2. bins in descending order: first position of bin i = number of samples in bins above i.
    //    Thread t scans bin (kSchedBins-1-t), so an exclusive prefix over t is a suffix sum over bins.
    {
        const int bin = kSchedBins - 1 - tid;
        const int cnt = hist[bin];
        const int incl = block_inclusive_scan(cnt, wave_sums);
        hist[bin] = incl - cnt;
    }
    __syncthreads();

    // 3. scatter samples to their bin; the per-sample block count is parked in tile_start[pos + 1]
    for (int b = tid; b < B; b += kSchedThreads) {
        const int64_t len = offsets[b + 1] - offsets[b];
        const int64_t nq = (len + block_rows - 1) / block_rows;
        const int bin = sort_key(b);
        const int pos = hist[bin] + atomicAdd(&cursor[bin], 1);
        order[pos] = b;
        tile_start[pos + 1] = (int)nq;
    }
    if (tid == 0) { tile_start[0] = 0; carry = 0; }
    __syncthreads();

    // 4. in-place inclusive scan of tile_start[1..B]
    for (int base = 0; base < B; base += kSchedThreads) {
        const int i = base + tid;
        const int x = i < B ? tile_start[i + 1] : 0;
        const int incl = block_inclusive_scan(x, wave_sums) + carry;
        if (i < B) tile_start[i + 1] = incl;
        __syncthreads();
        if (tid == kSchedThreads - 1) carry = incl;
        __syncthreads();
    }
}

__global__ void check_offsets_kernel(const int64_t *__restrict__ offsets, int B, int64_t max_len, int *flags) {
    int f = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0 && offsets[0] != 0) f |= 1;
    for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < B; b += gridDim.x * blockDim.x) {
        const int64_t len = offsets[b + 1] - offsets[b];
        if (len < 0) f |= 2;
        if (len > max_len) f |= 4;
    }
    if (f) atomicOr(flags, f);
}

hipError_t launch_schedule(const int64_t *offsets, const int64_t *offsets_other, int B, int block_rows, int32_t *order,
                           int32_t *tile_start, int32_t *counters, int n_counters, hipStream_t stream) {
    hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(kSchedThreads), 0, stream, offsets, offsets_other, B, block_rows, order,
                       tile_start, counters, n_counters);
    return hipGetLastError();
}

hipError_t launch_check_offsets(const int64_t *offsets, int B, int64_t max_len, int *flags, hipStream_t stream) {
    const int grid = B / 256 + 1 < 1024 ? B / 256 + 1 : 1024;
    hipLaunchKernelGGL(check_offsets_kernel, dim3(grid), dim3(256), 0, stream, offsets, B, max_len, flags);
    return hipGetLastError();
}

}  // namespace jfa

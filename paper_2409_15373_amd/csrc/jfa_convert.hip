// Jagged <-> padded-dense conversion (paper Section 2.2): dense[b, i] = values[offsets[b] + i] for i < L_b, the
// pad pattern otherwise; and back.  Pure data movement, bound by HBM: rows are opaque strings of 16-byte chunks.
//
// A two-dimensional grid: blockIdx.y walks the samples (offsets are read once per sample and workgroup, nothing is
// divided), blockIdx.x the sample's tiles of `rows` consecutive dense rows.  Inside a sample the data rows are a
// prefix, so a tile is all padding (a fill, or nothing to do on the way back), all data, or data followed by padding,
// and it is one contiguous block on the jagged side too.  All accesses are 16 bytes per lane on consecutive addresses,
// and every store covers whole 128-byte lines (a row is a multiple of 16 bytes; anything at or above 128 bytes per
// row keeps lines whole).
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kCvThreads = 256;

template <bool TO_DENSE>
__global__ __launch_bounds__(kCvThreads) void convert_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                             const int64_t *__restrict__ offsets, int B, int max_len,
                                                             int row_chunks, int rows, uint32_t pad) {
    const int tid = threadIdx.x;
    const u32x4 padv = {pad, pad, pad, pad};
    const int tiles_x = gridDim.x, samples_y = gridDim.y;
    for (int b = blockIdx.y; b < B; b += samples_y) {
        const int64_t s0 = offsets[b];
        const int L = (int)(offsets[b + 1] - s0);
        const int64_t dense0 = (int64_t)b * max_len;
        for (int i0 = blockIdx.x * rows; i0 < max_len; i0 += tiles_x * rows) {
            const int here = i0 + rows <= max_len ? rows : max_len - i0;                  // rows of this tile
            const int data = L - i0 < 0 ? 0 : (L - i0 < here ? L - i0 : here);           // ... of which the first hold data
            const int n = here * row_chunks, n_data = data * row_chunks;
            u32x4 *d = dst + (TO_DENSE ? dense0 + i0 : s0 + i0) * row_chunks;            // first chunk of the tile, output side
            const u32x4 *s = src + (TO_DENSE ? s0 + i0 : dense0 + i0) * row_chunks;      // ... and input side
            if (n_data == 0) {   // all padding
                if (TO_DENSE)
                    for (int id = tid; id < n; id += kCvThreads) d[id] = padv;
            } else if (n_data == n) {   // all data
#pragma unroll 4
                for (int id = tid; id < n; id += kCvThreads) d[id] = s[id];
            } else {   // the sample ends inside the tile
                for (int id = tid; id < (TO_DENSE ? n : n_data); id += kCvThreads) d[id] = id < n_data ? s[id] : padv;
            }
        }
    }
}

// Tile heights and grid sizes are measured choices (B = 512, max_len = 4096, 2 KB rows): towards dense, where most
// tiles are fills, small tiles and one workgroup per tile; back, where most tiles have nothing to do, larger tiles and
// fewer workgroups.  Narrow rows get taller tiles so that a tile still gives every thread a chunk or two.
hipError_t launch_convert(bool to_dense, const void *src, void *dst, const int64_t *offsets, int B, int64_t max_len,
                          int64_t row_chunks, uint32_t pad, int cus, hipStream_t stream) {
    if (B <= 0 || max_len <= 0) return hipSuccess;
    const int64_t chunks_per_tile = to_dense ? 512 : 1024;
    int64_t rows = (chunks_per_tile + row_chunks - 1) / row_chunks;
    if (rows < (to_dense ? 4 : 8)) rows = to_dense ? 4 : 8;
    if (rows > max_len) rows = max_len;
    const int64_t tiles = (max_len + rows - 1) / rows;
    const int gy = B < 32768 ? B : 32768;
    int64_t gx = ((int64_t)cus * (to_dense ? 4096 : 256) + gy - 1) / gy;   // workgroups in all: the loops take the rest
    if (gx > tiles) gx = tiles;
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)gy);
    if (to_dense)
        hipLaunchKernelGGL(convert_kernel<true>, grid, dim3(kCvThreads), 0, stream, (const u32x4 *)src, (u32x4 *)dst,
                           offsets, B, (int)max_len, (int)row_chunks, (int)rows, pad);
    else
        hipLaunchKernelGGL(convert_kernel<false>, grid, dim3(kCvThreads), 0, stream, (const u32x4 *)src, (u32x4 *)dst,
                           offsets, B, (int)max_len, (int)row_chunks, (int)rows, pad);
    return hipGetLastError();
}

}  // namespace jfa

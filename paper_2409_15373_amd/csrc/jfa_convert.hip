// Jagged <-> padded-dense conversion (paper Section 2.2): dense[b, i] = values[offsets[b] + i] for i < L_b, the
// pad pattern otherwise; and back.  Pure data movement, bound by HBM: rows are opaque strings of 16-byte chunks.
//
// Both directions walk the DENSE tensor in tiles of 8 consecutive rows (flat row id b * max_len + i), one tile
// per workgroup step.  A tile that lies inside one sample is either all padding (a fill, or nothing to do on the
// way back), or all data -- then it is one contiguous block on the jagged side too, because a sample's rows are
// consecutive -- or it holds the sample's end; only the last kind and tiles that cross into the next sample look
// at offsets per chunk.  All accesses are 16 bytes per lane on consecutive addresses, and every store covers whole
// 128-byte lines (a row is a multiple of 16 bytes; anything at or above 128 bytes per row keeps lines whole).
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kCvThreads = 256;
constexpr int kCvRows = 8;

template <bool TO_DENSE>
__global__ __launch_bounds__(kCvThreads) void convert_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                             const int64_t *__restrict__ offsets, int B, int max_len,
                                                             int row_chunks, uint32_t pad) {
    const int tid = threadIdx.x;
    const int64_t n_rows = (int64_t)B * max_len;
    const int n = kCvRows * row_chunks;   // chunks per tile
    const u32x4 padv = {pad, pad, pad, pad};
    for (int64_t r0 = (int64_t)blockIdx.x * kCvRows; r0 < n_rows; r0 += (int64_t)gridDim.x * kCvRows) {
        const int b0 = (int)(r0 / max_len);
        const int i0 = (int)(r0 - (int64_t)b0 * max_len);
        const int64_t s0 = offsets[b0];
        const int64_t L0 = offsets[b0 + 1] - s0;
        u32x4 *d = dst + (TO_DENSE ? r0 : s0 + i0) * row_chunks;         // first chunk of the tile on the output side
        const u32x4 *s = src + (TO_DENSE ? s0 + i0 : r0) * row_chunks;   // ... and on the input side (if it is all data)
        if (i0 + kCvRows <= max_len && i0 >= L0) {   // all padding
            if (TO_DENSE)
                for (int id = tid; id < n; id += kCvThreads) d[id] = padv;
        } else if (i0 + kCvRows <= max_len && i0 + kCvRows <= L0) {   // all data: a contiguous block on both sides
#pragma unroll 4
            for (int id = tid; id < n; id += kCvThreads) d[id] = s[id];
        } else {   // a sample ends inside the tile, or the tile crosses into the next sample(s)
            for (int id = tid; id < n; id += kCvThreads) {
                const int dr = id / row_chunks, k = id - dr * row_chunks;
                if (r0 + dr >= n_rows) break;
                int b = b0, i = i0 + dr;
                while (i >= max_len) { i -= max_len; ++b; }
                const int64_t sb = offsets[b];
                const bool data = i < offsets[b + 1] - sb;
                if (TO_DENSE) dst[(r0 + dr) * row_chunks + k] = data ? src[(sb + i) * row_chunks + k] : padv;
                else if (data) dst[(sb + i) * row_chunks + k] = src[(r0 + dr) * row_chunks + k];
            }
        }
    }
}

hipError_t launch_convert(bool to_dense, const void *src, void *dst, const int64_t *offsets, int B, int64_t max_len,
                          int64_t row_chunks, uint32_t pad, int cus, hipStream_t stream) {
    const int64_t tiles = ((int64_t)B * max_len + kCvRows - 1) / kCvRows;
    const int64_t cap = (int64_t)cus * 64;   // enough workgroups in flight to hide latency; the loop takes the rest
    const int grid = (int)(tiles < cap ? (tiles > 0 ? tiles : 1) : cap);
    if (to_dense)
        hipLaunchKernelGGL(convert_kernel<true>, dim3(grid), dim3(kCvThreads), 0, stream, (const u32x4 *)src, (u32x4 *)dst,
                           offsets, B, (int)max_len, (int)row_chunks, pad);
    else
        hipLaunchKernelGGL(convert_kernel<false>, dim3(grid), dim3(kCvThreads), 0, stream, (const u32x4 *)src, (u32x4 *)dst,
                           offsets, B, (int)max_len, (int)row_chunks, pad);
    return hipGetLastError();
}

}  // namespace jfa

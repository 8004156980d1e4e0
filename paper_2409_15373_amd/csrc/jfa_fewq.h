// Pieces shared by the two kernels for cross attention with few queries per sample (at most 32, D = 128): a work
// item is a (sample, head), a workgroup is four waves (one per SIMD), and each wave works on blocks of 32 keys whose
// K and V rows it copies into LDS buffers of its own.  Not part of the C ABI.
#pragma once
#include "jfa_bwd_dma.h"

namespace jfa {

constexpr int kFqThreads = 256;
constexpr int kFqWaves = kFqThreads / 64;
constexpr int kFqRows = kFewqRows;               // queries per item (at most), keys per block
constexpr int kFqTile = kFqRows * kBdD * 2;      // bytes of 32 rows
constexpr int kFqKSteps = kBdD / 16;
constexpr int kFqDBlocks = kBdD / 32;

// A lane's place in the 32 x 32 matrix instructions and its LDS read addresses inside a 32-row tile (row r, 16-byte
// chunk ch at r * 256 + ((ch ^ swz(r)) << 4)).
struct FqLane {
    int lane, col, half;
    int raddr[kFqKSteps];       // row reads: this lane's row `col`, chunk 2 ks + half
    int taddr[2][kFqDBlocks];   // transposing reads: row = 4 half + (lane & 15) / 4 (+8 for the operand's second half)
    __device__ FqLane() {
        lane = threadIdx.x & 63;
        col = lane & 31;
        half = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < kFqKSteps; ++ks) raddr[ks] = col * 256 + (((2 * ks + half) ^ swz(col)) << 4);
        const int r = half * 4 + ((lane & 15) >> 2);
        const int chunk_in_group = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1), byte_in_chunk = (lane & 1) * 8;
        const int t0 = r * 256 + ((chunk_in_group ^ swz(r)) << 4) + byte_in_chunk;
#pragma unroll
        for (int db = 0; db < kFqDBlocks; ++db) {
            taddr[0][db] = t0 ^ (db << 6);
            taddr[1][db] = (t0 ^ (db << 6) ^ 32) + 2048;
        }
    }
    // copy of 32 rows (8 KB) by one wave: eight instructions of four rows each; rows past `valid` repeat the last one
    __device__ void copy_rows(const __bf16 *base, int row_stride, int valid, char *tile) const {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = 4 * u + (lane >> 4);
            const int rr = r < valid ? r : valid - 1;
            bd_dma16(base, 2u * (uint32_t)(rr * row_stride + (((lane & 15) ^ swz(r)) << 3)), tile + u * 1024);
        }
    }
    // this lane's operand registers of a tile: its row `col`, the halves of every 16-feature step
    __device__ void fragments(const char *tile, bf16x8 (&f)[kFqKSteps]) const {
#pragma unroll
        for (int ks = 0; ks < kFqKSteps; ++ks) f[ks] = lds_read_b128(tile + raddr[ks]);
    }
    // g^T += (tile)^T x, contraction over the tile's 32 rows in two steps of 16
    __device__ void accumulate(const char *tile, const f32x16 &x, f32x16 (&g)[kFqDBlocks]) const {
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
            const bf16x8 xb = pack_bf16(x, 8 * ts);
            bf16x8 top[kFqDBlocks];
#pragma unroll
            for (int db = 0; db < kFqDBlocks; ++db) {
                const char *base = tile + ts * 16 * 256;
                top[db] = concat(lds_read_tr16(base + taddr[0][db]), lds_read_tr16(base + taddr[1][db]));
            }
#pragma unroll
            for (int db = 0; db < kFqDBlocks; ++db) g[db] = mfma_32x32x16(top[db], xb, g[db]);
        }
    }
};

// acc[row of a][lane of b] += a . b over the 128 features
__device__ inline void fq_product(const bf16x8 (&a)[kFqKSteps], const bf16x8 (&b)[kFqKSteps], f32x16 &acc) {
#pragma unroll
    for (int ks = 0; ks < kFqKSteps; ++ks) acc = mfma_32x32x16(a[ks], b[ks], acc);
}

}  // namespace jfa

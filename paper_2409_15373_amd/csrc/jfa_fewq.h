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

// The walk of a workgroup through the work items ((sample, head) pairs: item w = position w / H of the schedule's
// sample order, head w % H), kept ONE ITEM AHEAD of the work by thread 0 so that neither the claim nor the decoding
// of an item -- an atomic and two dependent loads, microseconds for items that may hold a block or two of keys --
// is waited for: while item i is worked on, the parameters of item i + 1 are fetched and left in `slot[(i + 1) & 1]`,
// and the work id of item i + 2 is requested.  The first item of a workgroup is its own index; further ids are
// tickets from one work counter (items are independent of each other: nothing is gained by keeping neighbours on
// one die), or, without a schedule (sched.static_only), every gridDim-th item.
struct FqSlot {
    int valid;   // 0: no such item, the workgroup is done
    int sample, head, Lq, Lk;
    int q0_lo, q0_hi, k0_lo, k0_hi;   // first query row and first key row of the sample
};
struct FqAhead {       // thread 0's registers
    int64_t w1 = 0;    // work id of the item after the current one
    int64_t w2 = 0;    // and of the one after that (requested; its arrival is waited for an item later)
    int b1 = 0;        // sample of item w1
    int64_t q0 = 0, q1 = 0, k0 = 0, k1 = 0;   // its offsets
};
__device__ inline int64_t fq_next_id(const Schedule &sched, int64_t after) {
    return sched.static_only ? after + (int64_t)gridDim.x : (int64_t)gridDim.x + atomicAdd(sched.counter, 1);
}
__device__ inline int fq_sample_of(const Schedule &sched, int64_t w, int H) {
    const int pos = (int)(w / H);
    return sched.order ? sched.order[pos] : pos;
}
__device__ inline void fq_store_slot(FqSlot *slot, bool valid, int b, int head, int64_t q0, int64_t q1, int64_t k0, int64_t k1) {
    slot->valid = valid ? 1 : 0;
    slot->sample = b;
    slot->head = head;
    slot->Lq = (int)(q1 - q0);
    slot->Lk = (int)(k1 - k0);
    slot->q0_lo = (int)(uint32_t)q0;
    slot->q0_hi = (int)(uint32_t)((uint64_t)q0 >> 32);
    slot->k0_lo = (int)(uint32_t)k0;
    slot->k0_hi = (int)(uint32_t)((uint64_t)k0 >> 32);
}
// thread 0, before the first item: the workgroup's own item into slot[0], and the id of the one after it
__device__ inline void fq_walk_begin(FqAhead &a, FqSlot *slot, const Schedule &sched, const int64_t *offsets_q,
                                     const int64_t *offsets_kv, int H, int64_t total) {
    const int64_t w0 = blockIdx.x;
    if (w0 < total) {
        const int b = fq_sample_of(sched, w0, H);
        fq_store_slot(&slot[0], true, b, (int)(w0 % H), offsets_q[b], offsets_q[b + 1], offsets_kv[b], offsets_kv[b + 1]);
    } else {
        slot[0].valid = 0;
    }
    a.w1 = fq_next_id(sched, w0);
}
// thread 0, at the start of an item: request the id of the item two ahead, start decoding the next one
__device__ inline void fq_walk_ahead(FqAhead &a, const Schedule &sched, int H, int64_t total) {
    a.w2 = fq_next_id(sched, a.w1);
    if (a.w1 < total) a.b1 = fq_sample_of(sched, a.w1, H);
}
// thread 0, somewhat later (the sample's index has arrived by then): its offsets
__device__ inline void fq_walk_offsets(FqAhead &a, const int64_t *offsets_q, const int64_t *offsets_kv, int64_t total) {
    if (a.w1 < total) {
        a.q0 = offsets_q[a.b1]; a.q1 = offsets_q[a.b1 + 1];
        a.k0 = offsets_kv[a.b1]; a.k1 = offsets_kv[a.b1 + 1];
    }
}
// thread 0, at the end of item `it`: leave the next item's parameters for the whole workgroup, move on by one
__device__ inline void fq_walk_publish(FqAhead &a, FqSlot *slot, int it, int H, int64_t total) {
    fq_store_slot(&slot[(it + 1) & 1], a.w1 < total, a.b1, (int)(a.w1 % H), a.q0, a.q1, a.k0, a.k1);
    a.w1 = a.w2;
}

// acc[row of a][lane of b] += a . b over the 128 features
__device__ inline void fq_product(const bf16x8 (&a)[kFqKSteps], const bf16x8 (&b)[kFqKSteps], f32x16 &acc) {
#pragma unroll
    for (int ks = 0; ks < kFqKSteps; ++ks) acc = mfma_32x32x16(a[ks], b[ks], acc);
}

}  // namespace jfa

// Jagged flash attention backward, bf16, D = 128, cross attention with FEW QUERIES per sample (at most 32: a sample's
// target items against its long list of feature values, paper Section 2): dQ, dK and dV in ONE pass over K and V.
//
//   P = exp(S / sqrt(D) - lse),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = dS K / sqrt(D),  dK = dS^T Q / sqrt(D)
//
// With so few queries the matrix work per key is tiny and the operation is bound by reading K and V and writing dK
// and dV once (4 x sum_Bkv x H x D x 2 bytes); the kernels for long query lists read K and V in two passes, in tiles
// whose start-up costs more than their work.  Here a work item is a (sample, head); its queries' Q and dO rows sit in
// LDS for the whole item, and each of the workgroup's four waves (one per SIMD, so each has 512 registers) takes
// blocks of 32 keys on its own: it copies the block's K and V rows into its private part of LDS (global_load_lds, two
// buffers: the next block's rows are in flight while this block is computed), and computes everything those keys need.
// Matrix work is free here, so the score block is computed in BOTH orientations instead of being transposed:
//   keys on the MFMA row axis, queries on the lanes:   S, dP, dS with a query per lane, in operand position for
//                                                      dQ^T += K^T dS^T (accumulated over the wave's blocks);
//   queries on the row axis, keys on the lanes:        S, dP, dS, P with a key per lane, in operand position for
//                                                      dV^T = dO^T P and dK^T = Q^T dS, which are complete after the
//                                                      block (the contraction runs over the item's queries) and
//                                                      leave at once through an LDS transpose as whole row pieces.
// A lane's operand registers are the same in both orientations (its own row of the tile, read once per block for K
// and V and once per item for Q and dO): only which side of the matrix instruction they go to differs.
// The waves' partial dQ blocks are added in a fixed order through LDS at the end of the item: results are
// deterministic.  The kernel also writes both planes of the statistics buffer (delta = rowsum(dO o O), -lse * sqrt(D)).
// Work items are taken by the persistent workgroups, by tickets from a work counter, in the order of a schedule
// that lists the samples by their number of key blocks, longest first (item w = position w / H of that list, head
// w % H), so that the samples with thousands of keys do not end up on a few workgroups, and are decoded one item ahead
// of the work (FqAhead); a problem of at most four items per workgroup is dealt in turn in sample order, with no
// schedule.  Every sample is visited, so samples without queries get their dK = dV = 0 and samples without keys
// their dQ = 0.
#include "jfa_fewq.h"

namespace jfa {

constexpr int kFqStores = 16;                    // global store instructions of one full block (dK and dV, 8 KB each)

__global__ __launch_bounds__(kFqThreads) void bwd_cross_fewq_kernel(const __bf16 *__restrict__ q,
                                                                    const __bf16 *__restrict__ k,
                                                                    const __bf16 *__restrict__ v,
                                                                    const __bf16 *__restrict__ out_fwd,
                                                                    const __bf16 *__restrict__ dout,
                                                                    const float *__restrict__ lse,
                                                                    float *__restrict__ stats,   // [2, H, sum_Bq]
                                                                    const int64_t *__restrict__ offsets_q,
                                                                    const int64_t *__restrict__ offsets_kv, int B, int H,
                                                                    Schedule sched,
                                                                    __bf16 *__restrict__ dq, __bf16 *__restrict__ dk,
                                                                    __bf16 *__restrict__ dv) {
    constexpr int D = kBdD;
    constexpr int kKSteps = D / 16;
    constexpr int kDBlocks = D / 32;
    __shared__ __attribute__((aligned(1024))) char Qt[kFqTile];    // the item's Q rows (rows past the last query repeat it)
    __shared__ __attribute__((aligned(1024))) char Ot[kFqTile];    // the item's dO rows
    __shared__ __attribute__((aligned(1024))) char KV[kFqWaves][2][2 * kFqTile];   // per wave, two buffers: a block's K rows, then its V rows
    __shared__ __attribute__((aligned(16))) float row_lse2[kFqRows];            // -lse * sqrt(D) per query
    __shared__ __attribute__((aligned(16))) float row_delta[kFqRows];           // delta per query
    __shared__ FqSlot slot[2];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const FqLane ln;
    const int lane = ln.lane, col = ln.col, half = ln.half;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    const int64_t sum_Bq = offsets_q[B];
    const int64_t row_stride = (int64_t)H * D;
    auto copy_rows = [&](const __bf16 *base, int valid, char *tile) { ln.copy_rows(base, (int)row_stride, valid, tile); };
    auto fragments = [&](const char *tile, bf16x8 (&f)[kKSteps]) { ln.fragments(tile, f); };
    auto product = [&](const bf16x8 (&a)[kKSteps], const bf16x8 (&b)[kKSteps], f32x16 &acc) { fq_product(a, b, acc); };
    auto accumulate = [&](const char *tile, const f32x16 &x, f32x16 (&g)[kDBlocks]) { ln.accumulate(tile, x, g); };
    // One half (64 features: d-blocks 2 f and 2 f + 1) of a 128 x 32 gradient block that is complete after one block of
    // keys: g^T = (tile)^T x over the tile's 32 rows, scaled, transposed through 4 KB of LDS and stored as whole
    // 128-byte pieces of rows (this lane's column = row `col` of the result; rows >= valid are not stored).  Half a
    // block at a time keeps its accumulators at 32 registers.
    auto finish_half = [&](const char *tile, const f32x16 &x, int f, float out_scale, char *region, __bf16 *gbase, int valid) {
        f32x16 g[2];
#pragma unroll
        for (int dl = 0; dl < 2; ++dl)
#pragma unroll
            for (int e = 0; e < 16; ++e) g[dl][e] = 0.0f;
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
            const bf16x8 xb = pack_bf16(x, 8 * ts);
            bf16x8 top[2];
#pragma unroll
            for (int dl = 0; dl < 2; ++dl) {
                const char *base = tile + ts * 16 * 256;
                top[dl] = concat(lds_read_tr16(base + ln.taddr[0][2 * f + dl]), lds_read_tr16(base + ln.taddr[1][2 * f + dl]));
            }
#pragma unroll
            for (int dl = 0; dl < 2; ++dl) g[dl] = mfma_32x32x16(top[dl], xb, g[dl]);
        }
        const int wbase = col * 128 + ((half * 8) ^ ((col & 7) << 4));
        const uint32_t lane_off = 2u * (uint32_t)((lane >> 3) * (int)row_stride + (lane & 7) * 8);
#pragma unroll
        for (int dl = 0; dl < 2; ++dl)
#pragma unroll
            for (int gq4 = 0; gq4 < 4; ++gq4) {
                bf16x4 y;
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = (__bf16)(g[dl][4 * gq4 + e] * out_scale);
                *reinterpret_cast<bf16x4 *>(region + (wbase ^ (dl * 64 + gq4 * 16))) = y;
            }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = it * 8 + (lane >> 3);
            const u32x4 rowpiece = *reinterpret_cast<const u32x4 *>(region + r * 128 + (((lane & 7) ^ (r & 7)) << 4));
            char *dst = reinterpret_cast<char *>(gbase + (int64_t)it * 8 * row_stride + 64 * f) + lane_off;
            if (r < valid) *reinterpret_cast<u32x4 *>(dst) = rowpiece;
        }
    };

    const int64_t total = (int64_t)B * H;
    FqAhead ahead;   // thread 0's
    if (tid == 0) fq_walk_begin(ahead, slot, sched, offsets_q, offsets_kv, H, total);
    for (int it = 0;; ++it) {
        __syncthreads();   // this item's slot is written; the previous item's reads of the shared tiles and partial sums are done
        const FqSlot *const item = &slot[it & 1];
        if (__builtin_amdgcn_readfirstlane(item->valid) == 0) break;
        const int head = __builtin_amdgcn_readfirstlane(item->head);
        const int Lq = __builtin_amdgcn_readfirstlane(item->Lq), Lk = __builtin_amdgcn_readfirstlane(item->Lk);
        const int64_t q0 = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(item->q0_hi) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(item->q0_lo));
        const int64_t k0 = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(item->k0_hi) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(item->k0_lo));
        const int n_blocks = (Lk + kFqRows - 1) / kFqRows;
        if (tid == 0) fq_walk_ahead(ahead, sched, H, total);
        auto walk_on_at_once = [&]() {   // an item without blocks to hide the loads behind
            if (tid == 0) {
                fq_walk_offsets(ahead, offsets_q, offsets_kv, total);
                fq_walk_publish(ahead, slot, it, H, total);
            }
        };
        if (Lq == 0) {     // no query attends to these keys: their gradients are zero
            for (int blk = wave; blk < n_blocks; blk += kFqWaves) {
                const int j = blk * kFqRows + col;
                if (j < Lk) {
                    const int64_t off = (k0 + j) * row_stride + (int64_t)head * D + half * (D / 2);
#pragma unroll
                    for (int e = 0; e < D / 2; e += 8) {
                        *reinterpret_cast<u32x4 *>(dk + off + e) = u32x4{0, 0, 0, 0};
                        *reinterpret_cast<u32x4 *>(dv + off + e) = u32x4{0, 0, 0, 0};
                    }
                }
            }
            walk_on_at_once();
            continue;
        }
        const __bf16 *const kbase = k + k0 * row_stride + (int64_t)head * D;
        const __bf16 *const vbase = v + k0 * row_stride + (int64_t)head * D;
        auto fetch_block = [&](int blk, int buf) {   // K and V rows of block `blk` into this wave's buffer `buf`
            const int j0 = blk * kFqRows;
            const int valid = Lk - j0 < kFqRows ? Lk - j0 : kFqRows;
            copy_rows(kbase + j0 * row_stride, valid, KV[wave][buf]);
            copy_rows(vbase + j0 * row_stride, valid, KV[wave][buf] + kFqTile);
        };
        // ---- the item's queries: Q and dO rows into LDS (waves 0 and 1), statistics (wave 2); every wave's first block ----
        const __bf16 *const qbase = q + q0 * row_stride + (int64_t)head * D;
        const __bf16 *const obase = dout + q0 * row_stride + (int64_t)head * D;
        if (wave == 0) copy_rows(qbase, Lq, Qt);
        if (wave == 1) copy_rows(obase, Lq, Ot);
        if (wave < n_blocks) fetch_block(wave, 0);
        if (wave == 2) {   // delta = rowsum(dO o O) and -lse * sqrt(D): two lanes per query, 64 features each
            const int i = col < Lq ? col : Lq - 1;
            float dot = 0.0f, nl = INFINITY;   // a sample without keys: out = 0, lse = -inf
            if (Lk > 0) {
                const int64_t off = (q0 + i) * row_stride + (int64_t)head * D + half * (D / 2);
#pragma unroll
                for (int e = 0; e < D / 2; e += 8) {
                    const bf16x8 o = *reinterpret_cast<const bf16x8 *>(out_fwd + off + e);
                    const bf16x8 g = *reinterpret_cast<const bf16x8 *>(dout + off + e);
#pragma unroll
                    for (int x = 0; x < 8; ++x) dot = fmaf((float)o[x], (float)g[x], dot);
                }
                dot = pair_sum(dot);
                nl = -lse[(int64_t)head * sum_Bq + q0 + i] * sqrtf((float)D);
            }
            if (half == 0) {
                row_delta[col] = dot;
                row_lse2[col] = nl;
                if (col < Lq) {
                    stats[(int64_t)head * sum_Bq + q0 + col] = dot;
                    stats[(int64_t)(H + head) * sum_Bq + q0 + col] = nl;
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0070);   // this wave's copies have landed
        __syncthreads();                      // the tiles and the statistics are there for every wave
        if (Lk == 0) {     // nothing to attend to: dQ = 0
            if (wave == 0 && col < Lq) {
                const int64_t off = (q0 + col) * row_stride + (int64_t)head * D + half * (D / 2);
#pragma unroll
                for (int e = 0; e < D / 2; e += 8) *reinterpret_cast<u32x4 *>(dq + off + e) = u32x4{0, 0, 0, 0};
            }
            walk_on_at_once();
            continue;
        }
        if (tid == 0) fq_walk_offsets(ahead, offsets_q, offsets_kv, total);   // in flight during the item's blocks
        // per item: the lane's operand registers of Q and dO, and the statistics in both orientations
        bf16x8 Qf[kKSteps], Of[kKSteps];
        fragments(Qt, Qf);
        fragments(Ot, Of);
        const float my_lse2 = row_lse2[col], my_delta = row_delta[col];   // this lane's query (a query per lane)
        f32x16 rows_lse2, rows_delta;                                     // the accumulator rows' queries (a key per lane)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 l4 = *reinterpret_cast<const float4 *>(&row_lse2[g * 8 + half * 4]);
            rows_lse2[4 * g] = l4.x; rows_lse2[4 * g + 1] = l4.y; rows_lse2[4 * g + 2] = l4.z; rows_lse2[4 * g + 3] = l4.w;
            const float4 d4 = *reinterpret_cast<const float4 *>(&row_delta[g * 8 + half * 4]);
            rows_delta[4 * g] = -d4.x; rows_delta[4 * g + 1] = -d4.y; rows_delta[4 * g + 2] = -d4.z; rows_delta[4 * g + 3] = -d4.w;
        }
        f32x16 gq[kDBlocks];   // dQ^T of this wave's blocks
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) gq[db][e] = 0.0f;

        int buf = 0;
        for (int blk = wave; blk < n_blocks; blk += kFqWaves, buf ^= 1) {
            const int j0 = blk * kFqRows;
            const int valid = Lk - j0 < kFqRows ? Lk - j0 : kFqRows;   // keys of this block
            char *const Kt = KV[wave][buf], *const Vt = KV[wave][buf] + kFqTile;
            // This block's rows have landed: they were requested a block ago (or at the item's start), and the only
            // memory instructions issued since are the previous block's kFqStores stores, which need not be waited
            // for (memory instructions complete in order; the previous block was a full one, since only an item's
            // last block is ragged).  All LDS reads of the other buffer are done, so the next block's rows may go there.
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(kFqStores) : "memory");
            if (blk + kFqWaves < n_blocks) fetch_block(blk + kFqWaves, buf ^ 1);
            bf16x8 Kf[kKSteps], Vf[kKSteps];
            fragments(Kt, Kf);
            fragments(Vt, Vf);

            // ---- keys on the row axis, a query per lane: dQ^T += K^T dS^T ----
            {
                f32x16 s, dp;
#pragma unroll
                for (int e = 0; e < 16; ++e) { s[e] = my_lse2; dp[e] = -my_delta; }
                product(Kf, Qf, s);     // q . k - lse * sqrt(D)
                product(Vf, Of, dp);    // dO . v - delta
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float p = fast_exp2(s[e] * c);
                    if ((e >> 2) * 8 + half * 4 + (e & 3) >= valid) p = 0.0f;   // a key past the sample's end
                    dp[e] = p * dp[e];   // dS
                }
                accumulate(Kt, dp, gq);
            }
            // ---- queries on the row axis, a key per lane: dV^T = dO^T P, dK^T = Q^T dS, complete after this block ----
            {
                f32x16 s = rows_lse2, dp = rows_delta;
                product(Qf, Kf, s);
                product(Of, Vf, dp);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float p = fast_exp2(s[e] * c);
                    if ((e >> 2) * 8 + half * 4 + (e & 3) >= Lq) p = 0.0f;   // a row past the last query
                    s[e] = p;
                    dp[e] = p * dp[e];
                }
                // K and V of the block are no longer read: the K rows' place serves the transposes
                __bf16 *const dv_rows = dv + (k0 + j0) * row_stride + (int64_t)head * D;
                __bf16 *const dk_rows = dk + (k0 + j0) * row_stride + (int64_t)head * D;
                finish_half(Ot, s, 0, 1.0f, Kt, dv_rows, valid);
                finish_half(Ot, s, 1, 1.0f, Kt, dv_rows, valid);
                finish_half(Qt, dp, 0, scale, Kt, dk_rows, valid);
                finish_half(Qt, dp, 1, scale, Kt, dk_rows, valid);
            }
        }
        // ---- dQ: the waves' partial blocks, added in wave order (wave w leaves its block in its own first buffer as
        // fp32 [feature][query], 16 KB; no copy is in flight: the last block requested none) ----
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);
        {
            float *part = reinterpret_cast<float *>(KV[wave][0]);   // [feature d][query], 128 x 32 floats
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int d = db * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                    part[d * kFqRows + col] = gq[db][e];
                }
        }
        __syncthreads();
        {   // thread t sums elements (query t % 32, features 16 (t / 32) .. + 15) over the waves that had blocks
            const int qi = tid & 31, d0 = (tid >> 5) * 16;
            float sum[16];
#pragma unroll
            for (int x = 0; x < 16; ++x) sum[x] = 0.0f;
            const int n_parts = n_blocks < kFqWaves ? n_blocks : kFqWaves;
            for (int pw = 0; pw < n_parts; ++pw) {
                const float *part = reinterpret_cast<const float *>(KV[pw][0]);
#pragma unroll
                for (int x = 0; x < 16; ++x) sum[x] += part[(d0 + x) * kFqRows + qi];
            }
            if (qi < Lq) {
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8) {
                    bf16x8 o;
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[x] = (__bf16)(sum[8 * h8 + x] * scale);
                    *reinterpret_cast<bf16x8 *>(dq + (q0 + qi) * row_stride + (int64_t)head * D + d0 + 8 * h8) = o;
                }
            }
        }
        if (tid == 0) fq_walk_publish(ahead, slot, it, H, total);
    }
}

hipError_t launch_bwd_cross_fewq(const void *q, const void *k, const void *v, const void *out, const void *dout,
                                 const float *lse, float *stats, const int64_t *offsets_q, const int64_t *offsets_kv, int B,
                                 int H, int D, Schedule sched, void *dq, void *dk, void *dv, int cus, hipStream_t stream) {
    if (D != kBdD) return hipErrorInvalidValue;
    hipLaunchKernelGGL(bwd_cross_fewq_kernel, dim3(persistent_grid<bwd_cross_fewq_kernel>(kFqThreads, cus)), dim3(kFqThreads), 0,
                       stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, (const __bf16 *)out,
                       (const __bf16 *)dout, lse, stats, offsets_q, offsets_kv, B, H, sched, (__bf16 *)dq, (__bf16 *)dk, (__bf16 *)dv);
    return hipGetLastError();
}

}  // namespace jfa

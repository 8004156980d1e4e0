// Jagged flash attention forward, bf16, D = 128, cross attention with FEW QUERIES per sample (at most 32: a sample's
// target items against its long list of feature values, paper Section 2).
//
//   out = softmax(Q K^T / sqrt(D)) V,   lse = log sum_j exp(q . k_j / sqrt(D))
//
// With so few queries the operation is bound by reading K and V once.  The kernel for long query lists gives such a
// sample one tile of 256 queries, of which one wave has work, and pays a tile's start-up for every (sample, head);
// here a work item is a (sample, head) whose Q rows (8 KB) sit in LDS and, as operand registers, in every lane, and
// each of the workgroup's four waves (one per SIMD) takes blocks of 32 keys on its own: it copies the block's K and V
// rows into one of its two private LDS buffers (global_load_lds; the next block's rows are in flight while this one
// is computed), forms S^T = K Q^T (keys on the MFMA row axis, a query per lane), keeps a running maximum and sum
// per query (online softmax, Section 2.1) and adds V^T P^T to its partial output.  At the end of the item the waves'
// partial results (maximum, sum, output block) are merged in wave order through LDS: results are deterministic.
// Work items are taken as in the few-query backward kernel: samples with the longest key lists first, by tickets from
// a work counter, and decoded one item ahead of the work (FqAhead); a problem of at most four items per workgroup is
// dealt in turn in sample order.
#include "jfa_fewq.h"

namespace jfa {

__global__ __launch_bounds__(kFqThreads) void fwd_cross_fewq_kernel(const __bf16 *__restrict__ q,
                                                                    const __bf16 *__restrict__ k,
                                                                    const __bf16 *__restrict__ v,
                                                                    const int64_t *__restrict__ offsets_q,
                                                                    const int64_t *__restrict__ offsets_kv, int B, int H,
                                                                    Schedule sched, __bf16 *__restrict__ out,
                                                                    float *__restrict__ lse) {
    constexpr int D = kBdD;
    __shared__ __attribute__((aligned(1024))) char Qt[kFqTile];    // the item's Q rows (rows past the last query repeat it)
    __shared__ __attribute__((aligned(1024))) char KV[kFqWaves][2][2 * kFqTile];   // per wave, two buffers: a block's K rows, then its V rows
    __shared__ float part_m[kFqWaves][kFqRows];   // per wave and query: maximum of the raw dot products of its blocks
    __shared__ float part_l[kFqWaves][kFqRows];   //                     sum of its probabilities against that maximum
    __shared__ FqSlot slot[2];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const FqLane ln;
    const int col = ln.col, half = ln.half;
    const float c = 1.4426950408889634f / sqrtf((float)D);
    const int64_t sum_Bq = offsets_q[B];
    const int64_t row_stride = (int64_t)H * D;

    const int64_t total = (int64_t)B * H;
    FqAhead ahead;   // thread 0's
    if (tid == 0) fq_walk_begin(ahead, slot, sched, offsets_q, offsets_kv, H, total);
    for (int it = 0;; ++it) {
        __syncthreads();   // this item's slot is written; the previous item's reads of the Q tile and the partial results are done
        const FqSlot *const item = &slot[it & 1];
        if (__builtin_amdgcn_readfirstlane(item->valid) == 0) break;
        const int head = __builtin_amdgcn_readfirstlane(item->head);
        const int Lq = __builtin_amdgcn_readfirstlane(item->Lq), Lk = __builtin_amdgcn_readfirstlane(item->Lk);
        const int64_t q0 = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(item->q0_hi) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(item->q0_lo));
        const int64_t k0 = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(item->k0_hi) << 32) | (uint32_t)__builtin_amdgcn_readfirstlane(item->k0_lo));
        const int n_blocks = (Lk + kFqRows - 1) / kFqRows;
        if (tid == 0) fq_walk_ahead(ahead, sched, H, total);
        if (Lq == 0 || Lk == 0) {
            if (Lq > 0 && wave == 0 && col < Lq) {   // no keys: an empty softmax, out = 0 and lse = -inf
                const int64_t off = (q0 + col) * row_stride + (int64_t)head * D + half * (D / 2);
#pragma unroll
                for (int e = 0; e < D / 2; e += 8) *reinterpret_cast<u32x4 *>(out + off + e) = u32x4{0, 0, 0, 0};
                if (half == 0) lse[(int64_t)head * sum_Bq + q0 + col] = -INFINITY;
            }
            if (tid == 0) {
                fq_walk_offsets(ahead, offsets_q, offsets_kv, total);
                fq_walk_publish(ahead, slot, it, H, total);
            }
            continue;
        }
        const __bf16 *const kbase = k + k0 * row_stride + (int64_t)head * D;
        const __bf16 *const vbase = v + k0 * row_stride + (int64_t)head * D;
        auto fetch_block = [&](int blk, int buf) {   // K and V rows of block `blk` into this wave's buffer `buf`
            const int j0 = blk * kFqRows;
            const int valid = Lk - j0 < kFqRows ? Lk - j0 : kFqRows;
            ln.copy_rows(kbase + j0 * row_stride, (int)row_stride, valid, KV[wave][buf]);
            ln.copy_rows(vbase + j0 * row_stride, (int)row_stride, valid, KV[wave][buf] + kFqTile);
        };
        if (wave == 0) ln.copy_rows(q + q0 * row_stride + (int64_t)head * D, (int)row_stride, Lq, Qt);
        if (wave < n_blocks) fetch_block(wave, 0);
        __builtin_amdgcn_s_waitcnt(0x0070);   // this wave's copies have landed
        __syncthreads();                      // the Q tile is there for every wave
        if (tid == 0) fq_walk_offsets(ahead, offsets_q, offsets_kv, total);   // in flight during the item's blocks
        bf16x8 Qf[kFqKSteps];
        ln.fragments(Qt, Qf);
        float m = -INFINITY, l = 0.0f;   // raw-score maximum and probability sum of this lane's query over this wave's blocks
        f32x16 o[kFqDBlocks];            // out^T of this wave's blocks, not yet normalised
#pragma unroll
        for (int db = 0; db < kFqDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;

        int buf = 0;
        for (int blk = wave; blk < n_blocks; blk += kFqWaves, buf ^= 1) {
            const int j0 = blk * kFqRows;
            const int valid = Lk - j0 < kFqRows ? Lk - j0 : kFqRows;   // keys of this block
            const char *const Kt = KV[wave][buf], *const Vt = KV[wave][buf] + kFqTile;
            // This block's rows have landed (nothing else of this wave is in flight), and all LDS reads of the other
            // buffer are done, so the next block's rows may go there.
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            if (blk + kFqWaves < n_blocks) fetch_block(blk + kFqWaves, buf ^ 1);
            bf16x8 Kf[kFqKSteps];
            ln.fragments(Kt, Kf);
            f32x16 s;
#pragma unroll
            for (int e = 0; e < 16; ++e) s[e] = 0.0f;
            fq_product(Kf, Qf, s);   // keys on the rows, this lane's query
            float mb = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                if ((e >> 2) * 8 + half * 4 + (e & 3) >= valid) s[e] = -INFINITY;   // a key past the sample's end
                mb = fmaxf(mb, s[e]);
            }
            const float n = fmaxf(m, pair_max(mb));   // finite: every block has a valid key
            const float a = fast_exp2((m - n) * c);   // 0 for the wave's first block
            const float nc = n * c;
            m = n;
            l *= a;
#pragma unroll
            for (int db = 0; db < kFqDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= a;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                // the probabilities are rounded to bf16 for the second product; the sum adds what that product uses
                const float p = (float)(__bf16)fast_exp2(fmaf(s[e], c, -nc));
                s[e] = p;
                l += p;
            }
            ln.accumulate(Vt, s, o);
        }
        // ---- merge: wave w leaves its block in its own first buffer as fp32 [feature][query], 16 KB (no copy is in
        // flight: the last block requested none), its maxima and sums beside it ----
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);
        {
            float *part = reinterpret_cast<float *>(KV[wave][0]);
#pragma unroll
            for (int db = 0; db < kFqDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int d = db * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                    part[d * kFqRows + col] = o[db][e];
                }
            const float l_both = pair_sum(l);
            if (half == 0) {
                part_m[wave][col] = m;
                part_l[wave][col] = l_both;
            }
        }
        __syncthreads();
        {   // thread t merges query t % 32, features 16 (t / 32) .. + 15, over the waves that had blocks
            const int qi = tid & 31, d0 = (tid >> 5) * 16;
            const int n_parts = n_blocks < kFqWaves ? n_blocks : kFqWaves;
            float mx = -INFINITY;
            for (int pw = 0; pw < n_parts; ++pw) mx = fmaxf(mx, part_m[pw][qi]);
            float sum[16], total_l = 0.0f;
#pragma unroll
            for (int x = 0; x < 16; ++x) sum[x] = 0.0f;
            for (int pw = 0; pw < n_parts; ++pw) {
                const float wgt = fast_exp2((part_m[pw][qi] - mx) * c);
                total_l = fmaf(part_l[pw][qi], wgt, total_l);
                const float *part = reinterpret_cast<const float *>(KV[pw][0]);
#pragma unroll
                for (int x = 0; x < 16; ++x) sum[x] = fmaf(part[(d0 + x) * kFqRows + qi], wgt, sum[x]);
            }
            if (qi < Lq) {
                const float inv = 1.0f / total_l;
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8) {
                    bf16x8 y;
#pragma unroll
                    for (int x = 0; x < 8; ++x) y[x] = (__bf16)(sum[8 * h8 + x] * inv);
                    *reinterpret_cast<bf16x8 *>(out + (q0 + qi) * row_stride + (int64_t)head * D + d0 + 8 * h8) = y;
                }
                if (d0 == 0) lse[(int64_t)head * sum_Bq + q0 + qi] = (mx * c + fast_log2(total_l)) * 0.6931471805599453f;
            }
        }
        if (tid == 0) fq_walk_publish(ahead, slot, it, H, total);
    }
}

hipError_t launch_fwd_cross_fewq(const void *q, const void *k, const void *v, const int64_t *offsets_q,
                                 const int64_t *offsets_kv, int B, int H, int D, Schedule sched, void *out, float *lse, int cus,
                                 hipStream_t stream) {
    if (D != kBdD) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fwd_cross_fewq_kernel, dim3(persistent_grid<fwd_cross_fewq_kernel>(kFqThreads, cus)), dim3(kFqThreads), 0,
                       stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, offsets_q, offsets_kv, B, H, sched,
                       (__bf16 *)out, lse);
    return hipGetLastError();
}

}  // namespace jfa

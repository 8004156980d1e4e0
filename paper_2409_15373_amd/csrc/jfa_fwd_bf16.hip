// Jagged flash attention forward, bf16 on gfx950 matrix cores (paper Section 2.1).
//
// Work item = (sample, head, block of 128 queries), pulled by persistent workgroups from the
// offsets-driven schedule.  A workgroup is four waves; each wave owns 32 queries and keeps, in
// registers, their Q rows (as MFMA B operands), the running row maximum m, the running row sum l
// and the un-normalised output accumulator.  The sample's keys and values stream through LDS in
// blocks of 64 rows shared by the four waves; the score tile never leaves registers.
//
// Per key block a wave computes the TRANSPOSED score tile  S^T = K Q^T  (keys on the MFMA row
// axis, queries on the column axis).  In the accumulator layout a lane then holds 16 keys of ONE
// query (lane l: query l % 32), so the row maximum and row sum of the online softmax are
// in-register reductions plus a single exchange with lane l ^ 32, the rescale factor is a per-lane
// scalar, and the probabilities -- rounded to bf16 -- already sit where the B operand of
// O^T += V^T P^T wants them.  V^T tiles come from row-major V in LDS through the transposing LDS
// read, with key rows taken in the order the accumulator holds them.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kFwdThreads = 256;
constexpr int kFwdBN = 64;  // keys per LDS stage

template <int D>
struct alignas(16) FwdSmem {
    static constexpr int kStrideK = D * 2 + 16;  // bytes per K row: conflict-free 16-byte row reads
    static constexpr int kStrideV = D * 2 + 32;  // bytes per V row: conflict-free transposing reads
    char k[kFwdBN * kStrideK];
    char v[kFwdBN * kStrideV];
    int slot;
};

template <int D>
__global__ __launch_bounds__(kFwdThreads, 2) void fwd_bf16_kernel(const __bf16 *__restrict__ q,
                                                                  const __bf16 *__restrict__ k,
                                                                  const __bf16 *__restrict__ v,
                                                                  const int64_t *__restrict__ offsets, int B, int H,
                                                                  Schedule s, __bf16 *__restrict__ out,
                                                                  float *__restrict__ lse) {
    constexpr int kKSteps = D / 16;               // contraction steps of S^T = K Q^T
    constexpr int kDBlocks = D / 32;              // 32-row blocks of O^T
    constexpr int kChunksPerRow = D / 8;          // 16-byte chunks per row
    constexpr int kLoads = kFwdBN * kChunksPerRow / kFwdThreads;  // chunks per thread per tensor per stage
    using Smem = FwdSmem<D>;
    __shared__ Smem sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const float c = 1.4426950408889634f / sqrtf((float)D);  // log2(e) / sqrt(D): exp(x / sqrt(D)) = exp2(c x)
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];
    const int64_t row_stride = (int64_t)H * D;    // elements between consecutive rows of one head

    for (;;) {
        __syncthreads();
        if (tid == 0) sm.slot = atomicAdd(s.counter, 1);
        __syncthreads();
        const int64_t w = sm.slot;
        if (w >= total) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const __bf16 *kbase = k + t.row0 * row_stride + (int64_t)t.head * D;
        const __bf16 *vbase = v + t.row0 * row_stride + (int64_t)t.head * D;

        // ---- this lane's query row as B operands: Q[i][16 ks + 8 half .. +7] ----
        const int i = t.block * kFwdBlockRows + wave * 32 + col;   // query index inside the sample
        const int iq = i < L ? i : L - 1;                           // rows past the end recompute the last row
        bf16x8 qreg[kKSteps];
        {
            const __bf16 *qrow = q + (t.row0 + iq) * row_stride + (int64_t)t.head * D + 8 * half;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
        }

        f32x16 o[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
        float m = -INFINITY;   // running maximum of the raw (unscaled) scores of this lane's query
        float lsum = 0.0f;     // this lane's share of the running sum (keys held by this lane only)

        // ---- software pipeline: global -> registers for block jb+1 while block jb is computed ----
        u32x4 kpre[kLoads], vpre[kLoads];
        auto prefetch = [&](int j0) {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int chunk = tid + u * kFwdThreads;
                const int r = chunk / kChunksPerRow, cc = chunk % kChunksPerRow;
                const int j = j0 + r < L ? j0 + r : L - 1;          // tail rows repeat the last key (masked later)
                kpre[u] = *reinterpret_cast<const u32x4 *>(kbase + j * row_stride + cc * 8);
                vpre[u] = *reinterpret_cast<const u32x4 *>(vbase + j * row_stride + cc * 8);
            }
        };
        auto commit = [&]() {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int chunk = tid + u * kFwdThreads;
                const int r = chunk / kChunksPerRow, cc = chunk % kChunksPerRow;
                *reinterpret_cast<u32x4 *>(sm.k + r * Smem::kStrideK + cc * 16) = kpre[u];
                *reinterpret_cast<u32x4 *>(sm.v + r * Smem::kStrideV + cc * 16) = vpre[u];
            }
        };

        prefetch(0);
        for (int j0 = 0; j0 < L; j0 += kFwdBN) {
            __syncthreads();          // every wave is done reading the previous stage
            commit();
            __syncthreads();
            if (j0 + kFwdBN < L) prefetch(j0 + kFwdBN);

            // ---- S^T = K Q^T : two 32-key row blocks ----
            f32x16 st[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
                for (int e = 0; e < 16; ++e) st[mb][e] = 0.0f;
                const char *krow = sm.k + (mb * 32 + col) * Smem::kStrideK + half * 16;
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks)
                    st[mb] = mfma_32x32x16(lds_read_b128(krow + ks * 32), qreg[ks], st[mb]);
            }

            // ---- mask keys past the end of the sample (last block only) ----
            if (j0 + kFwdBN > L) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (j0 + mb * 32 + acc_row(e, half) >= L) st[mb][e] = -INFINITY;
            }

            // ---- online softmax for this lane's query ----
            float mx = st[0][0];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[mb][e]);
            mx = pair_max(mx);
            const float m_new = fmaxf(m, mx);
            const float alpha = fast_exp2((m - m_new) * c);   // exp2(-inf) = 0 on the first block
            const float mc = m_new * c;
            m = m_new;
            float psum = 0.0f;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = fast_exp2(fmaf(st[mb][e], c, -mc));
                    st[mb][e] = p;
                    psum += p;
                }
            lsum = fmaf(lsum, alpha, psum);
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;

            // ---- O^T += V^T P^T : contraction over the 64 keys in four steps of 16 ----
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int ts = 0; ts < 2; ++ts) {
                    const bf16x8 pb = pack_bf16(st[mb], 8 * ts);
                    // slot e of this lane is key 32 mb + 16 ts + 8 (e / 4) + 4 half + e % 4
                    const int key0 = mb * 32 + ts * 16 + half * 4 + ((lane & 15) >> 2);
                    const char *vrow = sm.v + key0 * Smem::kStrideV + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) {
                        const bf16x4 lo = lds_read_tr16(vrow + db * 64);
                        const bf16x4 hi = lds_read_tr16(vrow + db * 64 + 8 * Smem::kStrideV);
                        o[db] = mfma_32x32x16(concat(lo, hi), pb, o[db]);
                    }
                }
        }

        // ---- epilogue: normalise, store this lane's query row and its log-sum-exp ----
        const float l_total = pair_sum(lsum);
        if (i < L) {
            const float inv = 1.0f / l_total;
            __bf16 *orow = out + (t.row0 + i) * row_stride + (int64_t)t.head * D;
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = (__bf16)(o[db][4 * g + e] * inv);
                    *reinterpret_cast<bf16x4 *>(orow + db * 32 + g * 8 + half * 4) = x;
                }
            if (half == 0)
                lse[(int64_t)t.head * sum_B + t.row0 + i] = (m * c + fast_log2(l_total)) * 0.6931471805599453f;
        }
    }
}

hipError_t launch_fwd_bf16(const void *q, const void *k, const void *v, const int64_t *offsets, int B, int H, int D,
                           Schedule s, void *out, float *lse, int cus, hipStream_t stream) {
#define JFA_CASE(DD)                                                                                         \
    case DD:                                                                                                 \
        hipLaunchKernelGGL(fwd_bf16_kernel<DD>, dim3(persistent_grid<fwd_bf16_kernel<DD>>(kFwdThreads, cus)), dim3(kFwdThreads), 0, stream, (const __bf16 *)q, \
                           (const __bf16 *)k, (const __bf16 *)v, offsets, B, H, s, (__bf16 *)out, lse);      \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

}  // namespace jfa

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
    // 64 banks x 4 bytes: 16 lanes x 16 bytes (one pass of a 16-byte read) are conflict-free when rows are
    // 16 bytes apart modulo 256; 32 lanes x 8 bytes of the transposing read (4 rows x 64 bytes) are
    // conflict-free when rows are 64 bytes apart modulo 256.
    static constexpr int kStrideK = D * 2 + 16;
    static constexpr int kStrideV = D * 2 + 64;
    char k[2][kFwdBN * kStrideK];   // double buffered: stage jb lives in buffer jb % 2
    char v[2][kFwdBN * kStrideV];
    int64_t slot;
};

// CROSS: the keys and values of a sample are the rows of a second offsets array (cross attention); otherwise
// offsets_kv is not looked at and the code is that of self attention.  CAUSAL (self attention only): query i
// attends to keys 0 .. i of its sample; a tile streams the keys up to its last query and masks above the diagonal.
template <int D, bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kFwdThreads, 2) void fwd_bf16_kernel(const __bf16 *__restrict__ q,
                                                                  const __bf16 *__restrict__ k,
                                                                  const __bf16 *__restrict__ v,
                                                                  const int64_t *__restrict__ offsets,
                                                                  const int64_t *__restrict__ offsets_kv, int B, int H,
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
    // The running maximum is only raised when a block exceeds it by more than 2^8 in the exp2 domain;
    // until then probabilities are taken relative to the stale maximum (at most 256, exact in fp32 and
    // harmless in bf16), which keeps the rescaling of the accumulator off the common path.
    const float tau = 8.0f / c;
    static_assert(sizeof(Smem) >= kInlineScratchInts * sizeof(int), "the stage buffers double as the scheduler's scratch");
    __shared__ SmallWork mine;
    const bool small = s.build_rows != 0;   // small problem: no scheduler launch has run, the schedule is built here, in LDS
    if (small) build_small_work(offsets, CROSS ? offsets_kv : nullptr, B, H, s.build_rows, reinterpret_cast<int *>(&sm), &mine);
    const int64_t total = small ? 0 : (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];
    const int64_t row_stride = (int64_t)H * D;    // elements between consecutive rows of one head
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    // per-lane LDS offsets of the operand reads
    const int koff = col * Smem::kStrideK + half * 16;                       // K row `col`, slots 8 half .. +7
    const int voff = (half * 4 + ((lane & 15) >> 2)) * Smem::kStrideV        // V^T: key row inside a 16-key step
                     + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;        //      feature column of this lane

    WorkCursor cursor;
    cursor.static_only = s.static_only;
    for (int n = 0;; ++n) {
        Work t;
        if (small) {   // the workgroup's items were decoded when the schedule was built
            __syncthreads();   // the previous item's use of the stage buffers is over
            if (n >= __builtin_amdgcn_readfirstlane(mine.count) || !load_work<CROSS>(&mine.item[n], t)) break;
        } else {
            __syncthreads();
            if (tid == 0) sm.slot = next_work(s.counter, cursor, total);
            __syncthreads();
            const int64_t w = uniform64(sm.slot);
            if (w < 0) break;
            t = decode_work(s, offsets, B, H, w, CROSS ? offsets_kv : nullptr);
        }
        const int Lq = t.len;                      // queries of the sample
        const int L = CROSS ? t.olen : t.len;      // keys of the sample
        const int64_t krow0 = CROSS ? t.orow0 : t.row0;
        const int Lc = CAUSAL && (t.block + 1) * kFwdBlockRows < L ? (t.block + 1) * kFwdBlockRows : L;   // keys this tile needs
        const __bf16 *kbase = k + krow0 * row_stride + (int64_t)t.head * D;
        const __bf16 *vbase = v + krow0 * row_stride + (int64_t)t.head * D;

        // ---- this lane's query row as B operands: Q[i][16 ks + 8 half .. +7] ----
        const int i = t.block * kFwdBlockRows + wave * 32 + col;   // query index inside the sample
        const int iq = i < Lq ? i : Lq - 1;                         // rows past the end recompute the last row
        const bool wave_active = t.block * kFwdBlockRows + wave * 32 < Lq;
        if (CROSS && L == 0) {   // no keys: an empty softmax, out = 0 and lse = -inf
            if (i < Lq) {
                __bf16 *orow = out + (t.row0 + i) * row_stride + (int64_t)t.head * D;
#pragma unroll
                for (int e = 0; e < D / 2; e += 4) *reinterpret_cast<bf16x4 *>(orow + half * (D / 2) + e) = bf16x4{0, 0, 0, 0};
                if (half == 0) lse[(int64_t)t.head * sum_B + t.row0 + i] = -INFINITY;
            }
            continue;
        }
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
        float m = -INFINITY;   // reference maximum (raw, unscaled scores) of this lane's query
        float lsum = 0.0f;     // this lane's share of the running sum (keys held by this lane only)

        // ---- staging: global -> registers (in flight during the compute) -> the other LDS buffer ----
        u32x4 kpre[kLoads], vpre[kLoads];
        // Each thread always fetches the same chunk of rows r0 + u * rows_per_pass of the stage, so its source
        // pointers just advance by one stage per iteration; only a ragged last stage clamps its row indices.
        constexpr int kRowsPerPass = kFwdThreads / kChunksPerRow;
        const int my_r = tid / kChunksPerRow, my_cc = tid % kChunksPerRow;
        const __bf16 *kptr = kbase + (int64_t)my_r * row_stride + my_cc * 8;
        const __bf16 *vptr = vbase + (int64_t)my_r * row_stride + my_cc * 8;
        const int64_t pass_stride = (int64_t)kRowsPerPass * row_stride;
        const int64_t stage_stride = (int64_t)kFwdBN * row_stride;
        auto prefetch = [&](int j0) {
            if (j0 + kFwdBN <= L) {
#pragma unroll
                for (int u = 0; u < kLoads; ++u) {
                    kpre[u] = *reinterpret_cast<const u32x4 *>(kptr + u * pass_stride);
                    vpre[u] = *reinterpret_cast<const u32x4 *>(vptr + u * pass_stride);
                }
            } else {
#pragma unroll
                for (int u = 0; u < kLoads; ++u) {
                    const int r = my_r + u * kRowsPerPass;
                    const int j = j0 + r < L ? j0 + r : L - 1;      // tail rows repeat the last key (masked later)
                    kpre[u] = *reinterpret_cast<const u32x4 *>(kbase + j * row_stride + my_cc * 8);
                    vpre[u] = *reinterpret_cast<const u32x4 *>(vbase + j * row_stride + my_cc * 8);
                }
            }
            kptr += stage_stride;
            vptr += stage_stride;
        };
        auto commit = [&](int buf) {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int chunk = tid + u * kFwdThreads;
                const int r = chunk / kChunksPerRow, cc = chunk % kChunksPerRow;
                *reinterpret_cast<u32x4 *>(sm.k[buf] + r * Smem::kStrideK + cc * 16) = kpre[u];
                *reinterpret_cast<u32x4 *>(sm.v[buf] + r * Smem::kStrideV + cc * 16) = vpre[u];
            }
        };

        prefetch(0);
        commit(0);
        // Pin the completion of the Q loads here: left pending into the loop, their wait would be merged into
        // every iteration and stall the first matrix products on the stage prefetch issued just before them.
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qreg[ks]));
        __syncthreads();
        int buf = 0;
        for (int j0 = 0; j0 < Lc; j0 += kFwdBN, buf ^= 1) {
            const bool more = j0 + kFwdBN < Lc;
            if (more) prefetch(j0 + kFwdBN);
            if (wave_active) {
                const char *kt = sm.k[buf] + koff;
                const char *vt = sm.v[buf] + voff;

                // ---- S^T = K Q^T : two 32-key row blocks; operands of a block are fetched together ----
                f32x16 st[2];
                bf16x8 ka[kKSteps], kb[kKSteps];
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) ka[ks] = lds_read_b128(kt + ks * 32);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) kb[ks] = lds_read_b128(kt + 32 * Smem::kStrideK + ks * 32);
#pragma unroll
                for (int e = 0; e < 16; ++e) { st[0][e] = 0.0f; st[1][e] = 0.0f; }
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) st[0] = mfma_32x32x16(ka[ks], qreg[ks], st[0]);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) st[1] = mfma_32x32x16(kb[ks], qreg[ks], st[1]);
                // issue order: the first block's operand reads, then one read of the second block behind each
                // matrix product of the first, so that LDS latency hides under the matrix pipe
                __builtin_amdgcn_sched_group_barrier(0x100, kKSteps, 0);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, kKSteps, 0);

                // ---- mask keys past the end of the sample (last block only) and, if causal, above the diagonal ----
                const int first_q = t.block * kFwdBlockRows + wave * 32;   // no lane of this wave masks a key below first_q + 1
                if (j0 + kFwdBN > (CAUSAL && first_q + 1 < L ? first_q + 1 : L)) {
                    const int lim = CAUSAL && iq + 1 < L ? iq + 1 : L;     // this lane's query sees keys 0 .. lim - 1
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (j0 + mb * 32 + acc_row(e, half) >= lim) st[mb][e] = -INFINITY;
                }

                // ---- online softmax for this lane's query ----
                float mx = st[0][0];
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[mb][e]);
                mx = pair_max(mx);
                if (__builtin_amdgcn_ballot_w64(mx > m + tau) != 0) {
                    const float m_new = fmaxf(m, mx);
                    const float alpha = fast_exp2((m - m_new) * c);     // exp2(-inf) = 0 on the first block
                    m = m_new;
                    lsum *= alpha;
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                        for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
                }
                const float mc = m * c;
                bf16x8 pb[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x4 pw;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        bf16x2 pr;
                        pr[0] = (__bf16)fast_exp2(fmaf(st[g >> 1][8 * (g & 1) + 2 * e], c, -mc));
                        pr[1] = (__bf16)fast_exp2(fmaf(st[g >> 1][8 * (g & 1) + 2 * e + 1], c, -mc));
                        // row sum of the ROUNDED probabilities, the values the second product uses
                        lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum, false);
                        pw[e] = __builtin_bit_cast(uint32_t, pr);
                    }
                    pb[g] = __builtin_bit_cast(bf16x8, pw);
                }

                // ---- O^T += V^T P^T : contraction over the 64 keys in four steps of 16 ----
                // slot e of step g is key 16 g + 8 (e / 4) + 4 half + e % 4
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x8 va[kDBlocks];
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) {
                        const char *pv = vt + g * 16 * Smem::kStrideV + db * 64;
                        va[db] = concat(lds_read_tr16(pv), lds_read_tr16(pv + 8 * Smem::kStrideV));
                    }
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) o[db] = mfma_32x32x16(va[db], pb[g], o[db]);
                }
            }
            if (more) commit(buf ^ 1);
            __syncthreads();
        }

        // ---- epilogue: normalise, store this lane's query row and its log-sum-exp ----
        const float l_total = pair_sum(lsum);
        if (i < Lq) {
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

hipError_t launch_fwd_bf16(const void *q, const void *k, const void *v, const int64_t *offsets,
                           const int64_t *offsets_kv, bool causal, int B, int H, int D, Schedule s, void *out, float *lse,
                           int cus, hipStream_t stream) {
    if (causal && offsets_kv) return hipErrorInvalidValue;
#define JFA_LAUNCH(DD, CROSS, CAUSAL)                                                                        \
    hipLaunchKernelGGL((fwd_bf16_kernel<DD, CROSS, CAUSAL>), dim3(persistent_grid<fwd_bf16_kernel<DD, CROSS, CAUSAL>>(kFwdThreads, cus)), \
                       dim3(kFwdThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, offsets, offsets_kv, B, H, s, \
                       (__bf16 *)out, lse)
#define JFA_CASE(DD)                                                                                         \
    case DD:                                                                                                 \
        if (offsets_kv) JFA_LAUNCH(DD, true, false);                                                         \
        else if (causal) JFA_LAUNCH(DD, false, true);                                                        \
        else JFA_LAUNCH(DD, false, false);                                                                   \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
#undef JFA_LAUNCH
    return hipGetLastError();
}

}  // namespace jfa

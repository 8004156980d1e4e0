// Jagged flash attention backward, bf16 on gfx950 matrix cores (paper Section 2.2: every jagged
// operator has a backward; the formulas are those of softmax attention, with P recomputed from the
// stored log-sum-exp so that no score matrix is ever kept).
//
//   P  = exp(S / sqrt(D) - lse),   dP = dO V^T,   dS = P o (dP - delta),   delta = rowsum(dO o O)
//   dV = P^T dO,   dQ = dS K / sqrt(D),   dK = dS^T Q / sqrt(D)
//
// Deterministic two-kernel split, both persistent over the offsets-driven schedule:
//   dq_kernel   work item = (sample, head, 128 queries); a wave owns 32 queries (Q, dO rows in
//               registers as MFMA operands), streams the sample's K and V through LDS and
//               accumulates dQ^T.  Tiles are computed transposed (keys on the MFMA row axis) so
//               that dS^T leaves the accumulator already in operand position for dQ^T += K^T dS^T.
//   dkv_kernel  work item = (sample, head, 128 keys); a wave owns 32 keys (K, V rows in registers),
//               streams the sample's Q, dO, lse, delta through LDS and accumulates dK^T and dV^T;
//               here queries are on the MFMA row axis, so P and dS leave the accumulator in
//               operand position for dV^T += dO^T P and dK^T += Q^T dS.
// The transposed operands (K^T, Q^T, dO^T) come from row-major LDS tiles via the transposing read.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kBwdThreads = 256;
constexpr int kBwdStage = 64;  // streamed rows per LDS stage

// Global -> registers -> LDS staging of `kBwdStage` rows of one head of a [*, H, D] bf16 tensor.
template <int D>
struct Stage {
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kLoads = kBwdStage * kChunksPerRow / kBwdThreads;
    u32x4 regs[kLoads];
    __device__ inline void prefetch(const __bf16 *base, int64_t row_stride, int r0, int L) {
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int chunk = threadIdx.x + u * kBwdThreads;
            const int r = chunk / kChunksPerRow, cc = chunk % kChunksPerRow;
            const int j = r0 + r < L ? r0 + r : L - 1;  // rows past the end repeat the last row (masked by the caller)
            regs[u] = *reinterpret_cast<const u32x4 *>(base + j * row_stride + cc * 8);
        }
    }
    __device__ inline void commit(char *lds, int stride) const {
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int chunk = threadIdx.x + u * kBwdThreads;
            const int r = chunk / kChunksPerRow, cc = chunk % kChunksPerRow;
            *reinterpret_cast<u32x4 *>(lds + r * stride + cc * 16) = regs[u];
        }
    }
};

template <int D>
struct alignas(16) BwdSmem {
    // bytes per staged row: +80 keeps both the 16-byte row reads and the transposing reads (nearly) conflict-free
    // on the 64-bank LDS (16 lanes x 16 bytes need rows 16 bytes apart modulo 256, 4 rows x 64 bytes need them 64 apart)
    static constexpr int kStride = D * 2 + 80;
    char a[kBwdStage * kStride];                // dq: K      dkv: Q
    char b[kBwdStage * kStride];                // dq: V      dkv: dO
    float lse2[kBwdStage];                      // dkv only: lse * log2(e), +inf for rows past the end
    float delta[kBwdStage];                     // dkv only
    int64_t slot;
};

// Store a transposed accumulator (rows = features, column = this lane's row of the output tensor).
template <int D>
__device__ inline void store_rows(__bf16 *dst_row, const f32x16 (&acc)[D / 32], float scale, int half) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 x;
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = (__bf16)(acc[db][4 * g + e] * scale);
            *reinterpret_cast<bf16x4 *>(dst_row + db * 32 + g * 8 + half * 4) = x;
        }
}

// CROSS: keys and values are the rows of a second offsets array (offsets_kv); CAUSAL: query i sees keys 0 .. i.
// See the forward kernel.
template <int D, bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kBwdThreads, 2) void dq_bf16_kernel(const __bf16 *__restrict__ q,
                                                                 const __bf16 *__restrict__ k,
                                                                 const __bf16 *__restrict__ v,
                                                                 const __bf16 *__restrict__ dout,
                                                                 const float *__restrict__ lse,
                                                                 const __bf16 *__restrict__ out_fwd,   // see delta
                                                                 float *delta,
                                                                 const int64_t *__restrict__ offsets,
                                                                 const int64_t *__restrict__ offsets_kv, int B, int H,
                                                                 Schedule s, __bf16 *__restrict__ dq) {
    constexpr int kKSteps = D / 16, kDBlocks = D / 32;
    using Smem = BwdSmem<D>;
    __shared__ Smem sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    static_assert(sizeof(Smem) >= kInlineScratchInts * sizeof(int), "the stage buffers double as the scheduler's scratch");
    __shared__ SmallWork mine;
    const bool small = s.build_rows != 0;   // small problem: no scheduler launch has run, the schedule is built here, in LDS
    if (small) build_small_work(offsets, CROSS ? offsets_kv : nullptr, B, H, s.build_rows, reinterpret_cast<int *>(&sm), &mine);
    const int64_t total = small ? 0 : (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];
    const int64_t row_stride = (int64_t)H * D;

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
        const int Lc = CAUSAL && (t.block + 1) * kBwdBlockRows < L ? (t.block + 1) * kBwdBlockRows : L;   // keys this tile needs
        const __bf16 *kbase = k + krow0 * row_stride + (int64_t)t.head * D;
        const __bf16 *vbase = v + krow0 * row_stride + (int64_t)t.head * D;

        const int i = t.block * kBwdBlockRows + wave * 32 + col;
        const int iq = i < Lq ? i : Lq - 1;
        const bool wave_active = t.block * kBwdBlockRows + wave * 32 < Lq;
        bf16x8 qreg[kKSteps], doreg[kKSteps];
        {
            const int64_t off = (t.row0 + iq) * row_stride + (int64_t)t.head * D + 8 * half;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                qreg[ks] = *reinterpret_cast<const bf16x8 *>(q + off + 16 * ks);
                doreg[ks] = *reinterpret_cast<const bf16x8 *>(dout + off + 16 * ks);
            }
        }
        const float lse2 = lse[(int64_t)t.head * sum_B + t.row0 + iq] * 1.4426950408889634f;
        // delta = rowsum(dO o O) of this lane's query.  With out_fwd given this kernel is the first of the backward and
        // computes it from the dO row it holds (each lane of a pair has half of the row), leaving it in `delta` for the
        // dK / dV kernel; otherwise an earlier kernel has filled `delta`.
        float delta_i;
        if (out_fwd != nullptr) {
            const int64_t off = (t.row0 + iq) * row_stride + (int64_t)t.head * D + 8 * half;
            float dot = 0.0f;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                const bf16x8 o = *reinterpret_cast<const bf16x8 *>(out_fwd + off + 16 * ks);
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf((float)o[e], (float)doreg[ks][e], dot);
            }
            delta_i = pair_sum(dot);
            if (i < Lq && half == 0) delta[(int64_t)t.head * sum_B + t.row0 + i] = delta_i;
        } else {
            delta_i = delta[(int64_t)t.head * sum_B + t.row0 + iq];
        }

        f32x16 acc[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[db][e] = 0.0f;

        Stage<D> sk, sv;
        if (!CROSS || L > 0) {   // a sample without keys: nothing streams, dq = 0
            sk.prefetch(kbase, row_stride, 0, L);
            sv.prefetch(vbase, row_stride, 0, L);
        }
        for (int j0 = 0; j0 < Lc; j0 += kBwdStage) {
            __syncthreads();
            sk.commit(sm.a, Smem::kStride);
            sv.commit(sm.b, Smem::kStride);
            __syncthreads();
            if (j0 + kBwdStage < Lc) {
                sk.prefetch(kbase, row_stride, j0 + kBwdStage, L);
                sv.prefetch(vbase, row_stride, j0 + kBwdStage, L);
            }
            if (!wave_active) continue;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                if (j0 + mb * 32 >= Lc) break;
                f32x16 st, dpt;
#pragma unroll
                for (int e = 0; e < 16; ++e) { st[e] = 0.0f; dpt[e] = 0.0f; }
                const char *krow = sm.a + (mb * 32 + col) * Smem::kStride + half * 16;
                const char *vrow = sm.b + (mb * 32 + col) * Smem::kStride + half * 16;
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) st = mfma_32x32x16(lds_read_b128(krow + ks * 32), qreg[ks], st);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) dpt = mfma_32x32x16(lds_read_b128(vrow + ks * 32), doreg[ks], dpt);
                // dS^T = P^T o (dP^T - delta); keys past the end of the sample (and, if causal, above the diagonal) get P = 0
                const int first_q = t.block * kBwdBlockRows + wave * 32;   // no lane of this wave masks a key below first_q + 1
                const bool tail = j0 + mb * 32 + 32 > (CAUSAL && first_q + 1 < L ? first_q + 1 : L);
                const int lim = CAUSAL && iq + 1 < L ? iq + 1 : L;         // this lane's query sees keys 0 .. lim - 1
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float p = fast_exp2(fmaf(st[e], c, -lse2));
                    if (tail && j0 + mb * 32 + acc_row(e, half) >= lim) p = 0.0f;
                    st[e] = p * (dpt[e] - delta_i);
                }
                // dQ^T += K^T dS^T
#pragma unroll
                for (int ts = 0; ts < 2; ++ts) {
                    const bf16x8 dsb = pack_bf16(st, 8 * ts);
                    const int key0 = mb * 32 + ts * 16 + half * 4 + ((lane & 15) >> 2);
                    const char *kt = sm.a + key0 * Smem::kStride + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) {
                        const bf16x4 lo = lds_read_tr16(kt + db * 64);
                        const bf16x4 hi = lds_read_tr16(kt + db * 64 + 8 * Smem::kStride);
                        acc[db] = mfma_32x32x16(concat(lo, hi), dsb, acc[db]);
                    }
                }
            }
        }
        if (i < Lq) store_rows<D>(dq + (t.row0 + i) * row_stride + (int64_t)t.head * D, acc, scale, half);
    }
}

// CROSS: `offsets` are the keys' offsets (the work items are blocks of keys) and the queries, with dout, lse and
// delta, are the rows of offsets_q.  CAUSAL: key j is seen by queries j .. L - 1: the stream starts at the stage that
// holds the tile's first key, and streamed rows below the lane's key get P = 0.
template <int D, bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kBwdThreads, D <= 64 ? 2 : 1) void dkv_bf16_kernel(const __bf16 *__restrict__ q,
                                                                  const __bf16 *__restrict__ k,
                                                                  const __bf16 *__restrict__ v,
                                                                  const __bf16 *__restrict__ dout,
                                                                  const float *__restrict__ lse,
                                                                  const float *__restrict__ delta,
                                                                  const int64_t *__restrict__ offsets,
                                                                  const int64_t *__restrict__ offsets_q, int B, int H,
                                                                  Schedule s, __bf16 *__restrict__ dk,
                                                                  __bf16 *__restrict__ dv) {
    constexpr int kKSteps = D / 16, kDBlocks = D / 32;
    using Smem = BwdSmem<D>;
    __shared__ Smem sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    static_assert(sizeof(Smem) >= kInlineScratchInts * sizeof(int), "the stage buffers double as the scheduler's scratch");
    __shared__ SmallWork mine;
    const bool small = s.build_rows != 0;   // small problem: no scheduler launch has run, the schedule is built here, in LDS
    if (small) build_small_work(offsets, CROSS ? offsets_q : nullptr, B, H, s.build_rows, reinterpret_cast<int *>(&sm), &mine);
    const int64_t total = small ? 0 : (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = CROSS ? offsets_q[B] : offsets[B];   // lse and delta are indexed by query rows
    const int64_t row_stride = (int64_t)H * D;

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
            t = decode_work(s, offsets, B, H, w, CROSS ? offsets_q : nullptr);
        }
        const int Lk = t.len;                      // keys of the sample
        const int L = CROSS ? t.olen : t.len;      // queries of the sample
        const int64_t qrow0 = CROSS ? t.orow0 : t.row0;
        const __bf16 *qbase = q + qrow0 * row_stride + (int64_t)t.head * D;
        const __bf16 *dobase = dout + qrow0 * row_stride + (int64_t)t.head * D;
        const float *lse_base = lse + (int64_t)t.head * sum_B + qrow0;
        const float *delta_base = delta + (int64_t)t.head * sum_B + qrow0;

        const int j = t.block * kBwdBlockRows + wave * 32 + col;  // this lane's key
        const int jk = j < Lk ? j : Lk - 1;
        const bool wave_active = t.block * kBwdBlockRows + wave * 32 < Lk;
        bf16x8 kreg[kKSteps], vreg[kKSteps];
        {
            const int64_t off = (t.row0 + jk) * row_stride + (int64_t)t.head * D + 8 * half;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                kreg[ks] = *reinterpret_cast<const bf16x8 *>(k + off + 16 * ks);
                vreg[ks] = *reinterpret_cast<const bf16x8 *>(v + off + 16 * ks);
            }
        }
        f32x16 acck[kDBlocks], accv[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) { acck[db][e] = 0.0f; accv[db][e] = 0.0f; }

        Stage<D> sq, sdo;
        float lse_pre = 0.0f, delta_pre = 0.0f;
        auto prefetch_rows = [&](int i0) {
            sq.prefetch(qbase, row_stride, i0, L);
            sdo.prefetch(dobase, row_stride, i0, L);
            if (tid < kBwdStage) {
                const bool ok = i0 + tid < L;
                lse_pre = ok ? lse_base[i0 + tid] * 1.4426950408889634f : INFINITY;  // +inf => P = 0 past the end
                delta_pre = ok ? delta_base[i0 + tid] : 0.0f;
            }
        };
        const int istart = CAUSAL ? (t.block * kBwdBlockRows / kBwdStage) * kBwdStage : 0;
        if (!CROSS || L > 0) prefetch_rows(istart);   // a sample without queries: nothing streams, dk = dv = 0
        for (int i0 = istart; i0 < L; i0 += kBwdStage) {
            __syncthreads();
            sq.commit(sm.a, Smem::kStride);
            sdo.commit(sm.b, Smem::kStride);
            if (tid < kBwdStage) { sm.lse2[tid] = lse_pre; sm.delta[tid] = delta_pre; }
            __syncthreads();
            if (i0 + kBwdStage < L) prefetch_rows(i0 + kBwdStage);
            if (!wave_active) continue;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                if (i0 + mb * 32 >= L) break;
                f32x16 sc, dp;
#pragma unroll
                for (int e = 0; e < 16; ++e) { sc[e] = 0.0f; dp[e] = 0.0f; }
                const char *qrow = sm.a + (mb * 32 + col) * Smem::kStride + half * 16;
                const char *dorow = sm.b + (mb * 32 + col) * Smem::kStride + half * 16;
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) sc = mfma_32x32x16(lds_read_b128(qrow + ks * 32), kreg[ks], sc);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) dp = mfma_32x32x16(lds_read_b128(dorow + ks * 32), vreg[ks], dp);
                // P and dS for this lane's key and its 16 queries of the block
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 l4 = *reinterpret_cast<const float4 *>(&sm.lse2[mb * 32 + g * 8 + half * 4]);
                    const float4 d4 = *reinterpret_cast<const float4 *>(&sm.delta[mb * 32 + g * 8 + half * 4]);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float p = fast_exp2(fmaf(sc[4 * g + e], c, -lv[e]));
                        if (CAUSAL && i0 + mb * 32 + g * 8 + half * 4 + e < jk) p = 0.0f;   // queries before this lane's key
                        sc[4 * g + e] = p;
                        dp[4 * g + e] = p * (dp[4 * g + e] - dl[e]);
                    }
                }
                // dV^T += dO^T P ;  dK^T += Q^T dS   (contraction over the 32 queries in two steps of 16)
#pragma unroll
                for (int ts = 0; ts < 2; ++ts) {
                    const bf16x8 pb = pack_bf16(sc, 8 * ts);
                    const bf16x8 dsb = pack_bf16(dp, 8 * ts);
                    const int q0 = mb * 32 + ts * 16 + half * 4 + ((lane & 15) >> 2);
                    const int toff = q0 * Smem::kStride + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) {
                        const bf16x4 dlo = lds_read_tr16(sm.b + toff + db * 64);
                        const bf16x4 dhi = lds_read_tr16(sm.b + toff + db * 64 + 8 * Smem::kStride);
                        accv[db] = mfma_32x32x16(concat(dlo, dhi), pb, accv[db]);
                        const bf16x4 qlo = lds_read_tr16(sm.a + toff + db * 64);
                        const bf16x4 qhi = lds_read_tr16(sm.a + toff + db * 64 + 8 * Smem::kStride);
                        acck[db] = mfma_32x32x16(concat(qlo, qhi), dsb, acck[db]);
                    }
                }
            }
        }
        if (j < Lk) {
            const int64_t off = (t.row0 + j) * row_stride + (int64_t)t.head * D;
            store_rows<D>(dk + off, acck, scale, half);
            store_rows<D>(dv + off, accv, 1.0f, half);
        }
    }
}

hipError_t launch_dkv_bf16(const void *q, const void *k, const void *v, const void *dout, const float *lse,
                           const float *delta, const int64_t *offsets, const int64_t *offsets_q, bool causal, int B, int H,
                           int D, Schedule s, void *dk, void *dv, int cus, hipStream_t stream) {
    if (causal && offsets_q) return hipErrorInvalidValue;
#define JFA_LAUNCH(DD, CROSS, CAUSAL)                                                                            \
    hipLaunchKernelGGL((dkv_bf16_kernel<DD, CROSS, CAUSAL>), dim3(persistent_grid<dkv_bf16_kernel<DD, CROSS, CAUSAL>>(kBwdThreads, cus)), \
                       dim3(kBwdThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, (const __bf16 *)dout, lse, \
                       delta, offsets, offsets_q, B, H, s, (__bf16 *)dk, (__bf16 *)dv)
#define JFA_CASE(DD)                                                                                             \
    case DD:                                                                                                     \
        if (offsets_q) JFA_LAUNCH(DD, true, false);                                                              \
        else if (causal) JFA_LAUNCH(DD, false, true);                                                            \
        else JFA_LAUNCH(DD, false, false);                                                                       \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
#undef JFA_LAUNCH
    return hipGetLastError();
}

hipError_t launch_dq_bf16(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                          float *delta, const int64_t *offsets, const int64_t *offsets_kv, bool causal, int B, int H,
                          int D, Schedule s, void *dq, int cus, hipStream_t stream) {
    if (causal && offsets_kv) return hipErrorInvalidValue;
#define JFA_LAUNCH(DD, CROSS, CAUSAL)                                                                            \
    hipLaunchKernelGGL((dq_bf16_kernel<DD, CROSS, CAUSAL>), dim3(persistent_grid<dq_bf16_kernel<DD, CROSS, CAUSAL>>(kBwdThreads, cus)), \
                       dim3(kBwdThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, (const __bf16 *)dout, lse, \
                       (const __bf16 *)out, delta, offsets, offsets_kv, B, H, s, (__bf16 *)dq)
#define JFA_CASE(DD)                                                                                             \
    case DD:                                                                                                     \
        if (offsets_kv) JFA_LAUNCH(DD, true, false);                                                             \
        else if (causal) JFA_LAUNCH(DD, false, true);                                                            \
        else JFA_LAUNCH(DD, false, false);                                                                       \
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

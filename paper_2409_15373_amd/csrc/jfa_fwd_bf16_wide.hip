// Jagged flash attention forward, bf16, "wide" variant for long samples (paper Section 2.1).
//
// Same mathematics and operand layouts as fwd_bf16_kernel (transposed score tile S^T = K Q^T, a lane owns
// one query, V^T through the transposing LDS read), but a wave owns 64 queries as two 32-query column
// blocks and runs alone on its SIMD with the full register file.  That buys two things:
//   * every K and V^T operand fetched from LDS feeds two matrix products (one per column block), halving
//     LDS traffic per flop;
//   * the two column blocks give one instruction stream two independent chains, so the softmax of one
//     (exp2, convert, sums: VALU work) is interleaved with the matrix products of the other and the
//     matrix pipe does not idle during the softmax.
// The exponentials do not wait for the block maximum: they are taken against the running reference
// maximum right away, and the maximum of the block is only used afterwards to check that the reference
// was close enough (within 2^8); if not -- always on a query's first block, rarely later -- the unit is
// redone against the new maximum and the accumulator rescaled.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kWideThreads = 256;
constexpr int kWideBN = 64;  // keys per LDS stage

template <int D>
struct alignas(16) WideSmem {
    static constexpr int kStrideK = D * 2 + 16;
    static constexpr int kStrideV = D * 2 + 64;
    char k[2][kWideBN * kStrideK];
    char v[2][kWideBN * kStrideV];
    int64_t slot;
};

template <int N> using Int = std::integral_constant<int, N>;

template <int D>
__global__ __launch_bounds__(kWideThreads, 1) void fwd_bf16_wide_kernel(const __bf16 *__restrict__ q,
                                                                        const __bf16 *__restrict__ k,
                                                                        const __bf16 *__restrict__ v,
                                                                        const int64_t *__restrict__ offsets, int B,
                                                                        int H, Schedule s, __bf16 *__restrict__ out,
                                                                        float *__restrict__ lse) {
    constexpr int kKSteps = D / 16;
    constexpr int kDBlocks = D / 32;
    constexpr int kChunksPerRow = D / 8;
    constexpr int kLoads = kWideBN * kChunksPerRow / kWideThreads;
    constexpr int kRowsPerPass = kWideThreads / kChunksPerRow;
    using Smem = WideSmem<D>;
    __shared__ Smem sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const float c = 1.4426950408889634f / sqrtf((float)D);
    const float tau = 8.0f / c;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];
    const int64_t row_stride = (int64_t)H * D;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const int koff = col * Smem::kStrideK + half * 16;
    const int voff = (half * 4 + ((lane & 15) >> 2)) * Smem::kStrideV + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

    WorkCursor cursor;
    for (;;) {
        __syncthreads();
        if (tid == 0) sm.slot = next_work(s.counter, cursor, total);
        __syncthreads();
        const int64_t w = sm.slot;
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const __bf16 *kbase = k + t.row0 * row_stride + (int64_t)t.head * D;
        const __bf16 *vbase = v + t.row0 * row_stride + (int64_t)t.head * D;

        const int i0 = t.block * kFwdWideBlockRows + wave * 64 + col;   // query of column block 0; block 1 is +32
        const bool wave_active = t.block * kFwdWideBlockRows + wave * 64 < L;
        bf16x8 qreg[2][kKSteps];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int i = i0 + 32 * qb;
            const int iq = i < L ? i : L - 1;
            const __bf16 *qrow = q + (t.row0 + iq) * row_stride + (int64_t)t.head * D + 8 * half;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
        }

        f32x16 o[2][kDBlocks];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.0f;
        float m[2] = {-INFINITY, -INFINITY};
        float lsum[2] = {0.0f, 0.0f};

        // ---- staging: global -> registers (in flight during the compute) -> the other LDS buffer ----
        u32x4 kpre[kLoads], vpre[kLoads];
        const int my_r = tid / kChunksPerRow, my_cc = tid % kChunksPerRow;
        const __bf16 *kptr = kbase + (int64_t)my_r * row_stride + my_cc * 8;
        const __bf16 *vptr = vbase + (int64_t)my_r * row_stride + my_cc * 8;
        const int64_t pass_stride = (int64_t)kRowsPerPass * row_stride;
        const int64_t stage_stride = (int64_t)kWideBN * row_stride;
        auto prefetch = [&](int j0) {
            if (j0 + kWideBN <= L) {
#pragma unroll
                for (int u = 0; u < kLoads; ++u) {
                    kpre[u] = *reinterpret_cast<const u32x4 *>(kptr + u * pass_stride);
                    vpre[u] = *reinterpret_cast<const u32x4 *>(vptr + u * pass_stride);
                }
            } else {
#pragma unroll
                for (int u = 0; u < kLoads; ++u) {
                    const int r = my_r + u * kRowsPerPass;
                    const int j = j0 + r < L ? j0 + r : L - 1;
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
                const int r = my_r + u * kRowsPerPass;
                *reinterpret_cast<u32x4 *>(sm.k[buf] + r * Smem::kStrideK + my_cc * 16) = kpre[u];
                *reinterpret_cast<u32x4 *>(sm.v[buf] + r * Smem::kStrideV + my_cc * 16) = vpre[u];
            }
        };

        // ---- stage helpers (a stage = 64 keys = four units: column block qb x key block mb) ----
        auto load_k = [&](const char *kt, int mb, bf16x8 (&kop)[kKSteps]) {
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) kop[ks] = lds_read_b128(kt + mb * 32 * Smem::kStrideK + ks * 32);
        };
        auto load_v = [&](const char *vt, int mb, bf16x8 (&vop)[2][kDBlocks]) {
#pragma unroll
            for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *pv = vt + (mb * 32 + ts * 16) * Smem::kStrideV + db * 64;
                    vop[ts][db] = concat(lds_read_tr16(pv), lds_read_tr16(pv + 8 * Smem::kStrideV));
                }
        };
        // exponentials of one unit against the reference maximum; adds the rounded probabilities to `sum`
        auto exps = [&](const f32x16 &st, float mc, bf16x8 (&pb)[2], float &sum) {
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                u32x4 pw;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bf16x2 pr;
                    pr[0] = (__bf16)fast_exp2(fmaf(st[8 * ts + 2 * e], c, -mc));
                    pr[1] = (__bf16)fast_exp2(fmaf(st[8 * ts + 2 * e + 1], c, -mc));
                    sum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum, false);
                    pw[e] = __builtin_bit_cast(uint32_t, pr);
                }
                pb[ts] = __builtin_bit_cast(bf16x8, pw);
            }
        };

        prefetch(0);
        commit(0);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qreg[qb][ks]));   // Q loads complete here
        __syncthreads();

        // The hot loop never touches the output accumulators with VALU instructions.  When a stage's scores
        // exceed a reference maximum by more than 2^8 (always on the first stage, rarely afterwards) the
        // wave leaves the loop BEFORE the stage's barrier, raises the maxima, rescales, and re-enters the
        // loop at the same stage -- so every wave still passes exactly one barrier per stage.
        int buf = 0, j0 = 0;
        bool staged = false;      // the next stage's global loads are already in flight
        float mx0 = 0.0f, mx1 = 0.0f;
        for (;;) {
            bool raise = false;
            for (; j0 < L; j0 += kWideBN, buf ^= 1) {
                const bool more = j0 + kWideBN < L;
                if (more && !staged) prefetch(j0 + kWideBN);
                staged = true;
                if (wave_active) {
                    const char *kt = sm.k[buf] + koff;
                    const char *vt = sm.v[buf] + voff;
                    f32x16 st[2][2];   // [column block][key block]
                    const bool tail = j0 + kWideBN > L;
                    {
                        bf16x8 ka[kKSteps];
                        load_k(kt, 0, ka);
#pragma unroll
                        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                                for (int e = 0; e < 16; ++e) st[qb][mb][e] = 0.0f;
#pragma unroll
                        for (int ks = 0; ks < kKSteps; ++ks) {
                            st[0][0] = mfma_32x32x16(ka[ks], qreg[0][ks], st[0][0]);
                            st[1][0] = mfma_32x32x16(ka[ks], qreg[1][ks], st[1][0]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    {
                        // key block 1 runs on the matrix pipe while the maxima of key block 0 are taken
                        bf16x8 kb[kKSteps];
                        load_k(kt, 1, kb);
#pragma unroll
                        for (int ks = 0; ks < kKSteps; ++ks) {
                            st[0][1] = mfma_32x32x16(kb[ks], qreg[0][ks], st[0][1]);
                            st[1][1] = mfma_32x32x16(kb[ks], qreg[1][ks], st[1][1]);
                        }
                        if (tail) {
#pragma unroll
                            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                                for (int e = 0; e < 16; ++e)
                                    if (j0 + acc_row(e, half) >= L) st[qb][0][e] = -INFINITY;
                        }
                        mx0 = st[0][0][0];
                        mx1 = st[1][0][0];
#pragma unroll
                        for (int e = 1; e < 16; ++e) {
                            mx0 = fmaxf(mx0, st[0][0][e]);
                            mx1 = fmaxf(mx1, st[1][0][e]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (tail) {
#pragma unroll
                        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                            for (int e = 0; e < 16; ++e)
                                if (j0 + 32 + acc_row(e, half) >= L) st[qb][1][e] = -INFINITY;
                    }
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        mx0 = fmaxf(mx0, st[0][1][e]);
                        mx1 = fmaxf(mx1, st[1][1][e]);
                    }
                    mx0 = pair_max(mx0);
                    mx1 = pair_max(mx1);
                    if (__builtin_amdgcn_ballot_w64(mx0 > m[0] + tau || mx1 > m[1] + tau) != 0) {
                        raise = true;
                        break;
                    }
                    const float mc0 = m[0] * c, mc1 = m[1] * c;
                    bf16x8 vop[2][kDBlocks];
                    bf16x8 pb0[2], pb1[2];
                    load_v(vt, 0, vop);
                    exps(st[0][0], mc0, pb0, lsum[0]);
                    exps(st[1][0], mc1, pb1, lsum[1]);
#pragma unroll
                    for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                        for (int db = 0; db < kDBlocks; ++db) {
                            o[0][db] = mfma_32x32x16(vop[ts][db], pb0[ts], o[0][db]);
                            o[1][db] = mfma_32x32x16(vop[ts][db], pb1[ts], o[1][db]);
                        }
                    load_v(vt, 1, vop);
                    exps(st[0][1], mc0, pb0, lsum[0]);
                    exps(st[1][1], mc1, pb1, lsum[1]);
#pragma unroll
                    for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                        for (int db = 0; db < kDBlocks; ++db) {
                            o[0][db] = mfma_32x32x16(vop[ts][db], pb0[ts], o[0][db]);
                            o[1][db] = mfma_32x32x16(vop[ts][db], pb1[ts], o[1][db]);
                        }
                }
                if (more) commit(buf ^ 1);
                staged = false;
                __syncthreads();
            }
            if (!raise) break;
            {
                const float n0 = fmaxf(m[0], mx0), n1 = fmaxf(m[1], mx1);
                const float a0 = fast_exp2((m[0] - n0) * c), a1 = fast_exp2((m[1] - n1) * c);   // 0 on the first stage
                m[0] = n0;
                m[1] = n1;
                lsum[0] *= a0;
                lsum[1] *= a1;
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        o[0][db][e] *= a0;
                        o[1][db][e] *= a1;
                    }
            }
        }

        // ---- epilogue ----
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float l_total = pair_sum(lsum[qb]);
            const int i = i0 + 32 * qb;
            if (i < L) {
                const float inv = 1.0f / l_total;
                __bf16 *orow = out + (t.row0 + i) * row_stride + (int64_t)t.head * D;
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        bf16x4 x;
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = (__bf16)(o[qb][db][4 * g + e] * inv);
                        *reinterpret_cast<bf16x4 *>(orow + db * 32 + g * 8 + half * 4) = x;
                    }
                if (half == 0)
                    lse[(int64_t)t.head * sum_B + t.row0 + i] = (m[qb] * c + fast_log2(l_total)) * 0.6931471805599453f;
            }
        }
    }
}

hipError_t launch_fwd_bf16_wide(const void *q, const void *k, const void *v, const int64_t *offsets, int B, int H,
                                int D, Schedule s, void *out, float *lse, int cus, hipStream_t stream) {
#define JFA_CASE(DD)                                                                                              \
    case DD:                                                                                                      \
        hipLaunchKernelGGL(fwd_bf16_wide_kernel<DD>, dim3(persistent_grid<fwd_bf16_wide_kernel<DD>>(kWideThreads, cus)), \
                           dim3(kWideThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, \
                           offsets, B, H, s, (__bf16 *)out, lse);                                                 \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

}  // namespace jfa

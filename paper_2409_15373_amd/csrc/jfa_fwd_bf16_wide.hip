// Jagged flash attention forward, bf16, "wide" variant for long samples, D = 128 (paper Section 2.1).
//
// Same mathematics and operand layouts as fwd_bf16_kernel (transposed score tile S^T = K Q^T, a lane owns
// one query, V^T through the transposing LDS read).  What differs is the shape of the work and the pipeline:
//   * a workgroup is 256 queries; a wave owns 64 of them as two 32-query column blocks and runs alone on
//     its SIMD with the whole register file, so every K / V^T operand fetched from LDS feeds two matrix
//     products -- LDS traffic per flop is half that of the 32-query kernel, which is LDS-bound;
//   * K and V stages travel HBM/L2 -> LDS directly (global_load_lds_dwordx4), no staging registers; the
//     LDS tiles are unpadded and XOR-swizzled on 16-byte (K) / 64-byte (V) granules so that the 16-byte row
//     reads and the transposing reads are both conflict-free on the 64-bank LDS;
//   * inside a stage the matrix pipe never waits for the softmax: exponentials are taken against a FIXED
//     reference maximum per query (the maximum over the sample's first 32 keys) as soon as a score block is
//     ready, so the VALU works on key block 0 while the matrix pipe computes the scores of key block 1, and
//     on key block 1 while it accumulates O^T += V^T P^T of key block 0.  There is no running maximum, no
//     rescaling and no branch in the hot loop.  A reference below the true maximum only scales numerator
//     and denominator alike -- probabilities keep their relative precision in fp32 and in bf16 -- as long
//     as nothing overflows; a row sum above 2^62 (or not finite) at the end of the tile shows that it got
//     too stale, and the workgroup then redoes the tile in the conservative order (maximum first, online
//     rescaling).  On data whose scores are of one scale this second pass never runs.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kWideThreads = 256;
constexpr int kWideBN = 64;            // keys per LDS stage
constexpr int kWideD = 128;
constexpr int kWideTile = kWideBN * kWideD * 2;   // bytes of one K or V stage in LDS

template <int N> using Int = std::integral_constant<int, N>;

__device__ inline void dma16(const __bf16 *src, char *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

__global__ __launch_bounds__(kWideThreads, 1) void fwd_bf16_wide_kernel(const __bf16 *__restrict__ q,
                                                                        const __bf16 *__restrict__ k,
                                                                        const __bf16 *__restrict__ v,
                                                                        const int64_t *__restrict__ offsets, int B,
                                                                        int H, Schedule s, __bf16 *__restrict__ out,
                                                                        float *__restrict__ lse) {
    constexpr int D = kWideD;
    constexpr int kKSteps = D / 16;    // 8
    constexpr int kDBlocks = D / 32;   // 4
    // Separate arrays (not one indexed array) so that the compiler can tell the buffer being filled by the
    // DMA from the one being read and does not make the reads wait for the loads in flight.
    __shared__ __attribute__((aligned(1024))) char K0[kWideTile];
    __shared__ __attribute__((aligned(1024))) char K1[kWideTile];
    __shared__ __attribute__((aligned(1024))) char V0[kWideTile];
    __shared__ __attribute__((aligned(1024))) char V1[kWideTile];
    __shared__ __attribute__((aligned(1024))) char K2[kWideTile];   // third stage buffer: the DMA runs two stages ahead
    __shared__ __attribute__((aligned(1024))) char V2[kWideTile];
    __shared__ int64_t slot;
    __shared__ int restart;   // set by a wave whose reference maximum went stale beyond repair

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const float c = 1.4426950408889634f / sqrtf((float)D);
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];
    const int64_t row_stride = (int64_t)H * D;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    // ---- LDS read addresses (bytes inside a tile), fixed for the whole kernel ----
    // K element (row r, 16-byte chunk ch) sits at r * 256 + ((ch ^ (r & 15)) << 4).
    int kaddr[kKSteps];
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) kaddr[ks] = col * 256 + (((2 * ks + half) ^ (col & 15)) << 4);
    // V element (row r, 64-byte group g, byte b inside it) sits at r * 256 + ((g ^ (r & 3)) << 6) + b.
    // The transposing read of this lane: row = 4 half + (lane & 15) / 4 (+8 for the second half of the
    // operand, +16 per 16-key step), group = feature block db, bytes 32 * ((lane >> 4) & 1) + 8 * (lane & 3).
    int vaddr[kDBlocks];
    {
        const int r = half * 4 + ((lane & 15) >> 2);
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
            vaddr[db] = r * 256 + ((db ^ (r & 3)) << 6) + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
    }
    // ---- DMA: one instruction moves 64 lanes x 16 bytes = 4 rows; wave w, instruction u fills rows 16 w + 4 u .. +3.
    // Lane l lands on physical chunk l & 15 of row 16 w + 4 u + (l >> 4) and so fetches the logical chunk that
    // the swizzle puts there.
    const int dma_row0 = 16 * wave + (lane >> 4);
    const int pc = lane & 15;

    WorkCursor cursor;
    for (;;) {
        __syncthreads();
        if (tid == 0) slot = next_work(s.counter, cursor, total);
        __syncthreads();
        const int64_t w = uniform64(slot);
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const int n_stages = (L + kWideBN - 1) / kWideBN;
        const __bf16 *kbase = k + t.row0 * row_stride + (int64_t)t.head * D;
        const __bf16 *vbase = v + t.row0 * row_stride + (int64_t)t.head * D;

        // element offsets of this lane's four DMA chunks inside a full stage (K and V differ in the swizzle)
        int koffs[4], voffs[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = dma_row0 + 4 * u;
            koffs[u] = r * (int)row_stride + ((pc ^ (r & 15)) << 3);
            voffs[u] = r * (int)row_stride + ((pc ^ ((r & 3) << 2)) << 3);
        }
        auto issue = [&](const __bf16 *base, char *tile, int stage, bool is_k) {
            const int j0 = stage * kWideBN;
            const __bf16 *sbase = base + (int64_t)j0 * row_stride;
            if (j0 + kWideBN <= L) {
#pragma unroll
                for (int u = 0; u < 4; ++u) dma16(sbase + (is_k ? koffs[u] : voffs[u]), tile + (16 * wave + 4 * u) * 256);
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = dma_row0 + 4 * u;
                    const int ch = is_k ? (pc ^ (r & 15)) : (pc ^ ((r & 3) << 2));
                    const int jr = j0 + r < L ? r : L - 1 - j0;   // rows past the end repeat the last key (masked later)
                    dma16(sbase + (int64_t)jr * row_stride + ch * 8, tile + (16 * wave + 4 * u) * 256);
                }
            }
        };

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
        float m[2], lsum[2];

        // ---- helpers ----
        // S^T blocks of both column blocks for key block mb: operands are fetched four at a time, each feeding
        // two matrix products
        auto qk = [&](const char *tile, int mb, f32x16 &a, f32x16 &b) {
#pragma unroll
            for (int e = 0; e < 16; ++e) { a[e] = 0.0f; b[e] = 0.0f; }
#pragma unroll
            for (int k4 = 0; k4 < kKSteps; k4 += 4) {
                bf16x8 kop[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) kop[u] = lds_read_b128(tile + mb * 32 * 256 + kaddr[k4 + u]);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a = mfma_32x32x16(kop[u], qreg[0][k4 + u], a);
                    b = mfma_32x32x16(kop[u], qreg[1][k4 + u], b);
                }
            }
        };
        // O^T += V^T P^T of both column blocks for key block mb
        auto pv = [&](const char *tile, int mb, const bf16x8 (&pa)[2], const bf16x8 (&pb)[2]) {
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                bf16x8 vop[kDBlocks];
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *pvp = tile + (mb * 32 + ts * 16) * 256 + vaddr[db];
                    vop[db] = concat(lds_read_tr16(pvp), lds_read_tr16(pvp + 8 * 256));
                }
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    o[0][db] = mfma_32x32x16(vop[db], pa[ts], o[0][db]);
                    o[1][db] = mfma_32x32x16(vop[db], pb[ts], o[1][db]);
                }
            }
        };
        // exponentials of one unit (32 keys x 32 queries) against the reference maximum; the rounded
        // probabilities are what the second product uses, so they are what the row sum adds up
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
        auto mask = [&](f32x16 &st, int key0) {   // keys past the end of the sample
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (key0 + acc_row(e, half) >= L) st[e] = -INFINITY;
        };
        auto unit_max = [&](const f32x16 &a, float mx) {
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, a[e]);
            return mx;
        };

        // ---- stage pipeline ----
        // Stage j lives in buffer j & 1 (K and V alike); its DMA is issued at the top of stage j - 1 and has
        // landed for every wave after the barrier that ends stage j - 1.
        // pipelined(): fast order against the fixed reference maxima m[].
        auto pipelined = [&](auto PAR, auto RAGGED, int j) {
            constexpr int P = decltype(PAR)::value;   // buffer of this stage: j % 3
            constexpr bool kRagged = decltype(RAGGED)::value != 0;
            const char *const Kc = P == 0 ? K0 : (P == 1 ? K1 : K2);
            const char *const Vc = P == 0 ? V0 : (P == 1 ? V1 : V2);
            const float mc0 = m[0] * c, mc1 = m[1] * c;
            f32x16 sa[2], sb[2];        // scores: column block A / B, key block 0 / 1
            bf16x8 pa[2], pb[2];
            bf16x8 k0[kKSteps], k1[kKSteps], v0[2][kDBlocks], v1[2][kDBlocks];
            // operand fetches, each issued one phase before its matrix products
            auto fetch_k = [&](int mb, bf16x8 (&kop)[kKSteps]) {
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) kop[ks] = lds_read_b128(Kc + mb * 32 * 256 + kaddr[ks]);
            };
            auto fetch_v = [&](int mb, bf16x8 (&vop)[2][kDBlocks]) {
#pragma unroll
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) {
                        const char *pvp = Vc + (mb * 32 + ts * 16) * 256 + vaddr[db];
                        vop[ts][db] = concat(lds_read_tr16(pvp), lds_read_tr16(pvp + 8 * 256));
                    }
            };
            auto scores = [&](const bf16x8 (&kop)[kKSteps], f32x16 &x, f32x16 &y) {
#pragma unroll
                for (int e = 0; e < 16; ++e) { x[e] = 0.0f; y[e] = 0.0f; }
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) {
                    x = mfma_32x32x16(kop[ks], qreg[0][ks], x);
                    y = mfma_32x32x16(kop[ks], qreg[1][ks], y);
                }
            };
            auto accumulate = [&](const bf16x8 (&vop)[2][kDBlocks]) {
#pragma unroll
                for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                    for (int db = 0; db < kDBlocks; ++db) {
                        o[0][db] = mfma_32x32x16(vop[ts][db], pa[ts], o[0][db]);
                        o[1][db] = mfma_32x32x16(vop[ts][db], pb[ts], o[1][db]);
                    }
            };
            // phase 1: scores of key block 0                         | LDS: K operands of key block 1
            fetch_k(0, k0);
            fetch_k(1, k1);
            scores(k0, sa[0], sb[0]);
            // phase 2: scores of key block 1                         | VALU: exponentials of key block 0; LDS: V^T of block 0
            fetch_v(0, v0);
            scores(k1, sa[1], sb[1]);
            if (kRagged) { mask(sa[0], j * kWideBN); mask(sb[0], j * kWideBN); }
            exps(sa[0], mc0, pa, lsum[0]);
            exps(sb[0], mc1, pb, lsum[1]);
            // phase 3: O^T += V^T P^T of key block 0                 | VALU: exponentials of key block 1; LDS: V^T of block 1
            fetch_v(1, v1);
            accumulate(v0);
            if (kRagged) { mask(sa[1], j * kWideBN + 32); mask(sb[1], j * kWideBN + 32); }
            exps(sa[1], mc0, pa, lsum[0]);
            exps(sb[1], mc1, pb, lsum[1]);
            // phase 4: O^T += V^T P^T of key block 1
            accumulate(v1);
        };
        // conservative(): maximum first, rescale, then exponentials; used when a tile had to be restarted.
        auto conservative = [&](int par, int j) {
            const char *const Kc = par ? K1 : K0;
            const char *const Vc = par ? V1 : V0;
            f32x16 sa[2], sb[2];
            bf16x8 pa[2], pb[2];
            qk(Kc, 0, sa[0], sb[0]);
            qk(Kc, 1, sa[1], sb[1]);
            if ((j + 1) * kWideBN > L) {
                mask(sa[0], j * kWideBN); mask(sb[0], j * kWideBN);
                mask(sa[1], j * kWideBN + 32); mask(sb[1], j * kWideBN + 32);
            }
            const float x0 = pair_max(unit_max(sa[1], unit_max(sa[0], -INFINITY)));
            const float x1 = pair_max(unit_max(sb[1], unit_max(sb[0], -INFINITY)));
            const float n0 = fmaxf(m[0], x0), n1 = fmaxf(m[1], x1);
            const float a0 = fast_exp2((m[0] - n0) * c), a1 = fast_exp2((m[1] - n1) * c);   // 0 on the first stage
            m[0] = n0;
            m[1] = n1;
            lsum[0] *= a0;
            lsum[1] *= a1;
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) { o[0][db][e] *= a0; o[1][db][e] *= a1; }
            exps(sa[0], n0 * c, pa, lsum[0]);
            exps(sb[0], n1 * c, pb, lsum[1]);
            pv(Vc, 0, pa, pb);
            exps(sa[1], n0 * c, pa, lsum[0]);
            exps(sb[1], n1 * c, pb, lsum[1]);
            pv(Vc, 1, pa, pb);
        };

        auto start_tile = [&]() {   // stage 0 into LDS, state cleared
            if (tid == 0) restart = 0;
            issue(kbase, K0, 0, true);
            issue(vbase, V0, 0, false);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qreg[qb][ks]));   // Q loads complete here
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's DMA has landed
            __syncthreads();
            m[0] = m[1] = -INFINITY;
            lsum[0] = lsum[1] = 0.0f;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.0f;
        };
        auto issue_next = [&](int j) {
            if (j + 1 < n_stages) {
                issue(kbase, (j & 1) ? K0 : K1, j + 1, true);
                issue(vbase, (j & 1) ? V0 : V1, j + 1, false);
            }
        };
        auto end_stage = [&]() {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's DMA has landed
            __syncthreads();
        };

        // ---- pass 1: pipelined, three stage buffers, DMA two stages ahead ----
        // Stage j lives in buffer j % 3.  At the top of stage j the DMA of stage j + 2 is issued into the buffer
        // that stage j - 1 has just released; at the end of stage j each wave waits until only those newest
        // eight DMA operations are outstanding (so stage j + 1 has landed) and meets the others at a bare
        // s_barrier -- not __syncthreads(), whose release fence would wait for every load in flight.
        auto issue_stage = [&](auto BUF, int j) {
            constexpr int Bf = decltype(BUF)::value;
            issue(kbase, Bf == 0 ? K0 : (Bf == 1 ? K1 : K2), j, true);
            issue(vbase, Bf == 0 ? V0 : (Bf == 1 ? V1 : V2), j, false);
        };
        auto run_stage = [&](auto BUF, auto RAGGED, int j) {
            constexpr int Bf = decltype(BUF)::value;
            const bool ahead = j + 2 < n_stages;
            if (ahead) issue_stage(Int<(Bf + 2) % 3>{}, j + 2);
            if (wave_active) pipelined(BUF, RAGGED, j);
            asm volatile("" ::: "memory");
            if (ahead) __builtin_amdgcn_s_waitcnt(0x0078);   // vmcnt(8) lgkmcnt(0)
            else __builtin_amdgcn_s_waitcnt(0x0070);         // vmcnt(0) lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        };

        if (tid == 0) restart = 0;
        issue_stage(Int<0>{}, 0);
        if (n_stages > 1) issue_stage(Int<1>{}, 1);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qreg[qb][ks]));   // Q loads complete here
        if (n_stages > 1) __builtin_amdgcn_s_waitcnt(0x0078); else __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        m[0] = m[1] = -INFINITY;
        lsum[0] = lsum[1] = 0.0f;
        if (wave_active) {   // reference maxima: the first 32 keys
            f32x16 sa, sb;
            qk(K0, 0, sa, sb);
            if (L < 32) { mask(sa, 0); mask(sb, 0); }
            m[0] = pair_max(unit_max(sa, -INFINITY));
            m[1] = pair_max(unit_max(sb, -INFINITY));
        }
        {
            const int n_full = L / kWideBN;   // stages with all 64 keys valid; a ragged one may follow
            int j = 0;
            for (; j + 3 <= n_full; j += 3) {
                run_stage(Int<0>{}, Int<0>{}, j);
                run_stage(Int<1>{}, Int<0>{}, j + 1);
                run_stage(Int<2>{}, Int<0>{}, j + 2);
            }
            if (j < n_full) { run_stage(Int<0>{}, Int<0>{}, j); ++j; }
            if (j < n_full) { run_stage(Int<1>{}, Int<0>{}, j); ++j; }
            if (j < n_stages) {               // the ragged last stage, in buffer n_full % 3
                const int r = n_full % 3;
                if (r == 0) run_stage(Int<0>{}, Int<1>{}, j);
                else if (r == 1) run_stage(Int<1>{}, Int<1>{}, j);
                else run_stage(Int<2>{}, Int<1>{}, j);
            }
        }
        // a row sum this large (or not finite) means the fixed reference was too far below the true maximum
        {
            const bool bad = !(lsum[0] < 0x1p62f) || !(lsum[1] < 0x1p62f);
            if (wave_active && __builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) restart = 1;
        }
        __syncthreads();
        const bool again = restart != 0;

        // ---- pass 2 (never on data of one scale): the whole tile again, maximum first ----
        if (again) {
            __syncthreads();   // every wave has seen `restart` before it is cleared
            start_tile();
            for (int j = 0; j < n_stages; ++j) {
                issue_next(j);
                if (wave_active) conservative(j & 1, j);
                end_stage();
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

bool fwd_bf16_wide_supported(int D) { return D == kWideD; }

hipError_t launch_fwd_bf16_wide(const void *q, const void *k, const void *v, const int64_t *offsets, int B, int H,
                                int D, Schedule s, void *out, float *lse, int cus, hipStream_t stream) {
    if (D != kWideD) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fwd_bf16_wide_kernel, dim3(persistent_grid<fwd_bf16_wide_kernel>(kWideThreads, cus)),
                       dim3(kWideThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, offsets,
                       B, H, s, (__bf16 *)out, lse);
    return hipGetLastError();
}

}  // namespace jfa

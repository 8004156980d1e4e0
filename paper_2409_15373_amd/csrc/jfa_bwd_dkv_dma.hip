// Jagged flash attention backward, bf16, D = 128, long samples: dK and dV in ONE kernel (paper Section 2.2).
//
//   P = exp(S / sqrt(D) - lse),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dK = dS^T Q / sqrt(D)
//
// The two gradients of a block of keys need four matrix products (S, dV, dP, dK); computed in two kernels they need
// five, because each kernel recomputes S.  Both accumulators of 32 keys do not fit one wave at two waves per SIMD, so
// the work of 32 keys is shared by a PAIR of waves that sit on the same SIMD:
//   wave A (waves 0..3)   S = Q K^T from the streamed queries and its stationary K rows, P = exp2(c S - lse'),
//                         hands P (rounded to bf16, the operand of its own second product) to its partner
//                         through LDS, and accumulates dV^T += dO^T P;
//   wave B (waves 4..7)   dP = dO V^T with its stationary V rows (negated, accumulator started at delta),
//                         takes P from LDS, dS = P o (dP - delta), and accumulates dK^T += Q^T dS.
// A workgroup is four pairs = 128 keys; queries and dO stream through three XOR-swizzled LDS stage buffers filled by
// global_load_lds two stages ahead, one s_barrier per stage, as in the other direct-to-LDS kernels.  Inside a stage
// the hand-over of a 32 x 32 block of P is a sequence number in LDS that A bumps after writing the block and B polls
// before reading it; A never waits for B (the block buffers alternate with the stage's parity and a stage's barrier
// separates their reuse), so every wait ends.  The dependency also makes the pair alternate: while A takes
// exponentials B runs matrix products and the other way round.
// Layouts are those of bwd_bf16_dma_kernel: streamed rows on the MFMA row axis, stationary keys on the lane axis, so
// P and dS leave the accumulators in operand position, and A's and B's lanes hold the same (query, key) elements.
#include "jfa_bwd_dma.h"

namespace jfa {

constexpr int kDkvPairs = 4;                       // pairs of waves per workgroup
constexpr int kPxBlock = 2048;                     // bytes of one 32 x 32 block of bf16 probabilities
constexpr int kPxStage = 2 * kPxBlock;             // two blocks per stage
constexpr int kPxPair = 2 * kPxStage;              // two stages in flight (parity of the stage index)

// LDS accesses with explicit instructions (address = byte offset inside the workgroup's LDS).  Every access to LDS
// that is not the target of a global -> LDS copy goes through these: for such an access the compiler inserts a wait
// for ALL copies in flight (it cannot prove that the location is not one of their targets), which would stall each
// stage on the loads that are meant to stay two stages ahead.  An instruction the compiler does not count only makes
// its own LDS waits more conservative (LDS returns in order); the reads below wait for their results themselves.
__device__ inline uint32_t lds_address(const void *p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}
__device__ inline void lds_store_u32(uint32_t addr, uint32_t value) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(value) : "memory");
}
__device__ inline uint32_t lds_load_u32(uint32_t addr) {
    uint32_t value;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(value) : "v"(addr) : "memory");
    return value;
}
typedef __attribute__((ext_vector_type(4))) float f32x4;
__device__ inline void lds_load_4x_b128(uint32_t addr, f32x4 &a, f32x4 &b, f32x4 &c, f32x4 &d) {   // at addr + 0, 32, 64, 96
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:32\n\tds_read_b128 %2, %4 offset:64\n\t"
                 "ds_read_b128 %3, %4 offset:96\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d) : "v"(addr) : "memory");
}
__device__ inline void lds_store_2x_b128(uint32_t addr, u32x4 lo, u32x4 hi) {   // lo at addr, hi at addr + 1024
    asm volatile("ds_write_b128 %0, %1\n\tds_write_b128 %0, %2 offset:1024" : : "v"(addr), "v"(lo), "v"(hi) : "memory");
}
__device__ inline void lds_load_2x_b128(uint32_t addr, u32x4 &lo, u32x4 &hi) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:1024\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(lo), "=&v"(hi) : "v"(addr) : "memory");
}

__global__ __launch_bounds__(kBdThreads, 2) void bwd_dkv_dma_kernel(const __bf16 *__restrict__ q,
                                                                    const __bf16 *__restrict__ k,
                                                                    const __bf16 *__restrict__ v,
                                                                    const __bf16 *__restrict__ dout,
                                                                    const float *__restrict__ stats,   // [2, H, sum_B]: delta, -lse * sqrt(D)
                                                                    const int64_t *__restrict__ offsets, int B, int H,
                                                                    Schedule s, __bf16 *__restrict__ dk,
                                                                    __bf16 *__restrict__ dv) {
    constexpr int D = kBdD;
    constexpr int kKSteps = D / 16;
    constexpr int kDBlocks = D / 32;
    // Three stages, each the streamed Q rows followed by the streamed dO rows.  One array per stage (not per tile): the
    // compiler keeps apart only a handful of targets of global -> LDS copies, and reads of a target beyond that number
    // wait for every copy in flight instead of their own stage's.
    __shared__ __attribute__((aligned(1024))) char T0[2 * kBdTile];
    __shared__ __attribute__((aligned(1024))) char T1[2 * kBdTile];
    __shared__ __attribute__((aligned(1024))) char T2[2 * kBdTile];
    char *const A0 = T0, *const A1 = T1, *const A2 = T2;
    char *const B0 = T0 + kBdTile, *const B1 = T1 + kBdTile, *const B2 = T2 + kBdTile;
    // Per stage: -lse * sqrt(D) [64] and delta [64] of the streamed rows (six targets of global -> LDS copies in all: the
    // compiler keeps apart only a handful, and reads of a target beyond that number wait for every copy in flight).
    __shared__ __attribute__((aligned(256))) char S0[512];
    __shared__ __attribute__((aligned(256))) char S1[512];
    __shared__ __attribute__((aligned(256))) char S2[512];
    __shared__ __attribute__((aligned(1024))) char Px[kDkvPairs * kPxPair];   // P blocks on their way from A to B
    __shared__ int handed[kDkvPairs];   // per pair: number of P blocks A has written since the kernel started
    __shared__ WorkSlot slot;
    __shared__ LdsSchedule<false> tab;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int pair = wave & 3;
    const bool is_a = wave < 4;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];
    const int64_t row_stride = (int64_t)H * D;

    // LDS read addresses inside a stage tile: one of each kind is kept, the others differ by constant bit patterns
    const int raddr0 = col * 256 + ((half ^ swz(col)) << 4);   // 16-byte row reads: row = col (+32 per block), chunk 2 ks + half
    int taddr0;                                                // transposing reads: row = 4 half + (lane & 15) / 4 (+8 for the operand's second half)
    {
        const int r = half * 4 + ((lane & 15) >> 2);
        const int chunk_in_group = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1), byte_in_chunk = (lane & 1) * 8;
        taddr0 = r * 256 + ((chunk_in_group ^ swz(r)) << 4) + byte_in_chunk;
    }
    const uint32_t px_pair = lds_address(Px) + pair * kPxPair;
    const uint32_t handed_addr = lds_address(&handed[pair]);

    struct Stream {
        const __bf16 *abase, *bbase;
        const float *delta_rows, *lse2_rows;
        int L, n_stages;
    };
    auto stream_of = [&](const Work &w) {
        Stream st;
        st.L = w.len;
        st.n_stages = (st.L + kBdBN - 1) / kBdBN;
        const int64_t head_off = w.row0 * row_stride + (int64_t)w.head * D;
        st.abase = q + head_off;
        st.bbase = dout + head_off;
        st.delta_rows = stats + (int64_t)w.head * sum_B + w.row0;
        st.lse2_rows = stats + (int64_t)(H + w.head) * sum_B + w.row0;
        return st;
    };
    // per-lane DMA offsets are rebuilt at every issue (values used once per stage are the first to be spilled)
    auto issue_from = [&](const Stream &st, const __bf16 *base, char *tile, int stage) {
        const int L = st.L;
        const int j0 = stage * kBdBN;
        const __bf16 *sbase = base + (int64_t)j0 * row_stride;
        int t_opaque = tid;
        asm volatile("" : "+v"(t_opaque));
        const int dma_row0 = 8 * wave + ((t_opaque >> 4) & 3);
        const int pc = t_opaque & 15;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int r = dma_row0 + 4 * u;
            const int jr = j0 + r < L ? r : L - 1 - j0;   // rows past the end repeat the last row (their P is zeroed)
            bd_dma16(sbase, 2u * (uint32_t)(jr * (int)row_stride + ((pc ^ swz(r)) << 3)), tile + (8 * wave + 4 * u) * 256);
        }
    };
    auto issue_stage_from = [&](const Stream &st, auto BUF, int j) {
        constexpr int Bf = decltype(BUF)::value;
        issue_from(st, st.abase, Bf == 0 ? A0 : (Bf == 1 ? A1 : A2), j);
        issue_from(st, st.bbase, Bf == 0 ? B0 : (Bf == 1 ? B1 : B2), j);
        {   // lse and delta of the 64 streamed rows.  Every wave copies them (to the same place, the same values): with
            // the copies on one wave only, the waves would differ in their count of copies in flight, and the compiler,
            // which sees one program for all of them, would protect each stage's reads with a wait for everything.
            // destinations as LDS pointers from the start: a generic pointer plus an offset is cast with a null check,
            // after which the compiler no longer knows which array the copy goes to
            typedef __attribute__((address_space(3))) char lds_char;
            lds_char *st_lds = (lds_char *)(Bf == 0 ? S0 : (Bf == 1 ? S1 : S2));
            const int j0 = j * kBdBN;
            const uint32_t jj = 4u * (uint32_t)(j0 + lane < st.L ? j0 + lane : st.L - 1);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)((const char *)st.lse2_rows + jj),
                                             (__attribute__((address_space(3))) void *)st_lds, 4, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)((const char *)st.delta_rows + jj),
                                             (__attribute__((address_space(3))) void *)(st_lds + 256), 4, 0, 0);
        }
    };
    // stationary rows of the pair: K for wave A, V for wave B (rows past the end of the sample repeat its last row)
    bf16x8 sreg[kKSteps];
    auto load_stationary = [&](const Work &w) {
        const int iw = w.block * kDkvBlockRows + pair * 32 + col;
        const int64_t off = (w.row0 + (iw < w.len ? iw : w.len - 1)) * row_stride + (int64_t)w.head * D + 8 * half;
        const __bf16 *src = is_a ? k : v;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) sreg[ks] = *reinterpret_cast<const bf16x8 *>(src + off + 16 * ks);
    };

    const bool tabled = B <= kTabCap;
    WorkCursor cursor;
    auto claim_next = [&]() {   // wave 0, every lane
        if (!tabled) {
            claim_and_decode(&slot, s, offsets, B, H, total, cursor, nullptr);
            return;
        }
        int64_t w = -1;
        if (lane == 0) w = next_work(s.counter, cursor, total);
        tab.decode(&slot, B, H, uniform64(w));
    };
    if (tid < kDkvPairs) handed[tid] = 0;
    if (wave == 0) claim_and_decode(&slot, s, offsets, B, H, total, cursor, nullptr);
    if (tabled) tab.fill(s, offsets, nullptr, B);
    __syncthreads();
    uint32_t blocks_done = 0;   // P blocks this wave has written (A) or taken (B) since the kernel started
    Work t;
    bool have = load_work<false>(&slot, t);
    while (have) {
        __syncthreads();   // every wave has read the slot before wave 0 refills it
        const Stream cur = stream_of(t);
        const int Ls = t.len;
        const int L = cur.L;
        const int tile0 = t.block * kDkvBlockRows;
        const int n_stages = cur.n_stages;
        const bool wave_active = tile0 + pair * 32 < Ls;
        load_stationary(t);
        issue_stage_from(cur, IntB<0>{}, 0);
        if (n_stages > 1) issue_stage_from(cur, IntB<1>{}, 1);
        if (wave == 0) claim_next();   // overlaps with the loads in flight
        f32x16 acc[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[db][e] = 0.0f;

        auto addresses = [&](int (&ra)[kKSteps], int (&ta)[2][kDBlocks]) {
            int rb = raddr0, tb = taddr0;
            asm volatile("" : "+v"(rb), "+v"(tb));   // rebuilt per block, not hoisted and spilled
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) ra[ks] = rb ^ (ks << 5);
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db) {
                ta[0][db] = tb ^ (db << 6);
                ta[1][db] = (tb ^ (db << 6) ^ 32) + 2048;
            }
        };
        // accumulator <- row statistics of the 32 streamed rows of block mb (four 16-byte LDS reads), then the
        // product of the block's streamed rows (row reads of `tile`) with this wave's stationary rows
        auto product = [&](const char *tile, const char *st_plane, int mb, f32x16 &a) {
            int ra[kKSteps], ta[2][kDBlocks];
            addresses(ra, ta);
#pragma unroll
            for (int k4 = 0; k4 < kKSteps; k4 += 4) {
                bf16x8 op[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) op[u] = lds_read_b128(tile + mb * 32 * 256 + ra[k4 + u]);
                if (k4 == 0) {   // the first operands are on their way when the statistics are asked for (and waited for)
                    f32x4 x0, x1, x2, x3;
                    int h_opaque = half;
                    asm volatile("" : "+v"(h_opaque));
                    lds_load_4x_b128(lds_address(st_plane) + mb * 128 + h_opaque * 16, x0, x1, x2, x3);
                    a = __builtin_shufflevector(__builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7),
                                                __builtin_shufflevector(x2, x3, 0, 1, 2, 3, 4, 5, 6, 7),
                                                0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) a = mfma_32x32x16(op[u], sreg[k4 + u], a);
            }
        };
        // acc^T += (streamed tile)^T x, contraction over the block's 32 streamed rows in two steps of 16
        auto accumulate = [&](const char *tile, int mb, const bf16x8 (&x)[2]) {
            int ra[kKSteps], ta[2][kDBlocks];
            addresses(ra, ta);
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                bf16x8 top[kDBlocks];
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *base = tile + (mb * 32 + ts * 16) * 256;
                    top[db] = concat(lds_read_tr16(base + ta[0][db]), lds_read_tr16(base + ta[1][db]));
                }
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) acc[db] = mfma_32x32x16(top[db], x[ts], acc[db]);
            }
        };
        // where block mb of stage j travels: [stage parity][block][half of the lane's sixteen values][lane]
        auto px_slot = [&](int j, int mb) {
            int l_opaque = lane;
            asm volatile("" : "+v"(l_opaque));
            return px_pair + (uint32_t)((j & 1) * kPxStage + mb * kPxBlock + l_opaque * 16);
        };

        // ---- wave A: one block of 32 streamed queries ----
        auto a_scores = [&](auto RAGGED, const char *At, const char *St, int mb, int j, bf16x8 (&p)[2]) {
            constexpr bool ragged = decltype(RAGGED)::value != 0;
            f32x16 sc;
            product(At, St, mb, sc);   // dot products minus lse * sqrt(D) of the streamed rows
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float pe = fast_exp2(sc[e] * c);
                if (ragged && j * kBdBN + mb * 32 + (e >> 2) * 8 + half * 4 + (e & 3) >= L) pe = 0.0f;   // past the sample's end
                sc[e] = pe;
            }
            p[0] = pack_bf16(sc, 0);
            p[1] = pack_bf16(sc, 8);
            // the block is written before it is announced: LDS keeps a wave's operations in order
            lds_store_2x_b128(px_slot(j, mb), __builtin_bit_cast(u32x4, p[0]), __builtin_bit_cast(u32x4, p[1]));
            ++blocks_done;
            lds_store_u32(handed_addr, blocks_done);
        };
        // ---- wave B: dS of one block from its dP accumulator and the partner's P ----
        auto b_take = [&](int mb, int j, const f32x16 &dp, bf16x8 (&ds)[2]) {
            ++blocks_done;
            for (;;) {
                if ((int32_t)(lds_load_u32(handed_addr) - blocks_done) >= 0) break;
                __builtin_amdgcn_s_sleep(1);
            }
            u32x4 lo, hi;
            lds_load_2x_b128(px_slot(j, mb), lo, hi);
            f32x16 x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {   // bf16 pairs -> fp32, times (delta - dP) = -dS (the sign goes into the output scale)
                x[2 * e] = __uint_as_float(lo[e] << 16) * dp[2 * e];
                x[2 * e + 1] = __uint_as_float(lo[e] & 0xffff0000u) * dp[2 * e + 1];
                x[8 + 2 * e] = __uint_as_float(hi[e] << 16) * dp[8 + 2 * e];
                x[8 + 2 * e + 1] = __uint_as_float(hi[e] & 0xffff0000u) * dp[8 + 2 * e + 1];
            }
            ds[0] = pack_bf16(x, 0);
            ds[1] = pack_bf16(x, 8);
        };

        // vmcnt(copies of one stage) lgkmcnt(0): four tile copies and two statistics copies per wave and stage
        auto wait_one_stage_outstanding = [&]() { __builtin_amdgcn_s_waitcnt(0x0070 | 6); };
        // SURE: the caller knows that stage j + 2 exists (the copies are then sent unconditionally, and the compiler,
        // which counts copies in flight along every path, does not have to protect this stage's reads against the
        // path on which they were not sent with a wait for everything)
        // ROLE_A: the stage as wave A or as wave B runs it.  The role is fixed for the whole tile outside the stage loop:
        // a branch on it inside a stage would merge the two roles' accumulators after every stage, at the price of
        // register copies of all 64 of them.
        auto run_stage = [&](auto ROLE_A, auto BUF, auto RAGGED, auto SURE, int j) {
            constexpr bool role_a = decltype(ROLE_A)::value != 0;
            constexpr int Bf = decltype(BUF)::value;
            constexpr bool ragged = decltype(RAGGED)::value != 0;
            const bool ahead = decltype(SURE)::value != 0 || j + 2 < n_stages;
            if (ahead) issue_stage_from(cur, IntB<(Bf + 2) % 3>{}, j + 2);
            if (wave_active) {
                const char *At = Bf == 0 ? A0 : (Bf == 1 ? A1 : A2);
                const char *Bt = Bf == 0 ? B0 : (Bf == 1 ? B1 : B2);
                const char *St = Bf == 0 ? S0 : (Bf == 1 ? S1 : S2);
                const bool second = !ragged || j * kBdBN + 32 < L;   // the sample's last stage may hold one block only
                if (role_a) {
                    bf16x8 p0[2], p1[2];
                    a_scores(RAGGED, At, St, 0, j, p0);
                    if (second) a_scores(RAGGED, At, St, 1, j, p1);
                    accumulate(Bt, 0, p0);               // dV^T += dO^T P
                    if (second) accumulate(Bt, 1, p1);
                } else {
                    f32x16 dp0, dp1;
                    bf16x8 ds[2];
                    product(Bt, St + 256, 0, dp0);       // delta - dO V^T (V is held negated)
                    if (second) product(Bt, St + 256, 1, dp1);
                    b_take(0, j, dp0, ds);
                    accumulate(At, 0, ds);               // dK^T -= Q^T dS
                    if (second) {
                        b_take(1, j, dp1, ds);
                        accumulate(At, 1, ds);
                    }
                }
            }
            asm volatile("" ::: "memory");
            if (ahead) wait_one_stage_outstanding(); else __builtin_amdgcn_s_waitcnt(0x0070);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        };

#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(sreg[ks]));   // stationary-row loads complete here
        if (!is_a) {   // V enters negated: the dP accumulator starts at delta and ends as delta - dP
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                u32x4 w = __builtin_bit_cast(u32x4, sreg[ks]);
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] ^= 0x80008000u;
                sreg[ks] = __builtin_bit_cast(bf16x8, w);
            }
        }
        if (n_stages > 1) wait_one_stage_outstanding(); else __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        auto all_stages = [&](auto ROLE_A) {
            const int n_full = L / kBdBN;   // stages with all 64 streamed rows valid; a ragged one may follow
            int j = 0;
            // Six stages per trip where they exist: the first stage of a loop body is compiled with a wait for every
            // copy in flight (the compiler's bookkeeping of copies is at its most cautious where the loop closes), so
            // the longer body halves how often that wait is met.
            for (; j + 8 <= n_stages; j += 6) {
                run_stage(ROLE_A, IntB<0>{}, IntB<0>{}, IntB<1>{}, j);
                run_stage(ROLE_A, IntB<1>{}, IntB<0>{}, IntB<1>{}, j + 1);
                run_stage(ROLE_A, IntB<2>{}, IntB<0>{}, IntB<1>{}, j + 2);
                run_stage(ROLE_A, IntB<0>{}, IntB<0>{}, IntB<1>{}, j + 3);
                run_stage(ROLE_A, IntB<1>{}, IntB<0>{}, IntB<1>{}, j + 4);
                run_stage(ROLE_A, IntB<2>{}, IntB<0>{}, IntB<1>{}, j + 5);
            }
            for (; j + 5 <= n_stages; j += 3) {   // three full stages, and the two after them exist
                run_stage(ROLE_A, IntB<0>{}, IntB<0>{}, IntB<1>{}, j);
                run_stage(ROLE_A, IntB<1>{}, IntB<0>{}, IntB<1>{}, j + 1);
                run_stage(ROLE_A, IntB<2>{}, IntB<0>{}, IntB<1>{}, j + 2);
            }
            for (; j < n_stages; ++j) {           // the last stages (at most four), stage j in buffer j % 3
                const int r = j % 3;
                if (j < n_full) {
                    if (r == 0) run_stage(ROLE_A, IntB<0>{}, IntB<0>{}, IntB<0>{}, j);
                    else if (r == 1) run_stage(ROLE_A, IntB<1>{}, IntB<0>{}, IntB<0>{}, j);
                    else run_stage(ROLE_A, IntB<2>{}, IntB<0>{}, IntB<0>{}, j);
                } else {                          // the ragged one
                    if (r == 0) run_stage(ROLE_A, IntB<0>{}, IntB<1>{}, IntB<0>{}, j);
                    else if (r == 1) run_stage(ROLE_A, IntB<1>{}, IntB<1>{}, IntB<0>{}, j);
                    else run_stage(ROLE_A, IntB<2>{}, IntB<1>{}, IntB<0>{}, j);
                }
            }
        };
        if (is_a) all_stages(IntB<1>{}); else all_stages(IntB<0>{});

        Work nt;   // the next work item: wave 0 parked it in the slot before this tile's first barrier
        const bool have_next = load_work<false>(&slot, nt);

        // ---- epilogue: scale, transpose the wave's 32 x 128 gradient block through LDS, 64 features at a time, and
        // store whole 128-byte pieces of rows.  The stage buffers are idle (every wave is past the last stage's barrier,
        // no DMA is in flight, the next tile's loads start behind the barrier at the top of the loop); wave w uses 4 KB
        // of the third pair: row r of its block at r * 128, 16-byte chunk ch at (ch ^ (r & 7)) << 4.
        {
            char *const region = (is_a ? A2 : B2) + pair * 4096;
            const float out_scale = is_a ? 1.0f : -scale;
            int lane_e = lane;
            asm volatile("" : "+v"(lane_e));
            const int col_e = lane_e & 31, half_e = lane_e >> 5;
            const int wbase = col_e * 128 + ((half_e * 8) ^ ((col_e & 7) << 4));
            const int r0 = tile0 + pair * 32;   // first key of this pair
            __bf16 *const gbase = (is_a ? dv : dk) + (t.row0 + r0) * row_stride + (int64_t)t.head * D;
            const uint32_t lane_off = 2u * (uint32_t)((lane_e >> 3) * (int)row_stride + (lane_e & 7) * 8);
#pragma unroll
            for (int f = 0; f < 2; ++f) {
#pragma unroll
                for (int dl = 0; dl < 2; ++dl)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        bf16x4 x;
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = (__bf16)(acc[2 * f + dl][4 * g + e] * out_scale);
                        *reinterpret_cast<bf16x4 *>(region + (wbase ^ (dl * 64 + g * 16))) = x;
                    }
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int r = it * 8 + (lane_e >> 3);
                    const u32x4 rowpiece = *reinterpret_cast<const u32x4 *>(region + r * 128 + (((lane_e & 7) ^ (r & 7)) << 4));
                    char *dst = reinterpret_cast<char *>(gbase + (int64_t)it * 8 * row_stride + 64 * f) + lane_off;
                    if (r0 + r < Ls) *reinterpret_cast<u32x4 *>(dst) = rowpiece;
                }
            }
        }
        t = nt;
        have = have_next;
    }
}

hipError_t launch_bwd_dkv_dma(const void *q, const void *k, const void *v, const void *dout, const float *stats,
                              const int64_t *offsets, int B, int H, int D, Schedule s, void *dk, void *dv, int cus,
                              hipStream_t stream) {
    if (D != kBdD) return hipErrorInvalidValue;
    hipLaunchKernelGGL(bwd_dkv_dma_kernel, dim3(persistent_grid<bwd_dkv_dma_kernel>(kBdThreads, cus)), dim3(kBdThreads), 0,
                       stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, (const __bf16 *)dout, stats, offsets, B,
                       H, s, (__bf16 *)dk, (__bf16 *)dv);
    return hipGetLastError();
}

}  // namespace jfa

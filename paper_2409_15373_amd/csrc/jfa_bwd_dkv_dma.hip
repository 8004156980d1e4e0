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
// Layouts are those of bwd_dq_dma_kernel: streamed rows on the MFMA row axis, stationary keys on the lane axis, so
// P and dS leave the accumulators in operand position, and A's and B's lanes hold the same (query, key) elements.
#include "jfa_bwd_dma.h"

namespace jfa {

constexpr int kDkvPairs = 4;                       // pairs of waves per workgroup
constexpr int kPxBlock = 2048;                     // bytes of one 32 x 32 block of bf16 probabilities
constexpr int kPxStage = 2 * kPxBlock;             // two blocks per stage
constexpr int kPxPair = kPxStage;                  // one stage: B has read a stage's blocks before the stage's barrier, A writes the next behind it

// Issue priorities (s_setprio) of the two roles in the parts of a stage.  The two waves of a pair share a SIMD: where
// both are ready, the one with the higher priority issues.
constexpr int kPrioAS0 = 2, kPrioAS1 = 0, kPrioAExp = 0, kPrioAAcc = 0;
constexpr int kPrioBProd = 1, kPrioBTake = 1, kPrioBAcc = 1;
template <int P> __device__ inline void set_priority() { __builtin_amdgcn_s_setprio(P); }

// The hand-over of P between the two waves of a pair, with explicit instructions (address = byte offset inside the
// workgroup's LDS): the block must be written before its sequence number, and the number read before the block.  LDS
// executes a wave's operations in order, so issuing them in that order is enough; written as ordinary C++ accesses,
// the compiler would be free to reorder them.  The reads wait for their results themselves.
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
__device__ inline void lds_store_2x_b128(uint32_t addr, u32x4 lo, u32x4 hi) {   // lo at addr, hi at addr + 1024
    asm volatile("ds_write_b128 %0, %1\n\tds_write_b128 %0, %2 offset:1024" : : "v"(addr), "v"(lo), "v"(hi) : "memory");
}
__device__ inline void lds_load_2x_b128(uint32_t addr, u32x4 &lo, u32x4 &hi) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:1024\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(lo), "=&v"(hi) : "v"(addr) : "memory");
}

// CAUSAL: query i sees keys 0 .. i.  A tile of keys then streams the queries from its own first key on (stage
// `js`, in buffer 0); the two stages that cross the diagonal zero P for the queries before the lane's key, in the form
// of a stage that also handles the sample's ragged end.
// CROSS (cross attention): `offsets` belongs to the keys (the stationary rows), offsets_other to the queries that
// stream past them; the row statistics are indexed by query rows.  Otherwise offsets_other is not looked at.
template <bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kBdThreads, 2) void bwd_dkv_dma_kernel(const __bf16 *__restrict__ q,
                                                                    const __bf16 *__restrict__ k,
                                                                    const __bf16 *__restrict__ v,
                                                                    const __bf16 *__restrict__ dout,
                                                                    const float *__restrict__ stats,   // [2, H, sum_B]: delta, -lse * sqrt(D)
                                                                    const int64_t *__restrict__ offsets,
                                                                    const int64_t *__restrict__ offsets_other, int B, int H,
                                                                    Schedule s, __bf16 *__restrict__ dk,
                                                                    __bf16 *__restrict__ dv) {
    constexpr int D = kBdD;
    constexpr int kKSteps = D / 16;
    constexpr int kDBlocks = D / 32;
    // Three stages, each the streamed Q rows (kBdTile bytes) followed by the streamed dO rows.
    constexpr int kStageBytes = 2 * kBdTile;
    __shared__ __attribute__((aligned(1024))) char T[3 * kStageBytes];
    // Per stage: -lse * sqrt(D) [64] and delta [64] of the streamed rows.
    constexpr int kStatBytes = 512;
    __shared__ __attribute__((aligned(256))) char S[3 * kStatBytes];
    __shared__ __attribute__((aligned(1024))) char Px[kDkvPairs * kPxPair];   // P blocks on their way from A to B
    __shared__ int handed[kDkvPairs];   // per pair: number of P blocks A has written since the kernel started
    __shared__ WorkSlot slot;
    __shared__ LdsSchedule<CROSS> tab;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int pair = wave & 3;
    const bool is_a = wave < 4;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = CROSS ? offsets_other[B] : offsets[B];   // query rows
    const int64_t row_stride = (int64_t)H * D;

    // LDS read addresses inside a stage tile: one of each kind is kept, the others differ by constant bit patterns
    const int raddr0 = col * 256 + ((half ^ swz(col)) << 4);   // 16-byte row reads: row = col (+32 per block), chunk 2 ks + half
    int taddr0;                                                // transposing reads: row = 4 half + (lane & 15) / 4 (+8 for the operand's second half)
    {
        const int r = half * 4 + ((lane & 15) >> 2);
        const int chunk_in_group = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1), byte_in_chunk = (lane & 1) * 8;
        taddr0 = r * 256 + ((chunk_in_group ^ swz(r)) << 4) + byte_in_chunk;
    }
    // Every LDS read address is a per-lane constant plus a constant of the stage, block and step, which travels in the
    // instruction's offset field: computed once here, no address arithmetic is left in the stage loop.
    uint32_t row_at[kKSteps], tr_lo[kDBlocks], tr_hi[kDBlocks];
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) row_at[ks] = lds_byte_address(T) + (uint32_t)(raddr0 ^ (ks << 5));
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db) {
        tr_lo[db] = lds_byte_address(T) + (uint32_t)(taddr0 ^ (db << 6));
        tr_hi[db] = lds_byte_address(T) + (uint32_t)((taddr0 ^ (db << 6) ^ 32) + 2048);
    }
    const uint32_t stat_at = lds_byte_address(S) + (uint32_t)(half * 16);
    // Global -> LDS copies of a full stage: per-lane source offsets that do not depend on the stage (two rows of the
    // wave's eight per tile), and the lane's row for the statistics.
    uint32_t dma_off[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int r = 8 * wave + ((tid >> 4) & 3) + 4 * u;
        dma_off[u] = 2u * (uint32_t)(r * (int)((int64_t)H * D) + (((tid & 15) ^ swz(r)) << 3));
    }
    const uint32_t lane4 = 4u * (uint32_t)lane;
    const uint32_t px_pair = lds_address(Px) + pair * kPxPair;
    const uint32_t handed_addr = lds_address(&handed[pair]);

    struct Stream {
        const __bf16 *abase, *bbase;
        const float *delta_rows, *lse2_rows;
        int L, n_stages;   // rows of the sample; its number of 64-row stages
        int js;            // first stage of the stream (stage j lives in buffer (j - js) % 3)
    };
    auto stream_of = [&](const Work &w) {
        Stream st;
        st.L = CROSS ? w.olen : w.len;
        const int64_t srow0 = CROSS ? w.orow0 : w.row0;   // first streamed row (a query)
        st.n_stages = (st.L + kBdBN - 1) / kBdBN;
        st.js = CAUSAL ? w.block * kDkvBlockRows / kBdBN : 0;
        const int64_t head_off = srow0 * row_stride + (int64_t)w.head * D;
        st.abase = q + head_off;
        st.bbase = dout + head_off;
        st.delta_rows = stats + (int64_t)w.head * sum_B + srow0;
        st.lse2_rows = stats + (int64_t)(H + w.head) * sum_B + srow0;
        return st;
    };
    // One stage's copies: six per wave (two of Q rows, two of dO rows, two of row statistics).  A stage with all 64
    // rows inside the sample takes the constant offsets; the sample's last, shorter stage rebuilds them with rows past
    // the end repeating the last row (their P is zeroed).  The copies of a stage can be sent in three parts, so that a
    // wave can send them at different points of the stage before: sent all at once behind the barrier, the copies of
    // all eight waves queue up in the CU's one vector memory path and every wave stands still until its own have
    // been accepted.
    struct Copies {
        const __bf16 *a, *b;          // first streamed row of the stage in Q and dO (this head)
        const float *lse2, *delta;    // bases for the statistics copies
        uint32_t off[2], stat;        // per-lane byte offsets
    };
    auto copies_of = [&](const Stream &st, int stage) {
        Copies cp;
        const int j0 = stage * kBdBN;
        cp.a = st.abase + (int64_t)j0 * row_stride;
        cp.b = st.bbase + (int64_t)j0 * row_stride;
        if (j0 + kBdBN <= st.L) {
            cp.lse2 = st.lse2_rows + j0;
            cp.delta = st.delta_rows + j0;
            cp.off[0] = dma_off[0];
            cp.off[1] = dma_off[1];
            cp.stat = lane4;
        } else {
            int t_opaque = tid;
            asm volatile("" : "+v"(t_opaque));
            const int pc = t_opaque & 15;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = 8 * wave + ((t_opaque >> 4) & 3) + 4 * u;
                const int jr = j0 + r < st.L ? r : st.L - 1 - j0;
                cp.off[u] = 2u * (uint32_t)(jr * (int)row_stride + ((pc ^ swz(r)) << 3));
            }
            cp.lse2 = st.lse2_rows;
            cp.delta = st.delta_rows;
            cp.stat = 4u * (uint32_t)(j0 + lane < st.L ? j0 + lane : st.L - 1);
        }
        return cp;
    };
    auto issue_part = [&](const Copies &cp, auto BUF, auto PART) __attribute__((always_inline)) {
        constexpr int Bf = decltype(BUF)::value;
        constexpr int part = decltype(PART)::value;
        if constexpr (part < 2) {
            char *tile = T + Bf * kStageBytes + part * kBdTile;
#pragma unroll
            for (int u = 0; u < 2; ++u) bd_dma16(part == 0 ? cp.a : cp.b, cp.off[u], tile + (8 * wave + 4 * u) * 256);
        } else {
            // every wave copies the statistics (to the same place, the same values), so that all waves have the
            // same number of copies in flight and one wait count serves them all
            bd_dma4(cp.lse2, cp.stat, S + Bf * kStatBytes);
            bd_dma4(cp.delta, cp.stat, S + Bf * kStatBytes + 256);
        }
    };
    auto issue_stage_from = [&](const Stream &st, auto BUF, int j) {
        const Copies cp = copies_of(st, j);
        issue_part(cp, BUF, IntB<0>{});
        issue_part(cp, BUF, IntB<1>{});
        issue_part(cp, BUF, IntB<2>{});
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
            claim_and_decode(&slot, s, offsets, B, H, total, cursor, CROSS ? offsets_other : nullptr);
            return;
        }
        int64_t w = -1;
        if (lane == 0) w = next_work(s.counter, cursor, total);
        tab.decode(&slot, B, H, uniform64(w));
    };
    if (tid < kDkvPairs) handed[tid] = 0;
    if (wave == 0) claim_and_decode(&slot, s, offsets, B, H, total, cursor, CROSS ? offsets_other : nullptr);
    if (tabled) tab.fill(s, offsets, offsets_other, B);
    __syncthreads();
    uint32_t blocks_done = 0;   // P blocks this wave has written (A) or taken (B) since the kernel started
    Work t;
    bool have = load_work<CROSS>(&slot, t);
    while (have) {
        __syncthreads();   // every wave has read the slot before wave 0 refills it
        const Stream cur = stream_of(t);
        const int Ls = t.len;
        const int L = cur.L;
        const int tile0 = t.block * kDkvBlockRows;
        const int n_stages = cur.n_stages;
        if (CROSS && L == 0) {   // no query streams past these keys: their gradients are zero
            if (wave == 0) claim_next();
            const int i = tile0 + pair * 32 + (lane & 31);
            if (i < Ls) {
                __bf16 *grow = (is_a ? dv : dk) + (t.row0 + i) * row_stride + (int64_t)t.head * D + (lane >> 5) * (D / 2);
#pragma unroll
                for (int e = 0; e < D / 2; e += 8) *reinterpret_cast<u32x4 *>(grow + e) = u32x4{0, 0, 0, 0};
            }
            __syncthreads();   // the slot is written
            have = load_work<CROSS>(&slot, t);
            continue;
        }
        const bool wave_active = tile0 + pair * 32 < Ls;
        const int key = tile0 + pair * 32 + col;   // this lane's key (the causal mask compares queries with it)
        load_stationary(t);
        const int js = cur.js;
        issue_stage_from(cur, IntB<0>{}, js);
        if (n_stages - js > 1) issue_stage_from(cur, IntB<1>{}, js + 1);
        if (wave == 0) claim_next();   // overlaps with the loads in flight
        f32x16 acc[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[db][e] = 0.0f;

        // accumulator <- row statistics of 32 streamed rows (four 16-byte LDS reads at byte STAT of the statistics
        // array), then the product of the block of streamed rows at byte TILE of the stage array (row reads) with this
        // wave's stationary rows.  The operand reads run four matrix instructions ahead.
        auto product = [&](auto TILE, auto STAT, f32x16 &a) __attribute__((always_inline)) {
            constexpr int far = decltype(TILE)::value >= 65536 ? 65536 : 0;   // beyond the reach of the offset field
            constexpr int off = decltype(TILE)::value - far;
            f32x4 x0, x1, x2, x3;
            lds_fetch_4x_f32x4<decltype(STAT)::value>(stat_at, x0, x1, x2, x3);
            bf16x8 op[kKSteps];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) op[ks] = lds_fetch_b128<off>(row_at[ks] + far);
            lds_arrived<4>(x0, x1, x2, x3);
#pragma unroll
            for (int e = 0; e < 4; ++e) { a[e] = x0[e]; a[4 + e] = x1[e]; a[8 + e] = x2[e]; a[12 + e] = x3[e]; }
            static_assert(kKSteps == 8, "the read-ahead below is written for eight steps");
            op[4] = lds_fetch_b128<off>(row_at[4] + far); lds_arrived<4>(op[0], a); a = mfma_32x32x16(op[0], sreg[0], a);
            op[5] = lds_fetch_b128<off>(row_at[5] + far); lds_arrived<4>(op[1], a); a = mfma_32x32x16(op[1], sreg[1], a);
            op[6] = lds_fetch_b128<off>(row_at[6] + far); lds_arrived<4>(op[2], a); a = mfma_32x32x16(op[2], sreg[2], a);
            op[7] = lds_fetch_b128<off>(row_at[7] + far); lds_arrived<4>(op[3], a); a = mfma_32x32x16(op[3], sreg[3], a);
            lds_arrived<3>(op[4], a); a = mfma_32x32x16(op[4], sreg[4], a);
            lds_arrived<2>(op[5], a); a = mfma_32x32x16(op[5], sreg[5], a);
            lds_arrived<1>(op[6], a); a = mfma_32x32x16(op[6], sreg[6], a);
            lds_arrived<0>(op[7], a); a = mfma_32x32x16(op[7], sreg[7], a);
        };
        // acc^T += (block of streamed rows at byte TILE)^T x, contraction over the block's 32 rows in two steps of 16:
        // eight matrix instructions, each with an operand of two transposing reads; the reads run four instructions ahead.
        auto accumulate = [&](auto TILE, const bf16x8 (&x)[2]) __attribute__((always_inline)) {
            constexpr int far = decltype(TILE)::value >= 65536 ? 65536 : 0;
            constexpr int off = decltype(TILE)::value - far;
            bf16x4 lo[2 * kDBlocks], hi[2 * kDBlocks];   // operand i = ts * kDBlocks + db
            static_assert(kDBlocks == 4, "the read-ahead below is written for eight operands");
#define JFA_DKV_FETCH(i) lo[i] = lds_fetch_tr16<off + (i / 4) * 4096>(tr_lo[i % 4] + far); hi[i] = lds_fetch_tr16<off + (i / 4) * 4096>(tr_hi[i % 4] + far)
            JFA_DKV_FETCH(0); JFA_DKV_FETCH(1); JFA_DKV_FETCH(2); JFA_DKV_FETCH(3);
            JFA_DKV_FETCH(4); lds_arrived<8>(lo[0], hi[0], acc[0]); acc[0] = mfma_32x32x16(concat(lo[0], hi[0]), x[0], acc[0]);
            JFA_DKV_FETCH(5); lds_arrived<8>(lo[1], hi[1], acc[1]); acc[1] = mfma_32x32x16(concat(lo[1], hi[1]), x[0], acc[1]);
            JFA_DKV_FETCH(6); lds_arrived<8>(lo[2], hi[2], acc[2]); acc[2] = mfma_32x32x16(concat(lo[2], hi[2]), x[0], acc[2]);
            JFA_DKV_FETCH(7); lds_arrived<8>(lo[3], hi[3], acc[3]); acc[3] = mfma_32x32x16(concat(lo[3], hi[3]), x[0], acc[3]);
#undef JFA_DKV_FETCH
            lds_arrived<6>(lo[4], hi[4], acc[0]); acc[0] = mfma_32x32x16(concat(lo[4], hi[4]), x[1], acc[0]);
            lds_arrived<4>(lo[5], hi[5], acc[1]); acc[1] = mfma_32x32x16(concat(lo[5], hi[5]), x[1], acc[1]);
            lds_arrived<2>(lo[6], hi[6], acc[2]); acc[2] = mfma_32x32x16(concat(lo[6], hi[6]), x[1], acc[2]);
            lds_arrived<0>(lo[7], hi[7], acc[3]); acc[3] = mfma_32x32x16(concat(lo[7], hi[7]), x[1], acc[3]);
        };
        // where block mb of a stage travels: [block][half of the lane's sixteen values][lane]
        auto px_slot = [&](int j, int mb) __attribute__((always_inline)) {
            int l_opaque = lane;
            asm volatile("" : "+v"(l_opaque));
            return px_pair + (uint32_t)(mb * kPxBlock + l_opaque * 16);
        };

        // ---- wave A: one block of 32 streamed queries ----
        auto a_scores = [&](auto RAGGED, auto TILE, auto STAT, int mb, int j, bf16x8 (&p)[2]) __attribute__((always_inline)) {
            constexpr bool ragged = decltype(RAGGED)::value != 0;
            f32x16 sc;
            if (mb == 0) set_priority<kPrioAS0>(); else set_priority<kPrioAS1>();
            product(TILE, STAT, sc);   // dot products minus lse * sqrt(D) of the streamed rows
            set_priority<kPrioAExp>();
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float pe = fast_exp2(sc[e] * c);
                const int row = j * kBdBN + mb * 32 + (e >> 2) * 8 + half * 4 + (e & 3);   // the query of accumulator register e
                if (ragged && (row >= L || (CAUSAL && row < key))) pe = 0.0f;   // past the sample's end, or before the lane's key
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
        auto b_take = [&](int mb, int j, const f32x16 &dp, bf16x8 (&ds)[2]) __attribute__((always_inline)) {
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
        // SURE: the caller knows that stage j + 2 exists (no test for the sample's end in the stage).
        // ROLE_A: the stage as wave A or as wave B runs it.  The role is fixed for the whole tile outside the stage loop:
        // a branch on it inside a stage would merge the two roles' accumulators after every stage, at the price of
        // register copies of all 64 of them.
        auto run_stage = [&](auto ROLE_A, auto BUF, auto RAGGED, auto SURE, int j) __attribute__((always_inline)) {
            constexpr bool role_a = decltype(ROLE_A)::value != 0;
            constexpr int Bf = decltype(BUF)::value;
            constexpr bool ragged = decltype(RAGGED)::value != 0;
            const bool ahead = decltype(SURE)::value != 0 || j + 2 < n_stages;
            Copies cp;
            if (ahead) cp = copies_of(cur, j + 2);
            auto ahead_part = [&](auto PART) __attribute__((always_inline)) { if (ahead) issue_part(cp, IntB<(Bf + 2) % 3>{}, PART); };
            if (!wave_active) { ahead_part(IntB<0>{}); ahead_part(IntB<1>{}); ahead_part(IntB<2>{}); }
            if (wave_active) {
                constexpr int At = Bf * kStageBytes, Bt = At + kBdTile, St = Bf * kStatBytes;   // bytes into T and S
                constexpr int kBlock = 32 * 256;   // 32 streamed rows
                const bool second = !ragged || j * kBdBN + 32 < L;   // the sample's last stage may hold one block only
                if (role_a) {
                    bf16x8 p0[2], p1[2];
                    a_scores(RAGGED, IntB<At>{}, IntB<St>{}, 0, j, p0);
                    ahead_part(IntB<0>{});
                    if (second) a_scores(RAGGED, IntB<At + kBlock>{}, IntB<St + 128>{}, 1, j, p1);
                    ahead_part(IntB<1>{});
                    set_priority<kPrioAAcc>();
                    accumulate(IntB<Bt>{}, p0);               // dV^T += dO^T P
                    ahead_part(IntB<2>{});
                    if (second) accumulate(IntB<Bt + kBlock>{}, p1);
                } else {
                    f32x16 dp0, dp1;
                    bf16x8 ds[2];
                    set_priority<kPrioBProd>();
                    product(IntB<Bt>{}, IntB<St + 256>{}, dp0);       // delta - dO V^T (V is held negated)
                    ahead_part(IntB<0>{});
                    if (second) product(IntB<Bt + kBlock>{}, IntB<St + 256 + 128>{}, dp1);
                    ahead_part(IntB<1>{});
                    set_priority<kPrioBTake>();
                    b_take(0, j, dp0, ds);
                    set_priority<kPrioBAcc>();
                    accumulate(IntB<At>{}, ds);               // dK^T -= Q^T dS
                    ahead_part(IntB<2>{});
                    if (second) {
                        set_priority<kPrioBTake>();
                        b_take(1, j, dp1, ds);
                        set_priority<kPrioBAcc>();
                        accumulate(IntB<At + kBlock>{}, ds);
                    }
                }
            }
            set_priority<0>();
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
        if (n_stages - js > 1) wait_one_stage_outstanding(); else __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        auto all_stages = [&](auto ROLE_A) __attribute__((always_inline)) {
            constexpr int R0 = CAUSAL ? 2 : 0;   // buffer of the first stage of the unrolled loops
            constexpr int R1 = (R0 + 1) % 3, R2 = (R0 + 2) % 3;
            const int n_full = L / kBdBN;   // stages with all 64 streamed rows valid; a ragged one may follow
            int j = js;
            if (CAUSAL) {   // the two stages that cross the diagonal, in buffers 0 and 1, in the masking form
                if (j < n_stages) { run_stage(ROLE_A, IntB<0>{}, IntB<1>{}, IntB<0>{}, j); ++j; }
                if (j < n_stages) { run_stage(ROLE_A, IntB<1>{}, IntB<1>{}, IntB<0>{}, j); ++j; }
            }
            for (; j + 8 <= n_stages; j += 6) {   // six full stages, and the two after them exist
                run_stage(ROLE_A, IntB<R0>{}, IntB<0>{}, IntB<1>{}, j);
                run_stage(ROLE_A, IntB<R1>{}, IntB<0>{}, IntB<1>{}, j + 1);
                run_stage(ROLE_A, IntB<R2>{}, IntB<0>{}, IntB<1>{}, j + 2);
                run_stage(ROLE_A, IntB<R0>{}, IntB<0>{}, IntB<1>{}, j + 3);
                run_stage(ROLE_A, IntB<R1>{}, IntB<0>{}, IntB<1>{}, j + 4);
                run_stage(ROLE_A, IntB<R2>{}, IntB<0>{}, IntB<1>{}, j + 5);
            }
            for (; j + 5 <= n_stages; j += 3) {   // three full stages, and the two after them exist
                run_stage(ROLE_A, IntB<R0>{}, IntB<0>{}, IntB<1>{}, j);
                run_stage(ROLE_A, IntB<R1>{}, IntB<0>{}, IntB<1>{}, j + 1);
                run_stage(ROLE_A, IntB<R2>{}, IntB<0>{}, IntB<1>{}, j + 2);
            }
            for (; j < n_stages; ++j) {           // the last stages (at most four), stage j in buffer (j - js) % 3
                const int r = (j - js) % 3;
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
        const bool have_next = load_work<CROSS>(&slot, nt);

        // ---- epilogue: scale, transpose the wave's 32 x 128 gradient block through LDS, 64 features at a time, and
        // store whole 128-byte pieces of rows.  The stage buffers are idle (every wave is past the last stage's barrier,
        // no DMA is in flight, the next tile's loads start behind the barrier at the top of the loop); wave w uses 4 KB
        // of the third pair: row r of its block at r * 128, 16-byte chunk ch at (ch ^ (r & 7)) << 4.
        {
            char *const region = T + 2 * kStageBytes + (is_a ? 0 : kBdTile) + pair * 4096;
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
                              const int64_t *offsets, const int64_t *offsets_other, bool causal, int B, int H, int D,
                              Schedule s, void *dk, void *dv, int cus, hipStream_t stream) {
    if (D != kBdD || (causal && offsets_other)) return hipErrorInvalidValue;
#define JFA_LAUNCH(CROSS, CAUSAL)                                                                                           \
    hipLaunchKernelGGL((bwd_dkv_dma_kernel<CROSS, CAUSAL>),                                                                \
                       dim3(persistent_grid<bwd_dkv_dma_kernel<CROSS, CAUSAL>>(kBdThreads, cus)), dim3(kBdThreads), 0,      \
                       stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, (const __bf16 *)dout, stats,        \
                       offsets, offsets_other, B, H, s, (__bf16 *)dk, (__bf16 *)dv)
    if (offsets_other) JFA_LAUNCH(true, false);
    else if (causal) JFA_LAUNCH(false, true);
    else JFA_LAUNCH(false, false);
#undef JFA_LAUNCH
    return hipGetLastError();
}

}  // namespace jfa

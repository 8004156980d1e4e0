// Jagged flash attention backward, bf16, D = 128, long samples: the dQ kernel (paper Section 2.2).
//
//   P = exp(S / sqrt(D) - lse),  dP = dO V^T,  dS = P o (dP - delta),  dQ = dS K / sqrt(D)
//
// Shaped like the direct-to-LDS forward kernel: a workgroup is eight waves (two per SIMD), a wave owns 32 queries
// whose Q and dO rows stay in registers (one query per lane) and whose gradient it accumulates, and the sample's
// keys and values stream through three XOR-swizzled LDS stage buffers filled by global_load_lds two stages ahead
// (bare s_barrier + partial vmcnt wait per stage).  The score tile has the keys on the MFMA row axis and the queries
// on the column (= lane) axis, so dS leaves the accumulator already in operand position for dQ^T += K^T dS^T, whose
// other operand is the transposing LDS read of the K tile.  The kernel is the first of the backward: it also forms
// delta = rowsum(dO o O) and -lse * sqrt(D) for its queries and stores them for the dK / dV kernel
// (jfa_bwd_dkv_dma.hip).  Nothing is accumulated with atomics: results are deterministic.
#include "jfa_bwd_dma.h"

namespace jfa {

// CROSS (cross attention): `offsets` belongs to the queries and offsets_other to the keys and values that stream past
// them; otherwise offsets_other is not looked at.
// CAUSAL (self attention only): query i sees keys 0 .. i.  A tile streams the keys up to its last query and masks above
// the diagonal in the stages that reach past the tile's first query, in the form of a stage that also handles the
// sample's ragged end.
template <bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kBdThreads, 2) void bwd_dq_dma_kernel(const __bf16 *__restrict__ q,
                                                                     const __bf16 *__restrict__ k,
                                                                     const __bf16 *__restrict__ v,
                                                                     const __bf16 *__restrict__ dout,
                                                                     const float *__restrict__ lse,
                                                                     const __bf16 *__restrict__ out_fwd,   // dQ only; see below
                                                                     float *delta,
                                                                     const int64_t *__restrict__ offsets,
                                                                     const int64_t *__restrict__ offsets_other, int B, int H,
                                                                     Schedule s, __bf16 *__restrict__ grad) {
    constexpr int D = kBdD;
    constexpr int kKSteps = D / 16;
    constexpr int kDBlocks = D / 32;
    // streamed tile A: K (16-byte row reads and transposing reads); streamed tile B: V (16-byte row reads)
    __shared__ __attribute__((aligned(1024))) char A0[kBdTile];
    __shared__ __attribute__((aligned(1024))) char A1[kBdTile];
    __shared__ __attribute__((aligned(1024))) char A2[kBdTile];
    __shared__ __attribute__((aligned(1024))) char B0[kBdTile];
    __shared__ __attribute__((aligned(1024))) char B1[kBdTile];
    __shared__ __attribute__((aligned(1024))) char B2[kBdTile];
    // Per lane, four copies each of minus lse * sqrt(D) (the log-sum-exp in units of the raw dot product) and
    // minus delta of the lane's query.  The score and dP accumulators of every block start from these (four 16-byte
    // LDS reads each, no VALU work, no registers held across the stage): P = exp2(c * acc) with c = log2(e) / sqrt(D)
    // applied in fp32, and dS = P * acc.
    __shared__ float4 lane_init[kBdThreads * 2];
    __shared__ WorkSlot slot;   // the NEXT work item, claimed and decoded while the current one starts up
    __shared__ LdsSchedule<CROSS> tab;   // the schedule, copied once per workgroup when it fits

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];   // query rows: lse and delta are indexed by them
    const int64_t row_stride = (int64_t)H * D;

    // LDS read addresses inside a tile
    int raddr[kKSteps];   // 16-byte row reads: row = col (+32 per block), chunk 2 ks + half
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) raddr[ks] = col * 256 + (((2 * ks + half) ^ swz(col)) << 4);
    int taddr[2][kDBlocks];   // transposing reads: row = 4 half + (lane & 15) / 4 (+8 for the operand's second half)
    {
        const int r = half * 4 + ((lane & 15) >> 2);
        const int chunk_in_group = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1), byte_in_chunk = (lane & 1) * 8;
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
                taddr[h2][db] = (r + 8 * h2) * 256 + (((db * 4 + chunk_in_group) ^ swz(r + 8 * h2)) << 4) + byte_in_chunk;
    }
    // What streams past a tile: first rows of K and V, the tile's queries' statistics, number of keys of the sample
    // and of stages (causal tiles need only a part of the sample).
    struct Stream {
        const __bf16 *abase, *bbase;
        const float *delta_rows, *lse2_rows;   // plane 0 of the statistics buffer: delta; plane 1: -lse * sqrt(D)
        int L, Lc, js, n_stages;
    };
    auto stream_of = [&](const Work &w) {
        Stream st;
        st.L = CROSS ? w.olen : w.len;
        const int64_t srow0 = CROSS ? w.orow0 : w.row0;
        const int w_tile0 = w.block * kDmaBlockRows;   // first stationary row of the tile
        // causal: the keys a tile needs are 0 .. (tile's last query)
        st.Lc = CAUSAL && w_tile0 + kDmaBlockRows < st.L ? w_tile0 + kDmaBlockRows : st.L;
        st.js = 0;
        st.n_stages = (st.Lc + kBdBN - 1) / kBdBN;
        const int64_t head_off = srow0 * row_stride + (int64_t)w.head * D;
        st.abase = k + head_off;
        st.bbase = v + head_off;
        const int64_t qrow0 = w.row0;   // first query row of the sample
        st.delta_rows = delta + (int64_t)w.head * sum_B + qrow0;
        st.lse2_rows = delta + (int64_t)(H + w.head) * sum_B + qrow0;
        return st;
    };
    // The per-lane byte offsets of the two DMA chunks of a full stage are the same for every stage and both tensors:
    // two registers for the whole kernel.  The sample's last, shorter stage rebuilds them from the thread id with
    // rows past the end repeating the last row; so does every stage of the cross-attention instance, which has no
    // registers left for them (values used once per stage are the first to be spilled, and a reload from scratch
    // waits on the vector-memory counter, i.e. on the very loads that are meant to stay in flight).
    uint32_t dma_off[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int r = 8 * wave + ((tid >> 4) & 3) + 4 * u;
        dma_off[u] = 2u * (uint32_t)(r * (int)row_stride + (((tid & 15) ^ swz(r)) << 3));
    }
    auto issue_from = [&](const Stream &st, const __bf16 *base, char *tile, int stage) {
        const int L = st.L;
        const int j0 = stage * kBdBN;
        const __bf16 *sbase = base + (int64_t)j0 * row_stride;
        if (!CROSS && j0 + kBdBN <= L) {
#pragma unroll
            for (int u = 0; u < 2; ++u) bd_dma16(sbase, dma_off[u], tile + (8 * wave + 4 * u) * 256);
        } else {
            int t_opaque = tid;
            asm volatile("" : "+v"(t_opaque));
            const int dma_row0 = 8 * wave + ((t_opaque >> 4) & 3);
            const int pc = t_opaque & 15;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = dma_row0 + 4 * u;
                const int jr = j0 + r < L ? r : L - 1 - j0;   // rows past the end repeat the last row (masked later)
                bd_dma16(sbase, 2u * (uint32_t)(jr * (int)row_stride + ((pc ^ swz(r)) << 3)), tile + (8 * wave + 4 * u) * 256);
            }
        }
    };
    auto issue_stage_from = [&](const Stream &st, auto BUF, int j) {
        constexpr int Bf = decltype(BUF)::value;
        issue_from(st, st.abase, Bf == 0 ? A0 : (Bf == 1 ? A1 : A2), j);
        issue_from(st, st.bbase, Bf == 0 ? B0 : (Bf == 1 ? B1 : B2), j);
    };
    // ---- stationary rows: this lane's row as B operands (rows past the end of the sample repeat its last row) ----
    bf16x8 xreg[kKSteps], yreg[kKSteps];   // the lane's Q and dO rows
    auto load_stationary = [&](const Work &w) {
        const int iw = w.block * kDmaBlockRows + wave * 32 + col;
        const int64_t off = (w.row0 + (iw < w.len ? iw : w.len - 1)) * row_stride + (int64_t)w.head * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            xreg[ks] = *reinterpret_cast<const bf16x8 *>(q + off + 16 * ks);
            yreg[ks] = *reinterpret_cast<const bf16x8 *>(dout + off + 16 * ks);
        }
    };

    // The claim of the next item runs while a tile's first loads travel, and the tile cannot start before it is done:
    // with the schedule in LDS it is one atomic and a few LDS reads instead of five dependent trips to memory.
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
    if (wave == 0) claim_and_decode(&slot, s, offsets, B, H, total, cursor, CROSS ? offsets_other : nullptr);
    if (tabled) tab.fill(s, offsets, offsets_other, B);
    __syncthreads();   // the slot and the tables are written
    Work t;
    bool have = load_work<CROSS>(&slot, t);
    while (have) {
        __syncthreads();   // every wave has read the slot before wave 0 refills it
        const Stream cur = stream_of(t);
        const int Ls = t.len;                      // stationary rows of the sample
        const int L = cur.L;                       // streamed rows of the sample
        const int tile0 = t.block * kDmaBlockRows;   // first stationary row of the tile
        const int Lc = cur.Lc;
        const int js = cur.js;                     // first stage of the stream
        const int n_stages = cur.n_stages;
        if (CROSS && L == 0) {   // nothing streams past these rows: their gradient is zero
            if (wave == 0) claim_next();
            const int i = t.block * kDmaBlockRows + wave * 32 + (lane & 31);
            if (i < Ls) {
                __bf16 *grow = grad + (t.row0 + i) * row_stride + (int64_t)t.head * D + (lane >> 5) * (D / 2);
#pragma unroll
                for (int e = 0; e < D / 2; e += 8) *reinterpret_cast<u32x4 *>(grow + e) = u32x4{0, 0, 0, 0};
                if (out_fwd != nullptr && lane < 32) {   // out = 0 there: delta = 0; lse = -inf
                    delta[(int64_t)t.head * sum_B + t.row0 + i] = 0.0f;
                    delta[(int64_t)(H + t.head) * sum_B + t.row0 + i] = INFINITY;
                }
            }
            __syncthreads();   // the slot is written
            have = load_work<CROSS>(&slot, t);
            continue;
        }
        const float *const delta_rows = cur.delta_rows;
        const float *const lse2_rows = cur.lse2_rows;

        const int i = t.block * kDmaBlockRows + wave * 32 + col;
        const int ic = i < Ls ? i : Ls - 1;
        const bool wave_active = t.block * kDmaBlockRows + wave * 32 < Ls;
        load_stationary(t);
        issue_stage_from(cur, IntB<0>{}, js);
        if (n_stages - js > 1) issue_stage_from(cur, IntB<1>{}, js + 1);
        if (wave == 0) claim_next();   // overlaps with the loads in flight
        f32x16 acc[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[db][e] = 0.0f;

        // ---- one stage: 64 streamed rows in two blocks of 32 ----
        auto run_block = [&](auto RAGGED, const char *At, const char *Bt, int mb, int j0) {
            constexpr bool ragged = decltype(RAGGED)::value != 0;
            // LDS read addresses of this block.  There are no registers to spare for sixteen loop-invariant
            // addresses: the eight of the transposing reads are kept, of the row reads only one, and the others are
            // rebuilt per block with one XOR each (the swizzle makes them differ by a constant bit pattern); the empty
            // asm keeps the compiler from hoisting the rebuilt values back out of the loop.  (Keeping the row
            // addresses too, or this lane's address in lane_init, spills in the stages and costs 10 %.)
            int ra[kKSteps], ta[2][kDBlocks];
            {
                int rb = raddr[0];
                asm volatile("" : "+v"(rb));
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) ra[ks] = rb ^ (ks << 5);
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    ta[0][db] = taddr[0][db];
                    ta[1][db] = taddr[1][db];
                }
            }
            f32x16 sc, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sc[e] = 0.0f; dp[e] = 0.0f; }
            {   // both accumulators start at this lane's query's statistics: P = exp2(c * acc), dS = P * acc
                int t_opaque = tid;
                asm volatile("" : "+v"(t_opaque));   // the address is rebuilt here, not carried through the stage
                int mine = (t_opaque >> 6) * 128 + (t_opaque & 63);   // index of this lane's first 16-byte slot
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    asm volatile("" : "+v"(mine));   // four separate loads: one load and twelve register copies would be VALU work
                    const float4 l4 = lane_init[mine], d4 = lane_init[mine + 64];
                    sc[4 * g] = l4.x; sc[4 * g + 1] = l4.y; sc[4 * g + 2] = l4.z; sc[4 * g + 3] = l4.w;
                    dp[4 * g] = d4.x; dp[4 * g + 1] = d4.y; dp[4 * g + 2] = d4.z; dp[4 * g + 3] = d4.w;
                }
            }
            // operands are fetched four at a time to keep the register footprint at two waves per SIMD
#pragma unroll
            for (int k4 = 0; k4 < kKSteps; k4 += 4) {
                bf16x8 aop[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) aop[u] = lds_read_b128(At + mb * 32 * 256 + ra[k4 + u]);
#pragma unroll
                for (int u = 0; u < 4; ++u) sc = mfma_32x32x16(aop[u], xreg[k4 + u], sc);
            }
#pragma unroll
            for (int k4 = 0; k4 < kKSteps; k4 += 4) {
                bf16x8 bop[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) bop[u] = lds_read_b128(Bt + mb * 32 * 256 + ra[k4 + u]);
#pragma unroll
                for (int u = 0; u < 4; ++u) dp = mfma_32x32x16(bop[u], yreg[k4 + u], dp);
            }
            // P and dS for this lane's query and its 16 keys
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float p = fast_exp2(sc[4 * g + e] * c);   // the scale is applied in fp32: operands stay exact
                    const int r = j0 + mb * 32 + g * 8 + half * 4 + e;   // this register's streamed row
                    if (ragged && r >= (CAUSAL && ic + 1 < L ? ic + 1 : L)) p = 0.0f;   // past the sample's end, or above the diagonal
                    sc[4 * g + e] = p;
                    dp[4 * g + e] = p * dp[4 * g + e];
                }
            }
            // gradient accumulation: contraction over the 32 streamed rows in two steps of 16
            const char *Tt = At;
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const bf16x8 pb = pack_bf16(dp, 8 * ts);
                bf16x8 top[kDBlocks];
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *base = Tt + (mb * 32 + ts * 16) * 256;
                    top[db] = concat(lds_read_tr16(base + ta[0][db]), lds_read_tr16(base + ta[1][db]));
                }
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) acc[db] = mfma_32x32x16(top[db], pb, acc[db]);
            }
        };
        auto issue_stage = [&](auto BUF, int j) { issue_stage_from(cur, BUF, j); };
        // DMA operations per wave per stage: 4 tile chunks
        auto wait_one_stage_outstanding = [&]() { __builtin_amdgcn_s_waitcnt(0x0070 | 4); };
        auto run_stage = [&](auto BUF, auto RAGGED, int j) {
            constexpr int Bf = decltype(BUF)::value;
            constexpr bool ragged = decltype(RAGGED)::value != 0;   // only the sample's last stage can be
            const bool ahead = j + 2 < n_stages;
            if (ahead) issue_stage(IntB<(Bf + 2) % 3>{}, j + 2);
            if (wave_active) {
                const char *At = Bf == 0 ? A0 : (Bf == 1 ? A1 : A2);
                const char *Bt = Bf == 0 ? B0 : (Bf == 1 ? B1 : B2);
                const int j0 = j * kBdBN;
                if (CAUSAL && ragged) {
                    // A masking stage of a causal tile, seen by one wave: its 32 stationary rows against each block of 32
                    // streamed rows.  Blocks wholly on the far side of the diagonal contribute nothing.
                    const int mine = (tile0 + wave * 32) / 32;
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) {
                        const int theirs = j0 / 32 + mb;
                        if (theirs * 32 >= Lc) continue;
                        if (theirs <= mine) run_block(RAGGED, At, Bt, mb, j0);
                    }
                } else {
                    run_block(RAGGED, At, Bt, 0, j0);
                    if (!ragged || j0 + 32 < Lc) run_block(RAGGED, At, Bt, 1, j0);
                }
            }
            asm volatile("" ::: "memory");
            if (ahead) wait_one_stage_outstanding(); else __builtin_amdgcn_s_waitcnt(0x0070);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        };

#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            asm volatile("" : "+v"(xreg[ks]));   // stationary-row loads complete here
            asm volatile("" : "+v"(yreg[ks]));
        }
        {
            // This lane's query's statistics: minus lse * sqrt(D) and minus delta = rowsum(dO o O).  With out_fwd given,
            // this kernel is the first of the backward and computes them itself from the rows it holds (each lane of
            // a pair has half of the row), leaving both planes of the statistics buffer for the dK / dV kernel;
            // otherwise an earlier kernel has filled the buffer.
            float nl, nd;
            if (out_fwd != nullptr) {
                const int64_t off = (t.row0 + ic) * row_stride + (int64_t)t.head * D + 8 * half;
                float dot = 0.0f;
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) {
                    const bf16x8 o = *reinterpret_cast<const bf16x8 *>(out_fwd + off + 16 * ks);
#pragma unroll
                    for (int e = 0; e < 8; ++e) dot = fmaf((float)o[e], (float)yreg[ks][e], dot);
                }
                dot = pair_sum(dot);
                nl = -lse[(int64_t)t.head * sum_B + t.row0 + ic] * sqrtf((float)D);
                nd = -dot;
                if (i < Ls && half == 0) {
                    delta[(int64_t)t.head * sum_B + t.row0 + i] = dot;
                    delta[(int64_t)(H + t.head) * sum_B + t.row0 + i] = nl;
                }
            } else {
                nl = lse2_rows[ic];
                nd = -delta_rows[ic];
            }
            float4 *mine = lane_init + wave * 128 + lane;   // consecutive lanes, consecutive 16-byte slots: no bank
            mine[0] = make_float4(nl, nl, nl, nl);          // conflicts; written and read by the same lane: no barrier
            mine[64] = make_float4(nd, nd, nd, nd);
        }
        // The first stage has landed once at most one stage's loads are outstanding: what this wave sent after it is
        // the second stage (and, on wave 0, the loads of the claim, which it has waited for itself).
        if (n_stages - js > 1) wait_one_stage_outstanding(); else __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        if (CAUSAL) {
            // keys 0 .. tile0 lie below every query of the tile (full stages, as without the mask); the stages that
            // reach past the tile's first query follow in the masking form
            const int n_full = (tile0 + 1 < L ? tile0 + 1 : L) / kBdBN;
            int j = 0;
            for (; j + 3 <= n_full; j += 3) {
                run_stage(IntB<0>{}, IntB<0>{}, j);
                run_stage(IntB<1>{}, IntB<0>{}, j + 1);
                run_stage(IntB<2>{}, IntB<0>{}, j + 2);
            }
            if (j < n_full) { run_stage(IntB<0>{}, IntB<0>{}, j); ++j; }
            if (j < n_full) { run_stage(IntB<1>{}, IntB<0>{}, j); ++j; }
            for (; j < n_stages; ++j) {
                const int r = j % 3;
                if (r == 0) run_stage(IntB<0>{}, IntB<1>{}, j);
                else if (r == 1) run_stage(IntB<1>{}, IntB<1>{}, j);
                else run_stage(IntB<2>{}, IntB<1>{}, j);
            }
        } else {
            const int n_full = L / kBdBN;   // stages with all 64 streamed rows valid; a ragged one may follow
            int j = 0;
            for (; j + 3 <= n_full; j += 3) {
                run_stage(IntB<0>{}, IntB<0>{}, j);
                run_stage(IntB<1>{}, IntB<0>{}, j + 1);
                run_stage(IntB<2>{}, IntB<0>{}, j + 2);
            }
            if (j < n_full) { run_stage(IntB<0>{}, IntB<0>{}, j); ++j; }
            if (j < n_full) { run_stage(IntB<1>{}, IntB<0>{}, j); ++j; }
            if (j < n_stages) {             // the ragged last stage, in buffer n_full % 3
                const int r = n_full % 3;
                if (r == 0) run_stage(IntB<0>{}, IntB<1>{}, j);
                else if (r == 1) run_stage(IntB<1>{}, IntB<1>{}, j);
                else run_stage(IntB<2>{}, IntB<1>{}, j);
            }
        }

        Work nt;   // the next work item: wave 0 parked it in the slot before this tile's first barrier
        const bool have_next = load_work<CROSS>(&slot, nt);

        // ---- epilogue: scale, transpose the wave's 32 x 128 gradient block through LDS, 64 features at a time, and store
        // whole 128-byte pieces of rows, eight rows per store instruction.  The stage buffers are idle (every wave is past
        // the last stage's barrier, no DMA is in flight, and the next tile's loads start behind the barrier at the top of
        // the loop); wave w uses 4 KB of the third pair: row r of its block at r * 128, 16-byte chunk ch at (ch ^ (r & 7)) << 4.
        {
            char *const region = (wave < 4 ? A2 : B2) + (wave & 3) * 4096;
            const float out_scale = scale;
            int lane_e = lane;   // every address below derives from this copy, which the compiler cannot see
            asm volatile("" : "+v"(lane_e));   // through: otherwise they are computed at tile start and spilled
            const int col_e = lane_e & 31, half_e = lane_e >> 5;
            const int wbase = col_e * 128 + ((half_e * 8) ^ ((col_e & 7) << 4));
            const int r0 = t.block * kDmaBlockRows + wave * 32;   // first stationary row of this wave
            __bf16 *const gbase = grad + (t.row0 + r0) * row_stride + (int64_t)t.head * D;
            const uint32_t lane_off = 2u * (uint32_t)((lane_e >> 3) * (int)row_stride + (lane_e & 7) * 8);
#pragma unroll
            for (int f = 0; f < 2; ++f) {   // features 64 f .. 64 f + 63
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

hipError_t launch_bwd_dq_dma(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                             float *delta, const int64_t *offsets, const int64_t *offsets_other, bool causal, int B, int H,
                             int D, Schedule s, void *dq, int cus, hipStream_t stream) {
    if (D != kBdD || (causal && offsets_other)) return hipErrorInvalidValue;
#define JFA_LAUNCH(CROSS, CAUSAL)                                                                                           \
    hipLaunchKernelGGL((bwd_dq_dma_kernel<CROSS, CAUSAL>), dim3(persistent_grid<bwd_dq_dma_kernel<CROSS, CAUSAL>>(kBdThreads, cus)), \
                       dim3(kBdThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v,                \
                       (const __bf16 *)dout, lse, (const __bf16 *)out, delta, offsets, offsets_other, B, H, s, (__bf16 *)dq)
    if (offsets_other) JFA_LAUNCH(true, false);
    else if (causal) JFA_LAUNCH(false, true);
    else JFA_LAUNCH(false, false);
#undef JFA_LAUNCH
    return hipGetLastError();
}

}  // namespace jfa

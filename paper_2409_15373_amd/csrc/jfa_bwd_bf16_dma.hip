// Jagged flash attention backward, bf16, D = 128, long-sample variant (paper Section 2.2).
//
//   P = exp(S / sqrt(D) - lse),  dP = dO V^T,  dS = P o (dP - delta),  dV = P^T dO,  dQ = dS K / sqrt(D),  dK = dS^T Q / sqrt(D)
//
// Three kernels of one template, all shaped like the direct-to-LDS forward kernel: a workgroup is eight
// waves (two per SIMD), a wave owns 32 "stationary" rows whose operands stay in registers and whose gradient
// it accumulates, and the sample's other rows stream through three XOR-swizzled LDS stage buffers filled by
// global_load_lds two stages ahead (bare s_barrier + partial vmcnt wait per stage):
//   dQ  stationary = queries (Q, dO rows, lse, delta per lane); streams K and V;      dQ^T += K^T dS^T
//   dK  stationary = keys (K, V rows); streams Q, dO and lse, delta per streamed row;  dK^T += Q^T dS
//   dV  stationary = keys (K rows);    streams Q, dO and lse;                          dV^T += dO^T P
// In every case the score tile has the streamed rows on the MFMA row axis and the stationary rows on the
// column (= lane) axis, so P / dS leave the accumulator already in operand position for the last product,
// whose other operand is the transposing LDS read of a streamed tile.  Keeping dK and dV in separate kernels
// costs one more recomputation of S but lets each of them run two waves per SIMD (their accumulators together
// need the whole register file), and nothing is accumulated with atomics: results are deterministic.
#include "jfa_bwd_dma.h"

namespace jfa {

// CROSS (cross attention): `offsets` belongs to the stationary rows (queries for dQ, keys for dK and dV) and
// offsets_other to the rows that stream past them; otherwise offsets_other is not looked at.
// CAUSAL (self attention only): query i sees keys 0 .. i.  dQ streams the keys up to the tile's last query and masks
// above the diagonal in the stages that reach past the tile's first query; dK and dV start their stream of queries at
// the stage of the tile's first key and zero P for the queries before the lane's key in the four stages that overlap
// the tile.  Masking stages use the form that also handles the sample's ragged end.
template <int MODE, bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kBdThreads, 2) void bwd_bf16_dma_kernel(const __bf16 *__restrict__ q,
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
    constexpr bool kRowStats = MODE != kModeDQ;   // lse / delta belong to the streamed rows
    constexpr bool kSecond = MODE != kModeDV;     // dP / dS are needed
    constexpr bool kLeanAddresses = MODE != kModeDV;
    // streamed tile A: dQ: K, dK: Q, dV: Q      (16-byte row reads; transposing reads too unless dV)
    // streamed tile B: dQ: V, dK: dO, dV: dO    (16-byte row reads; dV: transposing reads only)
    __shared__ __attribute__((aligned(1024))) char A0[kBdTile];
    __shared__ __attribute__((aligned(1024))) char A1[kBdTile];
    __shared__ __attribute__((aligned(1024))) char A2[kBdTile];
    __shared__ __attribute__((aligned(1024))) char B0[kBdTile];
    __shared__ __attribute__((aligned(1024))) char B1[kBdTile];
    __shared__ __attribute__((aligned(1024))) char B2[kBdTile];
    __shared__ __attribute__((aligned(256))) char S0[512];   // per stage: lse[64], delta[64] of the streamed rows
    __shared__ __attribute__((aligned(256))) char S1[512];
    __shared__ __attribute__((aligned(256))) char S2[512];
    // dQ only: per lane, four copies each of minus lse * sqrt(D) (the log-sum-exp in units of the raw dot product) and
    // minus delta of the lane's query.  The score and dP accumulators of every block start from these (four 16-byte
    // LDS reads each, no VALU work, no registers held across the stage): P = exp2(c * acc) with c = log2(e) / sqrt(D)
    // applied in fp32, and dS = P * acc.
    __shared__ float4 lane_init[MODE == kModeDQ ? kBdThreads * 2 : 1];
    __shared__ WorkSlot slot;   // the NEXT work item, claimed and decoded while the current one starts up
    __shared__ LdsSchedule<CROSS> tab;   // the schedule, copied once per workgroup when it fits

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const float scale = 1.0f / sqrtf((float)D);
    const float c = 1.4426950408889634f * scale;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = (CROSS && kRowStats) ? offsets_other[B] : offsets[B];   // query rows: lse and delta are indexed by them
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
    // What streams past a tile: first rows of the two streamed tensors and of the streamed rows' statistics, number of
    // streamed rows of the sample, first stage and number of stages (causal tiles need only a part of the sample).
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
        // causal: the streamed rows a tile needs are keys 0 .. (tile's last query) for dQ, queries (tile's first key) .. L - 1 for dK, dV
        st.Lc = CAUSAL && !kRowStats && w_tile0 + kDmaBlockRows < st.L ? w_tile0 + kDmaBlockRows : st.L;
        st.js = CAUSAL && kRowStats ? w_tile0 / kBdBN : 0;
        st.n_stages = (st.Lc + kBdBN - 1) / kBdBN;
        const int64_t head_off = srow0 * row_stride + (int64_t)w.head * D;
        st.abase = (MODE == kModeDQ ? k : q) + head_off;
        st.bbase = (MODE == kModeDQ ? v : dout) + head_off;
        const int64_t qrow0 = kRowStats ? srow0 : w.row0;   // first query row of the sample
        st.delta_rows = delta + (int64_t)w.head * sum_B + qrow0;
        st.lse2_rows = delta + (int64_t)(H + w.head) * sum_B + qrow0;
        return st;
    };
    // The per-lane byte offsets of the two DMA chunks of a stage are rebuilt from the thread id at every
    // issue (a handful of VALU operations per stage) instead of living in registers across the stage: values
    // used once per stage are the first the register allocator spills, and a reload from scratch memory
    // would wait on the vector-memory counter, i.e. on the very loads that are meant to stay in flight.
    auto issue_from = [&](const Stream &st, const __bf16 *base, char *tile, int stage) {
        const int L = st.L;
        const int j0 = stage * kBdBN;
        const __bf16 *sbase = base + (int64_t)j0 * row_stride;
        int t_opaque = tid;
        asm volatile("" : "+v"(t_opaque));
        const int dma_row0 = 8 * wave + ((t_opaque >> 4) & 3);
        const int pc = t_opaque & 15;
        if (j0 + kBdBN <= L) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = dma_row0 + 4 * u;
                bd_dma16(sbase, 2u * (uint32_t)(r * (int)row_stride + ((pc ^ swz(r)) << 3)), tile + (8 * wave + 4 * u) * 256);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = dma_row0 + 4 * u;
                const int jr = j0 + r < L ? r : L - 1 - j0;   // rows past the end repeat the last row (masked later)
                bd_dma16(sbase, 2u * (uint32_t)(jr * (int)row_stride + ((pc ^ swz(r)) << 3)), tile + (8 * wave + 4 * u) * 256);
            }
        }
    };
    auto issue_stats_from = [&](const Stream &st, char *stats, int stage) {   // wave 0 only: lse and delta of the 64 streamed rows
        const int j0 = stage * kBdBN;
        const uint32_t j = 4u * (uint32_t)(j0 + lane < st.L ? j0 + lane : st.L - 1);
        bd_dma4(st.lse2_rows, j, stats);
        if (kSecond) bd_dma4(st.delta_rows, j, stats + 256);
    };
    auto issue_stage_from = [&](const Stream &st, auto BUF, int j) {
        constexpr int Bf = decltype(BUF)::value;
        issue_from(st, st.abase, Bf == 0 ? A0 : (Bf == 1 ? A1 : A2), j);
        issue_from(st, st.bbase, Bf == 0 ? B0 : (Bf == 1 ? B1 : B2), j);
        if (kRowStats && wave == 0) issue_stats_from(st, Bf == 0 ? S0 : (Bf == 1 ? S1 : S2), j);
    };
    // ---- stationary rows: this lane's row as B operands (rows past the end of the sample repeat its last row) ----
    bf16x8 xreg[kKSteps], yreg[kKSteps];   // dQ: Q, dO rows   dK: K, V rows   dV: K rows
    auto load_stationary = [&](const Work &w) {
        const int iw = w.block * kDmaBlockRows + wave * 32 + col;
        const int64_t off = (w.row0 + (iw < w.len ? iw : w.len - 1)) * row_stride + (int64_t)w.head * D + 8 * half;
        const __bf16 *xsrc = MODE == kModeDQ ? q : k;
        const __bf16 *ysrc = MODE == kModeDQ ? dout : v;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            xreg[ks] = *reinterpret_cast<const bf16x8 *>(xsrc + off + 16 * ks);
            if (kSecond) yreg[ks] = *reinterpret_cast<const bf16x8 *>(ysrc + off + 16 * ks);
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
                if (!kRowStats && out_fwd != nullptr && lane < 32) {   // out = 0 there: delta = 0; lse = -inf
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
        auto run_block = [&](auto RAGGED, const char *At, const char *Bt, const char *St, int mb, int j0) {
            constexpr bool ragged = decltype(RAGGED)::value != 0;
            // LDS read addresses of this block.  The dQ and dK kernels have no registers to spare for sixteen
            // loop-invariant addresses: they keep one of each kind and rebuild the others per block with one
            // XOR each (the swizzle makes them differ by a constant bit pattern); the empty asm keeps the
            // compiler from hoisting the rebuilt values back out of the loop.
            int ra[kKSteps], ta[2][kDBlocks];
            if (kLeanAddresses) {
                int rb = raddr[0], tb = taddr[0][0];
                asm volatile("" : "+v"(rb), "+v"(tb));
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) ra[ks] = rb ^ (ks << 5);
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    ta[0][db] = tb ^ (db << 6);
                    ta[1][db] = (tb ^ (db << 6) ^ 32) + 2048;
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) ra[ks] = raddr[ks];
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) { ta[0][db] = taddr[0][db]; ta[1][db] = taddr[1][db]; }
            }
            f32x16 sc, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sc[e] = 0.0f; dp[e] = 0.0f; }
            if (kRowStats) {   // the dot products start at minus the streamed rows' lse * sqrt(D): P = exp2(c * acc)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 l4 = *reinterpret_cast<const float4 *>(St + (mb * 32 + g * 8 + half * 4) * 4);
                    sc[4 * g] = l4.x; sc[4 * g + 1] = l4.y; sc[4 * g + 2] = l4.z; sc[4 * g + 3] = l4.w;
                }
            }
            if (MODE == kModeDQ) {   // both accumulators start at this lane's query's statistics
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
            if (MODE == kModeDK) {   // dP accumulator starts at the streamed rows' delta
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 d4 = *reinterpret_cast<const float4 *>(St + 256 + (mb * 32 + g * 8 + half * 4) * 4);
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
            if (kSecond) {
#pragma unroll
                for (int k4 = 0; k4 < kKSteps; k4 += 4) {
                    bf16x8 bop[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) bop[u] = lds_read_b128(Bt + mb * 32 * 256 + ra[k4 + u]);
#pragma unroll
                    for (int u = 0; u < 4; ++u) dp = mfma_32x32x16(bop[u], yreg[k4 + u], dp);
                }
            }
            // P (and dS, up to the sign in the dK kernel) for this lane's stationary row and its 16 streamed rows
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float p = fast_exp2(sc[4 * g + e] * c);   // the scale is applied in fp32: operands stay exact
                    const int r = j0 + mb * 32 + g * 8 + half * 4 + e;   // this register's streamed row
                    if (ragged && (r >= (CAUSAL && !kRowStats && ic + 1 < L ? ic + 1 : L) || (CAUSAL && kRowStats && r < ic)))
                        p = 0.0f;   // past the sample's end, or on the wrong side of the diagonal
                    sc[4 * g + e] = p;
                    if (MODE == kModeDK) dp[4 * g + e] = p * dp[4 * g + e];                  // = -dS
                    if (MODE == kModeDQ) dp[4 * g + e] = p * dp[4 * g + e];
                }
            }
            // gradient accumulation: contraction over the 32 streamed rows in two steps of 16
            const char *Tt = MODE == kModeDV ? Bt : At;
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                const bf16x8 pb = pack_bf16(kSecond ? dp : sc, 8 * ts);
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
        // DMA operations per wave per stage: 4 tile chunks, plus the row statistics on wave 0
        auto wait_one_stage_outstanding = [&]() {
            if (kRowStats && wave == 0) {
                if (kSecond) __builtin_amdgcn_s_waitcnt(0x0070 | 6); else __builtin_amdgcn_s_waitcnt(0x0070 | 5);
            } else {
                __builtin_amdgcn_s_waitcnt(0x0070 | 4);
            }
        };
        auto run_stage = [&](auto BUF, auto RAGGED, int j) {
            constexpr int Bf = decltype(BUF)::value;
            constexpr bool ragged = decltype(RAGGED)::value != 0;   // only the sample's last stage can be
            const bool ahead = j + 2 < n_stages;
            if (ahead) issue_stage(IntB<(Bf + 2) % 3>{}, j + 2);
            if (wave_active) {
                const char *At = Bf == 0 ? A0 : (Bf == 1 ? A1 : A2);
                const char *Bt = Bf == 0 ? B0 : (Bf == 1 ? B1 : B2);
                const char *St = Bf == 0 ? S0 : (Bf == 1 ? S1 : S2);
                const int j0 = j * kBdBN;
                if (CAUSAL && ragged) {
                    // A masking stage of a causal tile, seen by one wave: its 32 stationary rows against each block of 32
                    // streamed rows.  Blocks wholly on the far side of the diagonal contribute nothing.
                    const int mine = (tile0 + wave * 32) / 32;
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) {
                        const int theirs = j0 / 32 + mb;
                        if (theirs * 32 >= Lc) continue;
                        if (kRowStats ? theirs >= mine : theirs <= mine) run_block(RAGGED, At, Bt, St, mb, j0);
                    }
                } else {
                    run_block(RAGGED, At, Bt, St, 0, j0);
                    if (!ragged || j0 + 32 < Lc) run_block(RAGGED, At, Bt, St, 1, j0);
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
            if (kSecond) asm volatile("" : "+v"(yreg[ks]));
        }
        if (MODE == kModeDK) {   // V enters negated: the dP accumulator starts at delta and ends as delta - dP
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                u32x4 w = __builtin_bit_cast(u32x4, yreg[ks]);
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] ^= 0x80008000u;
                yreg[ks] = __builtin_bit_cast(bf16x8, w);
            }
        }
        if (!kRowStats) {
            // This lane's query's statistics: minus lse * sqrt(D) and minus delta = rowsum(dO o O).  With out_fwd given,
            // this kernel is the first of the backward and computes them itself from the rows it holds (each lane of
            // a pair has half of the row), leaving both planes of the statistics buffer for the dK and dV kernels;
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
        if (CAUSAL && !kRowStats) {
            // dQ: keys 0 .. tile0 lie below every query of the tile (full stages, as without the mask); the stages that
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
        } else if (CAUSAL) {
            // dK, dV: the stream of queries starts at the tile's first key; stage j lives in buffer (j - js) % 3.  Its first
            // four stages cross the diagonal (buffers 0, 1, 2, 0) and mask, full stages follow from buffer 1 on, and the
            // sample's ragged last stage masks again: one copy of the masking stages serves both ends.
            const int diagonal_end = js + kDmaBlockRows / kBdBN < n_stages ? js + kDmaBlockRows / kBdBN : n_stages;
            const int n_full = L / kBdBN;
            int j = js;
#pragma nounroll
            for (int part = 0; part < 2; ++part) {
                const int masking_end = part == 0 ? diagonal_end : n_stages;
                for (; j < masking_end; ++j) {
                    const int r = (j - js) % 3;
                    if (r == 0) run_stage(IntB<0>{}, IntB<1>{}, j);
                    else if (r == 1) run_stage(IntB<1>{}, IntB<1>{}, j);
                    else run_stage(IntB<2>{}, IntB<1>{}, j);
                }
                if (part == 0) {
                    for (; j + 3 <= n_full; j += 3) {
                        run_stage(IntB<1>{}, IntB<0>{}, j);
                        run_stage(IntB<2>{}, IntB<0>{}, j + 1);
                        run_stage(IntB<0>{}, IntB<0>{}, j + 2);
                    }
                    if (j < n_full) { run_stage(IntB<1>{}, IntB<0>{}, j); ++j; }
                    if (j < n_full) { run_stage(IntB<2>{}, IntB<0>{}, j); ++j; }
                }
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
            const float out_scale = MODE == kModeDV ? 1.0f : (MODE == kModeDK ? -scale : scale);
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

template <int MODE>
static hipError_t launch_mode(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                              float *delta, const int64_t *offsets, const int64_t *offsets_other, bool causal, int B,
                              int H, Schedule s, void *grad, int cus, hipStream_t stream) {
    if (causal && offsets_other) return hipErrorInvalidValue;
#define JFA_LAUNCH(CROSS, CAUSAL)                                                                                           \
    hipLaunchKernelGGL((bwd_bf16_dma_kernel<MODE, CROSS, CAUSAL>), dim3(persistent_grid<bwd_bf16_dma_kernel<MODE, CROSS, CAUSAL>>(kBdThreads, cus)), \
                       dim3(kBdThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v,                \
                       (const __bf16 *)dout, lse, (const __bf16 *)out, delta, offsets, offsets_other, B, H, s, (__bf16 *)grad)
    if (offsets_other) JFA_LAUNCH(true, false);
    else if (causal) JFA_LAUNCH(false, true);
    else JFA_LAUNCH(false, false);
#undef JFA_LAUNCH
    return hipGetLastError();
}

hipError_t launch_bwd_bf16_dma(int mode, const void *q, const void *k, const void *v, const void *out, const void *dout,
                               const float *lse, float *delta, const int64_t *offsets,
                               const int64_t *offsets_other, bool causal, int B, int H, int D, Schedule s, void *grad,
                               int cus, hipStream_t stream) {
    if (D != kBdD) return hipErrorInvalidValue;
    switch (mode) {
        case kModeDQ: return launch_mode<kModeDQ>(q, k, v, out, dout, lse, delta, offsets, offsets_other, causal, B, H, s, grad, cus, stream);
        case kModeDK: return launch_mode<kModeDK>(q, k, v, nullptr, dout, lse, delta, offsets, offsets_other, causal, B, H, s, grad, cus, stream);
        case kModeDV: return launch_mode<kModeDV>(q, k, v, nullptr, dout, lse, delta, offsets, offsets_other, causal, B, H, s, grad, cus, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace jfa

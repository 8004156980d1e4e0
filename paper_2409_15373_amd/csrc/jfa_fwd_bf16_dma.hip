// Jagged flash attention forward, bf16, D = 128, long-sample variant (paper Section 2.1).
//
// Same mathematics and operand layouts as fwd_bf16_kernel (transposed score tile S^T = K Q^T, a lane owns
// one query, V^T through the transposing LDS read, 32 queries per wave, two waves per SIMD).  What differs:
//   * a workgroup is eight waves = 256 queries sharing each K / V stage, so the HBM/L2 -> LDS traffic per
//     flop is half that of the 128-query kernel;
//   * stages travel HBM/L2 -> LDS directly (global_load_lds_dwordx4): no staging registers, no LDS store
//     instructions.  The tiles are unpadded and XOR-swizzled on 16-byte (K) / 64-byte (V) granules so that
//     the 16-byte row reads and the transposing reads are conflict-free on the 64-bank LDS;
//   * three stage buffers, DMA two stages ahead, and a bare s_barrier with a partial vmcnt wait at the end of a
//     stage (a __syncthreads() would wait for every load in flight);
//   * exponentials are taken against a FIXED reference maximum per query (the maximum over the sample's
//     first 32 keys): no running maximum, no rescaling, no branch in the hot loop.  A reference below the
//     true maximum only scales numerator and denominator alike -- probabilities keep their relative
//     precision in fp32 and bf16 -- as long as nothing overflows; a row sum above 2^62 (or not finite) at the
//     end of the tile shows that it got too stale, and the workgroup then redoes the tile in the conservative
//     order (maximum first, online rescaling).  On data whose scores are of one scale this never runs.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kDmaThreads = 512;
constexpr int kDmaWaves = kDmaThreads / 64;
constexpr int kDmaBN = 64;            // keys per LDS stage
constexpr int kDmaD = 128;
constexpr int kDmaTile = kDmaBN * kDmaD * 2;   // bytes of one K or V stage in LDS
constexpr int kDmaOpsPerStage = 2 * (kDmaBN / 4) / kDmaWaves;   // DMA instructions per wave per stage (K and V)

template <int N> using IntC = std::integral_constant<int, N>;

// 16 bytes per lane from `base` (wave-uniform, kept in scalar registers) + `byte_offset` (per lane, unsigned
// 32 bits) into LDS at lds_wave_base + 16 * lane: the scalar-base form needs no 64-bit vector arithmetic.
__device__ inline void dma16b(const __bf16 *base, uint32_t byte_offset, char *lds_wave_base) {
    const char *src = reinterpret_cast<const char *>(base) + byte_offset;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// CROSS: the keys and values of a sample are the rows of a second offsets array (cross attention); otherwise
// offsets_kv is not looked at and the code is that of self attention.  CAUSAL (self attention only): query i attends
// to keys 0 .. i.  A tile then streams the keys up to its last query; the stages whose keys all lie at or below the
// tile's first query run unmasked, the others (up to five) run in the masking form of a stage with the per-lane
// limit min(L, i + 1) in place of L.
template <bool CROSS, bool CAUSAL>
__global__ __launch_bounds__(kDmaThreads, 2) void fwd_bf16_dma_kernel(const __bf16 *__restrict__ q,
                                                                      const __bf16 *__restrict__ k,
                                                                      const __bf16 *__restrict__ v,
                                                                      const int64_t *__restrict__ offsets,
                                                                      const int64_t *__restrict__ offsets_kv, int B,
                                                                      int H, Schedule s, __bf16 *__restrict__ out,
                                                                      float *__restrict__ lse) {
    constexpr int D = kDmaD;
    constexpr int kKSteps = D / 16;    // 8
    constexpr int kDBlocks = D / 32;   // 4
    // Separate arrays (not one indexed array) so that the compiler can tell the buffer being filled by the
    // DMA from the one being read and does not make the reads wait for the loads in flight.
    __shared__ __attribute__((aligned(1024))) char K0[kDmaTile];
    __shared__ __attribute__((aligned(1024))) char K1[kDmaTile];
    __shared__ __attribute__((aligned(1024))) char K2[kDmaTile];
    __shared__ __attribute__((aligned(1024))) char V0[kDmaTile];
    __shared__ __attribute__((aligned(1024))) char V1[kDmaTile];
    __shared__ __attribute__((aligned(1024))) char V2[kDmaTile];
    __shared__ WorkSlot slot;   // the NEXT work item, claimed and decoded while the current one starts up
    __shared__ LdsSchedule<CROSS> tab;   // the schedule, copied once per workgroup when it fits
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
    // Only k-step 0's address is kept; step ks is at kaddr0 ^ (ks << 5) (the XOR swizzle makes the eight differ by
    // a constant bit pattern).  Each stage rebuilds them: twelve loop-invariant addresses held in registers
    // across the stage would be the first values the register allocator spills.
    const int kaddr0 = col * 256 + ((half ^ (col & 15)) << 4);
    // V element (row r, 64-byte group g, byte b inside it) sits at r * 256 + ((g ^ (r & 3)) << 6) + b.
    // The transposing read of this lane: row = 4 half + (lane & 15) / 4 (+8 for the second half of the
    // operand, +16 per 16-key step), group = feature block db, bytes 32 * ((lane >> 4) & 1) + 8 * (lane & 3).
    // Feature block db is at vaddr0 ^ (db << 6).
    int vaddr0;
    {
        const int r = half * 4 + ((lane & 15) >> 2);
        vaddr0 = r * 256 + ((r & 3) << 6) + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
    }
    auto lds_addresses = [&](int (&kaddr)[kKSteps], int (&vaddr)[kDBlocks]) {
        int kb = kaddr0, vb = vaddr0;
        asm volatile("" : "+v"(kb), "+v"(vb));   // keeps the rebuilt addresses from being hoisted out of the loop
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) kaddr[ks] = kb ^ (ks << 5);
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db) vaddr[db] = vb ^ (db << 6);
    };
    // ---- DMA: one instruction moves 64 lanes x 16 bytes = 4 rows; wave w, instruction u fills rows 8 w + 4 u .. +3.
    // Lane l lands on physical chunk l & 15 of row 8 w + 4 u + (l >> 4) and so fetches the logical chunk that
    // the swizzle puts there.
    const int dma_row0 = 8 * wave + (lane >> 4);
    const int pc = lane & 15;

    // byte offsets of this lane's DMA chunks inside a full stage (K and V differ in the swizzle)
    uint32_t koffs[2], voffs[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int r = dma_row0 + 4 * u;
        koffs[u] = 2u * (uint32_t)(r * (int)row_stride + ((pc ^ (r & 15)) << 3));
        voffs[u] = 2u * (uint32_t)(r * (int)row_stride + ((pc ^ ((r & 3) << 2)) << 3));
    }
    // The keys a tile streams: first rows of K and V, number of keys of the sample, number of 64-key stages.
    struct Stream {
        const __bf16 *kbase, *vbase;
        int L, n_stages;
    };
    auto stream_of = [&](const Work &w) {
        Stream st;
        st.L = CROSS ? w.olen : w.len;
        const int64_t krow0 = CROSS ? w.orow0 : w.row0;
        const int w_tile0 = w.block * kDmaBlockRows;
        const int Lc = CAUSAL && w_tile0 + kDmaBlockRows < st.L ? w_tile0 + kDmaBlockRows : st.L;   // keys the tile needs
        st.n_stages = (Lc + kDmaBN - 1) / kDmaBN;
        st.kbase = k + krow0 * row_stride + (int64_t)w.head * D;
        st.vbase = v + krow0 * row_stride + (int64_t)w.head * D;
        return st;
    };
    bf16x8 qreg[kKSteps];
    auto load_q = [&](const Work &w) {   // the lane's query row (rows past the end of the sample repeat its last row)
        const int iw = w.block * kDmaBlockRows + wave * 32 + col;
        const __bf16 *qrow = q + (w.row0 + (iw < w.len ? iw : w.len - 1)) * row_stride + (int64_t)w.head * D + 8 * half;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
    };
    // The claim of the next item runs while a tile's first loads travel, and the tile cannot start before it is done:
    // with the schedule in LDS it is one atomic and a few LDS reads instead of five dependent trips to memory.
    const bool tabled = B <= kTabCap;
    WorkCursor cursor;
    auto claim_next = [&]() {   // wave 0, every lane
        if (!tabled) {
            claim_and_decode(&slot, s, offsets, B, H, total, cursor, CROSS ? offsets_kv : nullptr);
            return;
        }
        int64_t w = -1;
        if (lane == 0) w = next_work(s.counter, cursor, total);
        tab.decode(&slot, B, H, uniform64(w));
    };
    if (wave == 0) claim_and_decode(&slot, s, offsets, B, H, total, cursor, CROSS ? offsets_kv : nullptr);
    if (tabled) tab.fill(s, offsets, offsets_kv, B);
    __syncthreads();   // the slot and the tables are written
    Work t;
    bool have = load_work<CROSS>(&slot, t);
    while (have) {
        __syncthreads();   // every wave has read the slot before wave 0 refills it
        const Stream cur = stream_of(t);
        const int Lq = t.len;                      // queries of the sample
        const int L = cur.L;                       // keys of the sample
        const int q_tile0 = t.block * kDmaBlockRows;   // first query of the tile
        const int n_stages = cur.n_stages;
        const __bf16 *const kbase = cur.kbase;
        const __bf16 *const vbase = cur.vbase;
        if (CROSS && L == 0) {   // no keys: an empty softmax, out = 0 and lse = -inf
            if (wave == 0) claim_next();
            const int i = t.block * kDmaBlockRows + wave * 32 + (lane & 31);
            if (i < Lq) {
                __bf16 *orow = out + (t.row0 + i) * row_stride + (int64_t)t.head * D + (lane >> 5) * (D / 2);
#pragma unroll
                for (int e = 0; e < D / 2; e += 8) *reinterpret_cast<u32x4 *>(orow + e) = u32x4{0, 0, 0, 0};
                if (lane < 32) lse[(int64_t)t.head * sum_B + t.row0 + i] = -INFINITY;
            }
            __syncthreads();   // the slot is written
            have = load_work<CROSS>(&slot, t);
            continue;
        }

        auto issue_from = [&](const Stream &st, const __bf16 *base, char *tile, int stage, bool is_k) {
            const int L = st.L;
            const int j0 = stage * kDmaBN;
            const __bf16 *sbase = base + (int64_t)j0 * row_stride;
            if (j0 + kDmaBN <= L) {
#pragma unroll
                for (int u = 0; u < 2; ++u) dma16b(sbase, is_k ? koffs[u] : voffs[u], tile + (8 * wave + 4 * u) * 256);
            } else {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int r = dma_row0 + 4 * u;
                    const int ch = is_k ? (pc ^ (r & 15)) : (pc ^ ((r & 3) << 2));
                    const int jr = j0 + r < L ? r : L - 1 - j0;   // rows past the end repeat the last key (masked later)
                    dma16b(sbase, 2u * (uint32_t)(jr * (int)row_stride + ch * 8), tile + (8 * wave + 4 * u) * 256);
                }
            }
        };
        auto issue = [&](const __bf16 *base, char *tile, int stage, bool is_k) { issue_from(cur, base, tile, stage, is_k); };

        const int i = t.block * kDmaBlockRows + wave * 32 + col;   // this lane's query
        const int iq = i < Lq ? i : Lq - 1;
        const bool wave_active = t.block * kDmaBlockRows + wave * 32 < Lq;

        f32x16 o[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
        float m = -INFINITY, lsum = 0.0f;
        f32x16 negm;   // minus the reference maximum, sixteen times: the addend the score products start from

        // ---- helpers ----
        auto scores = [&](const char *tile, int mb, f32x16 &a) {
            int kaddr[kKSteps], vaddr[kDBlocks];
            lds_addresses(kaddr, vaddr);
#pragma unroll
            for (int e = 0; e < 16; ++e) a[e] = 0.0f;
            bf16x8 kop[kKSteps];
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) kop[ks] = lds_read_b128(tile + mb * 32 * 256 + kaddr[ks]);
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) a = mfma_32x32x16(kop[ks], qreg[ks], a);
        };
        auto accumulate = [&](const char *tile, int mb, const bf16x8 (&p)[2], const int (&vaddr)[kDBlocks]) {
            bf16x8 vop[2][kDBlocks];
#pragma unroll
            for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *pvp = tile + (mb * 32 + ts * 16) * 256 + vaddr[db];
                    vop[ts][db] = concat(lds_read_tr16(pvp), lds_read_tr16(pvp + 8 * 256));
                }
#pragma unroll
            for (int ts = 0; ts < 2; ++ts)
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) o[db] = mfma_32x32x16(vop[ts][db], p[ts], o[db]);
        };
        // exponentials of one unit (32 keys x 32 queries) against the reference maximum; the rounded
        // probabilities are what the second product uses, so they are what the row sum adds up
        // st holds raw dot products (minus the raw reference in the fast order, whose subc is the constant 0); the
        // softmax scale and the change to base-2 exponentials are one fp32 multiply-add per score
        auto exps = [&](const f32x16 &st, auto FAST, float subc, bf16x8 (&p)[2]) {
            constexpr bool kFast = decltype(FAST)::value != 0;
#pragma unroll
            for (int ts = 0; ts < 2; ++ts) {
                u32x4 pw;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bf16x2 pr;
                    const float x0 = st[8 * ts + 2 * e], x1 = st[8 * ts + 2 * e + 1];
                    pr[0] = (__bf16)fast_exp2(kFast ? x0 * c : fmaf(x0, c, -subc));
                    pr[1] = (__bf16)fast_exp2(kFast ? x1 * c : fmaf(x1, c, -subc));
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum, false);
                    pw[e] = __builtin_bit_cast(uint32_t, pr);
                }
                p[ts] = __builtin_bit_cast(bf16x8, pw);
            }
        };
        auto mask = [&](f32x16 &st, int key0) {   // keys past the end of the sample (causal: and above the diagonal)
            int h = half;
            asm volatile("" : "+v"(h));   // keeps the sixteen thresholds from being computed at tile start and spilled
            const int lim = (CAUSAL && iq + 1 < L ? iq + 1 : L) - key0 - 4 * h;   // accumulator register e holds key key0 + (e / 4) * 8 + 4 * half + e % 4
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if ((e >> 2) * 8 + (e & 3) >= lim) st[e] = -INFINITY;
        };
        auto unit_max = [&](const f32x16 &a, float mx) {
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, a[e]);
            return mx;
        };
        auto kbuf = [&](int bsel) { return bsel == 0 ? K0 : (bsel == 1 ? K1 : K2); };
        auto vbuf = [&](int bsel) { return bsel == 0 ? V0 : (bsel == 1 ? V1 : V2); };

        // pipelined(): fast order against the fixed reference maximum m
        auto pipelined = [&](auto BUF, auto RAGGED, int j) {
            constexpr int P = decltype(BUF)::value;   // buffer of this stage: j % 3
            constexpr bool kRagged = decltype(RAGGED)::value != 0;
            const char *const Kc = P == 0 ? K0 : (P == 1 ? K1 : K2);
            const char *const Vc = P == 0 ? V0 : (P == 1 ? V1 : V2);
            int kaddr[kKSteps], vaddr[kDBlocks];
            lds_addresses(kaddr, vaddr);
            f32x16 s0 = negm, s1 = negm;   // the dot products start at minus the (raw) reference: no subtraction later
            bf16x8 p0[2], p1[2];
            {
                bf16x8 ka[kKSteps], kb[kKSteps];
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) ka[ks] = lds_read_b128(Kc + kaddr[ks]);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) kb[ks] = lds_read_b128(Kc + 32 * 256 + kaddr[ks]);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) s0 = mfma_32x32x16(ka[ks], qreg[ks], s0);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) s1 = mfma_32x32x16(kb[ks], qreg[ks], s1);   // scores of key block 1 ...
                // issue order: the first block's operand reads, then one read of the second block behind each
                // matrix product of the first, so that LDS latency hides under the matrix pipe
                __builtin_amdgcn_sched_group_barrier(0x100, kKSteps, 0);
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, kKSteps, 0);
            }
            if (kRagged) mask(s0, j * kDmaBN);
            exps(s0, IntC<1>{}, 0.0f, p0);             // ... VALU: exponentials of key block 0
            accumulate(Vc, 0, p0, vaddr);              // matrix pipe: O^T += V^T P^T of key block 0 ...
            if (kRagged) mask(s1, j * kDmaBN + 32);
            exps(s1, IntC<1>{}, 0.0f, p1);             // ... VALU: exponentials of key block 1
            accumulate(Vc, 1, p1, vaddr);
        };
        // conservative(): maximum first, rescale, then exponentials; used when a tile had to be restarted
        auto conservative = [&](int bsel, int j) {
            const char *const Kc = kbuf(bsel);
            const char *const Vc = vbuf(bsel);
            int kaddr[kKSteps], vaddr[kDBlocks];
            lds_addresses(kaddr, vaddr);
            f32x16 s0, s1;
            bf16x8 p0[2], p1[2];
            scores(Kc, 0, s0);
            scores(Kc, 1, s1);
            if (CAUSAL || (j + 1) * kDmaBN > L) { mask(s0, j * kDmaBN); mask(s1, j * kDmaBN + 32); }
            const float x = pair_max(unit_max(s1, unit_max(s0, -INFINITY)));
            const float n = fmaxf(m, x);
            const float a = fast_exp2((m - n) * c);   // 0 on the first stage
            m = n;
            lsum *= a;
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= a;
            exps(s0, IntC<0>{}, n * c, p0);
            accumulate(Vc, 0, p0, vaddr);
            exps(s1, IntC<0>{}, n * c, p1);
            accumulate(Vc, 1, p1, vaddr);
        };

        // ---- pass 1: pipelined, three stage buffers, DMA two stages ahead ----
        // Stage j lives in buffer j % 3.  At the top of stage j the DMA of stage j + 2 is issued into the buffer
        // that stage j - 1 has just released; at the end of stage j each wave waits until only those newest
        // DMA operations are outstanding (so stage j + 1 has landed) and meets the others at a bare s_barrier.
        auto issue_stage = [&](auto BUF, int j) {
            constexpr int Bf = decltype(BUF)::value;
            issue(kbase, Bf == 0 ? K0 : (Bf == 1 ? K1 : K2), j, true);
            issue(vbase, Bf == 0 ? V0 : (Bf == 1 ? V1 : V2), j, false);
        };
        auto run_stage = [&](auto BUF, auto RAGGED, int j) {
            constexpr int Bf = decltype(BUF)::value;
            const bool ahead = j + 2 < n_stages;
            if (ahead) issue_stage(IntC<(Bf + 2) % 3>{}, j + 2);
            if (CAUSAL && decltype(RAGGED)::value != 0) {
                // A masking stage of a causal tile, seen by one wave: its 32 queries lie inside one 64-key stage.  Earlier
                // stages hold only keys below all of them (no mask, and all inside the sample), later ones only keys above.
                const int j_diagonal = (q_tile0 + wave * 32) / kDmaBN;
                if (wave_active && j < j_diagonal) pipelined(BUF, IntC<0>{}, j);
                else if (wave_active && j == j_diagonal) pipelined(BUF, IntC<1>{}, j);
            } else if (wave_active) {
                pipelined(BUF, RAGGED, j);
            }
            asm volatile("" ::: "memory");
            if (ahead) __builtin_amdgcn_s_waitcnt(0x0070 | kDmaOpsPerStage);   // vmcnt(ops of one stage) lgkmcnt(0)
            else __builtin_amdgcn_s_waitcnt(0x0070);                           // vmcnt(0) lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        };

        load_q(t);
        issue_stage(IntC<0>{}, 0);
        if (n_stages > 1) issue_stage(IntC<1>{}, 1);
        if (wave == 0) claim_next();   // overlaps with the loads in flight
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qreg[ks]));   // Q loads complete here
        // Stage 0 has landed once at most one stage's loads are outstanding: what this wave sent after it is stage 1
        // (and, on wave 0, the loads of the claim, which it has waited for itself).
        if (n_stages > 1) __builtin_amdgcn_s_waitcnt(0x0070 | kDmaOpsPerStage); else __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        if (tid == 0) restart = 0;   // nobody looks at it between the previous tile's check and this barrier
        if (wave_active) {   // reference maximum: the first 32 keys
            f32x16 s0;
            scores(K0, 0, s0);
            if (CAUSAL || L < 32) mask(s0, 0);
            m = pair_max(unit_max(s0, -INFINITY));
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) negm[e] = -m;
        asm volatile("" : "+v"(negm));   // sixteen real registers: the matrix product reads its addend from them
        {
            // stages with all 64 keys valid for every query of the tile; the others follow in the masking form:
            // the sample's ragged last stage, and if causal the stages that reach above the tile's first query
            const int n_full = (CAUSAL && q_tile0 + 1 < L ? q_tile0 + 1 : L) / kDmaBN;
            int j = 0;
            for (; j + 3 <= n_full; j += 3) {
                run_stage(IntC<0>{}, IntC<0>{}, j);
                run_stage(IntC<1>{}, IntC<0>{}, j + 1);
                run_stage(IntC<2>{}, IntC<0>{}, j + 2);
            }
            if (j < n_full) { run_stage(IntC<0>{}, IntC<0>{}, j); ++j; }
            if (j < n_full) { run_stage(IntC<1>{}, IntC<0>{}, j); ++j; }
            for (; j < n_stages; ++j) {       // masking stages (one at most unless causal), stage j in buffer j % 3
                const int r = j % 3;
                if (r == 0) run_stage(IntC<0>{}, IntC<1>{}, j);
                else if (r == 1) run_stage(IntC<1>{}, IntC<1>{}, j);
                else run_stage(IntC<2>{}, IntC<1>{}, j);
            }
        }
        // a row sum this large (or not finite) means the fixed reference was too far below the true maximum
        if (wave_active && __builtin_amdgcn_ballot_w64(!(lsum < 0x1p62f)) != 0 && lane == 0) restart = 1;
        __syncthreads();   // `restart` is written
        const bool again = restart != 0;

        // ---- pass 2 (never on data of one scale): the whole tile again, maximum first, two buffers ----
        if (again) {
            issue(kbase, K0, 0, true);
            issue(vbase, V0, 0, false);
            __builtin_amdgcn_s_waitcnt(0x0070);
            __syncthreads();
            m = -INFINITY;
            lsum = 0.0f;
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
            for (int j = 0; j < n_stages; ++j) {
                if (j + 1 < n_stages) {
                    issue(kbase, kbuf((j + 1) & 1), j + 1, true);
                    issue(vbase, vbuf((j + 1) & 1), j + 1, false);
                }
                if (wave_active) conservative(j & 1, j);
                __builtin_amdgcn_s_waitcnt(0x0070);
                __syncthreads();
            }
        }

        Work nt;   // the next work item: wave 0 parked it in the slot before this tile's first barrier
        const bool have_next = load_work<CROSS>(&slot, nt);

        // ---- epilogue: normalise; transpose the wave's 32 x 128 output block through LDS, 64 features at a time, so
        // that it leaves as whole 128-byte pieces of rows (16 bytes per lane, eight rows per store instruction) instead
        // of 8-byte pieces of 32 different rows per instruction; store the log-sum-exp ----
        // The stage buffers are idle here (every wave is past the last stage's barrier and no DMA is in flight, and the
        // next tile's loads start behind the barrier at the top of the loop); wave w uses 4 KB of the third one: row r of its block at r * 128,
        // 16-byte chunk ch at (ch ^ (r & 7)) << 4.
        const float l_total = pair_sum(lsum);
        {
            char *const region = (wave < 4 ? K2 : V2) + (wave & 3) * 4096;
            const float inv = 1.0f / l_total;
            int lane_e = lane;   // every address below derives from this copy, which the compiler cannot see
            asm volatile("" : "+v"(lane_e));   // through: otherwise they are computed at tile start and spilled
            const int col_e = lane_e & 31, half_e = lane_e >> 5;
            const int wbase = col_e * 128 + ((half_e * 8) ^ ((col_e & 7) << 4));
            const int q0 = t.block * kDmaBlockRows + wave * 32;   // first query of this wave
            __bf16 *const obase = out + (t.row0 + q0) * row_stride + (int64_t)t.head * D;
            const uint32_t lane_off = 2u * (uint32_t)((lane_e >> 3) * (int)row_stride + (lane_e & 7) * 8);
#pragma unroll
            for (int f = 0; f < 2; ++f) {   // features 64 f .. 64 f + 63
#pragma unroll
                for (int dl = 0; dl < 2; ++dl)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        bf16x4 x;
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = (__bf16)(o[2 * f + dl][4 * g + e] * inv);
                        *reinterpret_cast<bf16x4 *>(region + (wbase ^ (dl * 64 + g * 16))) = x;
                    }
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int r = it * 8 + (lane_e >> 3);
                    const u32x4 rowpiece = *reinterpret_cast<const u32x4 *>(region + r * 128 + (((lane_e & 7) ^ (r & 7)) << 4));
                    char *dst = reinterpret_cast<char *>(obase + (int64_t)it * 8 * row_stride + 64 * f) + lane_off;   // scalar base + 32-bit lane offset
                    if (q0 + r < Lq) *reinterpret_cast<u32x4 *>(dst) = rowpiece;
                }
            }
        }
        if (i < Lq && half == 0)
            lse[(int64_t)t.head * sum_B + t.row0 + i] = (m * c + fast_log2(l_total)) * 0.6931471805599453f;
        t = nt;
        have = have_next;
    }
}

hipError_t launch_fwd_bf16_dma(const void *q, const void *k, const void *v, const int64_t *offsets,
                               const int64_t *offsets_kv, bool causal, int B, int H, int D, Schedule s, void *out, float *lse,
                               int cus, hipStream_t stream) {
    if (D != kDmaD || (causal && offsets_kv)) return hipErrorInvalidValue;
#define JFA_LAUNCH(CROSS, CAUSAL)                                                                                          \
    hipLaunchKernelGGL((fwd_bf16_dma_kernel<CROSS, CAUSAL>), dim3(persistent_grid<fwd_bf16_dma_kernel<CROSS, CAUSAL>>(kDmaThreads, cus)), \
                       dim3(kDmaThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v, offsets,     \
                       offsets_kv, B, H, s, (__bf16 *)out, lse)
    if (offsets_kv) JFA_LAUNCH(true, false);
    else if (causal) JFA_LAUNCH(false, true);
    else JFA_LAUNCH(false, false);
#undef JFA_LAUNCH
    return hipGetLastError();
}

}  // namespace jfa

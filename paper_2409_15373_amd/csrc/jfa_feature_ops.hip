// The jagged feature operators of the paper's Table 1 on bf16 tensors with fp32 accumulation:
//   jagged_dense_bmm    x [sum_B, D] x w [B, D, T]      -> out [sum_B, T]   out_i = x_i w_b          (i in sample b)
//   jagged_jagged_bmm   x [sum_B, D] x y [sum_B, T]     -> out [B, D, T]    out_b = sum_i x_i^T y_i  (i in sample b)
//   jagged_softmax      x [sum_B, D]                    -> y   [sum_B, D]   softmax along each sample's rows, per column
//   jagged_softmax_backward  y, dy -> dx = y (dy - sum_i dy_i y_i)
// All four move O(sum_B (D + T)) bytes for O(sum_B D T) flops with D, T <= 128: they are bound by HBM, and the
// matrix cores only keep the arithmetic out of the way.  Every global access is 16 bytes per lane on consecutive
// addresses (a sample's rows are one contiguous block), operands reach the MFMA layout through LDS, and results
// go back through LDS so that stores cover whole rows.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kFoThreads = 256;
constexpr int kFoRows = 128;   // rows of x per work item of jagged_dense_bmm

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Row stride of a [k][n] bf16 tile whose columns feed transposing reads (ds_read_b64_tr_b16): four consecutive
// rows' 64-byte column blocks must fall into different banks.
__host__ __device__ constexpr int tr_row_bytes(int n) { return n == 32 ? 64 : n * 2 + 64; }

// Address (bytes inside the tile) of this lane's transposing read: contraction rows 4 half + (lane & 15) / 4 of a
// 16-row step (+8 rows for the operand's second half), bytes 32 ((lane >> 4) & 1) + 8 (lane & 3) of a 64-byte
// column block.  Slot e of the resulting operand is contraction row 16 step + (e / 4) 8 + 4 half + e % 4.
__device__ inline int tr_lane_offset(int lane, int row_bytes) {
    return ((lane >> 5) * 4 + ((lane & 15) >> 2)) * row_bytes + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
}
__device__ inline bf16x8 tr_operand(const char *tile, int off, int step, int block, int row_bytes) {
    const char *p = tile + step * 16 * row_bytes + block * 64 + off;
    return concat(lds_read_tr16(p), lds_read_tr16(p + 8 * row_bytes));
}

// Per-sample work items in sample order: the first statically, the rest by one atomic each (dynamic claims even out
// samples of different lengths; an offsets-sorted order would cost a scheduler launch that takes longer than it saves).
__global__ void reset_counter_kernel(int32_t *counter) { if (threadIdx.x == 0) *counter = 0; }

// Samples are claimed kClaimGroup consecutive ones at a time (`group` holds the current group between calls).  With
// 64-byte rows a sample is a few kilobytes and a claim per sample costs more than moving it: two per claim took the
// operators at D = T = 32 from 2.6 - 3.8 to 2.9 - 5.3 TB/s; with longer rows pairs only unbalance the workgroups (2 - 4 %
// slower at 128- and 256-byte rows), so those claim one at a time.
template <int kClaimGroup>
__device__ inline int claim_sample(int32_t *counter, int n_claimed, int *slot, int &group) {
    __syncthreads();
    if (n_claimed % kClaimGroup == 0) {
        if (threadIdx.x == 0) *slot = n_claimed == 0 ? (int)blockIdx.x : (int)gridDim.x + atomicAdd(counter, 1);
        __syncthreads();
        group = __builtin_amdgcn_readfirstlane(*slot);
    }
    return group * kClaimGroup + n_claimed % kClaimGroup;
}

// ---- jagged_dense_bmm: out^T = w_b^T x^T, one sample per workgroup step, 128 rows at a time ----
// w_b goes to LDS once per sample.  Wave w owns rows 32 w .. 32 w + 31 of every 128-row block: its x rows and,
// after the product, its output rows share one private LDS region.
template <int D, int T>
__global__ __launch_bounds__(kFoThreads) void jagged_dense_bmm_kernel(const __bf16 *__restrict__ x,
                                                                      const __bf16 *__restrict__ w,
                                                                      const int64_t *__restrict__ offsets, int B,
                                                                      int32_t *__restrict__ counter, __bf16 *__restrict__ out) {
    constexpr int kKSteps = D / 16, kTBlocks = T / 32;
    constexpr int kXRow = D * 2 + 8;          // x rows: the 8-byte operand reads of 32 consecutive rows hit 32 different bank pairs
    constexpr int kWRow = tr_row_bytes(T);
    constexpr int kORow = T * 2 + 16;
    constexpr int kRegion = 32 * (kXRow > kORow ? kXRow : kORow);   // one wave's rows, as input and then as output
    __shared__ __attribute__((aligned(16))) char xt[4 * kRegion];
    __shared__ __attribute__((aligned(16))) char wt[D * kWRow];
    __shared__ int slot;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int woff = tr_lane_offset(lane, kWRow);
    char *mine = xt + wave * kRegion;
    int group = 0;
    for (int n_claimed = 0;; ++n_claimed) {
        const int p = claim_sample<(D + T <= 64 ? 2 : 1)>(counter, n_claimed, &slot, group);   // also: the previous sample's LDS tiles are free
        if (p >= B) break;
        const int b = p;
        const int64_t row0 = offsets[b];
        const int L = (int)(offsets[b + 1] - row0);
        if (L == 0) continue;
        {
            const u32x4 *wsrc = reinterpret_cast<const u32x4 *>(w + (int64_t)b * D * T);
            for (int c = tid; c < D * (T / 8); c += kFoThreads)
                *reinterpret_cast<u32x4 *>(wt + (c / (T / 8)) * kWRow + (c % (T / 8)) * 16) = wsrc[c];
        }
        // A block of x is rows * D * 2 contiguous bytes; rows past the sample's end become zeros.  The next block is
        // fetched into registers while the current one is multiplied.
        constexpr int kChunks = kFoRows * (D / 8) / kFoThreads;   // 16-byte chunks of a block per thread
        u32x4 xv[kChunks];
        auto fetch = [&](int r0) {
            const int rows = L - r0 < kFoRows ? L - r0 : kFoRows;
            const u32x4 *src = reinterpret_cast<const u32x4 *>(x + (row0 + r0) * D);
#pragma unroll
            for (int u = 0; u < kChunks; ++u) {
                const int c = tid + kFoThreads * u;
                xv[u] = u32x4{0, 0, 0, 0};
                if (c / (D / 8) < rows) xv[u] = src[c];
            }
        };
        fetch(0);
        for (int r0 = 0; r0 < L; r0 += kFoRows) {
            if (r0) __syncthreads();   // every wave is done with the previous block's region
            const int rows = L - r0 < kFoRows ? L - r0 : kFoRows;
#pragma unroll
            for (int u = 0; u < kChunks; ++u) {
                const int c = tid + kFoThreads * u, r = c / (D / 8), ch = c % (D / 8);
                char *dst = xt + (r >> 5) * kRegion + (r & 31) * kXRow + ch * 16;
                *reinterpret_cast<u32x2 *>(dst) = u32x2{xv[u][0], xv[u][1]};
                *reinterpret_cast<u32x2 *>(dst + 8) = u32x2{xv[u][2], xv[u][3]};
            }
            if (r0 + kFoRows < L) fetch(r0 + kFoRows);
            __syncthreads();
            if (wave * 32 >= rows) continue;
            f32x16 acc[kTBlocks];
#pragma unroll
            for (int tb = 0; tb < kTBlocks; ++tb)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[tb][e] = 0.0f;
            const char *xrow = mine + col * kXRow + half * 8;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                // B operand = x^T: this lane's row, features 16 ks + 4 half + 0..3 and 16 ks + 8 + 4 half + 0..3
                const u32x2 lo = *reinterpret_cast<const u32x2 *>(xrow + ks * 32);
                const u32x2 hi = *reinterpret_cast<const u32x2 *>(xrow + ks * 32 + 16);
                const bf16x8 xop = __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], hi[0], hi[1]});
#pragma unroll
                for (int tb = 0; tb < kTBlocks; ++tb) acc[tb] = mfma_32x32x16(tr_operand(wt, woff, ks, tb, kWRow), xop, acc[tb]);
            }
            // register 4 g + e of block tb: output column 32 tb + 8 g + 4 half + e of this lane's row
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int tb = 0; tb < kTBlocks; ++tb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (__bf16)acc[tb][4 * g + e];
                    *reinterpret_cast<bf16x4 *>(mine + col * kORow + (tb * 32 + g * 8 + half * 4) * 2) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            u32x4 *dst = reinterpret_cast<u32x4 *>(out + (row0 + r0 + wave * 32) * T);   // the wave's 32 rows: one contiguous block
            const int mine_rows = rows - wave * 32;
#pragma unroll
            for (int u = 0; u < 32 * (T / 8) / 64; ++u) {
                const int c = lane + 64 * u, r = c / (T / 8), ch = c % (T / 8);
                if (r < mine_rows) dst[c] = *reinterpret_cast<const u32x4 *>(mine + r * kORow + ch * 16);
            }
        }
    }
}

// ---- jagged_jagged_bmm: out_b^T = y_b^T x_b, one sample per workgroup step, 64 rows at a time ----
template <int D, int T>
__global__ __launch_bounds__(kFoThreads) void jagged_jagged_bmm_kernel(const __bf16 *__restrict__ x,
                                                                       const __bf16 *__restrict__ y,
                                                                       const int64_t *__restrict__ offsets, int B,
                                                                       int32_t *__restrict__ counter, __bf16 *__restrict__ out) {
    constexpr int kDBlocks = D / 32, kTBlocks = T / 32, kBlocks = kDBlocks * kTBlocks;
    constexpr int kMine = (kBlocks + 3) / 4;   // 32 x 32 output blocks per wave
    constexpr int kXRow = tr_row_bytes(D), kYRow = tr_row_bytes(T);
    constexpr int kORow = T * 2 + 16;
    constexpr int kStage = 64 * kXRow + 64 * kYRow, kOut = D * kORow;
    __shared__ __attribute__((aligned(16))) char lds[kStage > kOut ? kStage : kOut];
    __shared__ int slot;
    char *xs = lds, *ys = lds + 64 * kXRow;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int xoff = tr_lane_offset(lane, kXRow), yoff = tr_lane_offset(lane, kYRow);
    int group = 0;
    for (int n_claimed = 0;; ++n_claimed) {
        const int p = claim_sample<(D + T <= 64 ? 2 : 1)>(counter, n_claimed, &slot, group);   // also: the previous sample's LDS tiles are free
        if (p >= B) break;
        const int b = p;
        const int64_t row0 = offsets[b];
        const int L = (int)(offsets[b + 1] - row0);
        f32x16 acc[kMine];
#pragma unroll
        for (int m = 0; m < kMine; ++m)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][e] = 0.0f;
        // the next 64 rows of x and y are on their way into registers while the current ones are multiplied
        constexpr int kXLoads = 64 * (D / 8) / kFoThreads, kYLoads = 64 * (T / 8) / kFoThreads;
        u32x4 xpre[kXLoads], ypre[kYLoads];
        auto load_rows = [&](int i0) {
            const int rows = L - i0 < 64 ? L - i0 : 64;
            const u32x4 *xsrc = reinterpret_cast<const u32x4 *>(x + (row0 + i0) * D);
            const u32x4 *ysrc = reinterpret_cast<const u32x4 *>(y + (row0 + i0) * T);
#pragma unroll
            for (int u = 0; u < kXLoads; ++u) {
                const int c = tid + kFoThreads * u;
                xpre[u] = u32x4{0, 0, 0, 0};
                if (c / (D / 8) < rows) xpre[u] = xsrc[c];
            }
#pragma unroll
            for (int u = 0; u < kYLoads; ++u) {
                const int c = tid + kFoThreads * u;
                ypre[u] = u32x4{0, 0, 0, 0};
                if (c / (T / 8) < rows) ypre[u] = ysrc[c];
            }
        };
        if (L > 0) load_rows(0);
        for (int i0 = 0; i0 < L; i0 += 64) {
            if (i0) __syncthreads();
#pragma unroll
            for (int u = 0; u < kXLoads; ++u) {
                const int c = tid + kFoThreads * u;
                *reinterpret_cast<u32x4 *>(xs + (c / (D / 8)) * kXRow + (c % (D / 8)) * 16) = xpre[u];
            }
#pragma unroll
            for (int u = 0; u < kYLoads; ++u) {
                const int c = tid + kFoThreads * u;
                *reinterpret_cast<u32x4 *>(ys + (c / (T / 8)) * kYRow + (c % (T / 8)) * 16) = ypre[u];
            }
            __syncthreads();
            if (i0 + 64 < L) load_rows(i0 + 64);
#pragma unroll
            for (int m = 0; m < kMine; ++m) {
                const int blk = wave + 4 * m;   // block (db, tb) = (blk / kTBlocks, blk % kTBlocks)
                if (blk < kBlocks) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc[m] = mfma_32x32x16(tr_operand(ys, yoff, ks, blk % kTBlocks, kYRow),
                                               tr_operand(xs, xoff, ks, blk / kTBlocks, kXRow), acc[m]);
                }
            }
        }
        __syncthreads();   // the stage tiles are free: the output tile takes their place
        // register 4 g + e of block (db, tb): out[b][32 db + col][32 tb + 8 g + 4 half + e]
#pragma unroll
        for (int m = 0; m < kMine; ++m) {
            const int blk = wave + 4 * m;
            if (blk < kBlocks) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (__bf16)acc[m][4 * g + e];
                    *reinterpret_cast<bf16x4 *>(lds + ((blk / kTBlocks) * 32 + col) * kORow + ((blk % kTBlocks) * 32 + g * 8 + half * 4) * 2) = v;
                }
            }
        }
        __syncthreads();
        u32x4 *dst = reinterpret_cast<u32x4 *>(out + (int64_t)b * D * T);
        for (int c = tid; c < D * (T / 8); c += kFoThreads)
            dst[c] = *reinterpret_cast<const u32x4 *>(lds + (c / (T / 8)) * kORow + (c % (T / 8)) * 16);
    }
}

// ---- jagged_softmax and its backward: one sample per workgroup step, two sweeps over its rows ----
// A thread owns eight consecutive columns (16 bytes) and every (256 / (D / 8))-th row.  Sweep 1 gathers the
// per-column statistics (running maximum and sum of exponentials; for the backward the sum of dy y), which are
// then combined across the threads that share columns; sweep 2 writes the result.  The second sweep's reads come
// from cache for all but the longest samples.
template <int D, bool BACKWARD>
__global__ __launch_bounds__(kFoThreads) void jagged_softmax_kernel(const __bf16 *__restrict__ a,   // x, or y for the backward
                                                                    const __bf16 *__restrict__ g,   // dy (backward only)
                                                                    const int64_t *__restrict__ offsets, int B,
                                                                    int32_t *__restrict__ counter, __bf16 *__restrict__ out) {
    constexpr int kGroups = D / 8;                  // threads per row
    constexpr int kRowLanes = kFoThreads / kGroups;   // rows per sweep step
    constexpr int kBatch = 4;                         // rows per thread in flight
    __shared__ float stat_m[4][D], stat_l[4][D];
    __shared__ int slot;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = tid % kGroups, rl = tid / kGroups;
    int group = 0;
    for (int n_claimed = 0;; ++n_claimed) {
        const int p = claim_sample<(D <= 32 ? 2 : 1)>(counter, n_claimed, &slot, group);   // also: the previous sample's statistics have been read
        if (p >= B) break;
        const int b = p;
        const int64_t row0 = offsets[b];
        const int L = (int)(offsets[b + 1] - row0);
        if (L == 0) continue;
        const bf16x8 *arow = reinterpret_cast<const bf16x8 *>(a + row0 * D) + cg;
        const bf16x8 *grow = reinterpret_cast<const bf16x8 *>(g + row0 * D) + cg;
        float m[8], l[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { m[e] = -INFINITY; l[e] = 0.0f; }
        // Rows go through in batches of kBatch per thread, all of a batch's loads in flight together; the first
        // batch stays in registers for the second sweep (samples of up to kBatch * kRowLanes rows are read once).
        bf16x8 held[kBatch], held_g[BACKWARD ? kBatch : 1];
        auto load_batch = [&](int i0, bf16x8 (&v)[kBatch], bf16x8 (&d)[BACKWARD ? kBatch : 1]) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + u * kRowLanes;
                if (i < L) {
                    v[u] = arow[(int64_t)i * kGroups];
                    if (BACKWARD) d[u] = grow[(int64_t)i * kGroups];
                }
            }
        };
        auto gather = [&](int i0, const bf16x8 (&v)[kBatch], const bf16x8 (&d)[BACKWARD ? kBatch : 1]) {
            if (BACKWARD) {
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    if (i0 + u * kRowLanes >= L) break;
#pragma unroll
                    for (int e = 0; e < 8; ++e) l[e] += (float)v[u][e] * (float)d[u][e];
                }
            } else {   // the batch's maximum first: one rescaling of the running sum per batch, one exponential per element
                float bm[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) bm[e] = m[e];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    if (i0 + u * kRowLanes >= L) break;
#pragma unroll
                    for (int e = 0; e < 8; ++e) bm[e] = fmaxf(bm[e], (float)v[u][e]);
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    l[e] = m[e] == -INFINITY ? 0.0f : l[e] * __expf(m[e] - bm[e]);
                    m[e] = bm[e];
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    if (i0 + u * kRowLanes >= L) break;
#pragma unroll
                    for (int e = 0; e < 8; ++e) l[e] += __expf((float)v[u][e] - bm[e]);
                }
            }
        };
        load_batch(rl, held, held_g);
        gather(rl, held, held_g);
        for (int i0 = rl + kBatch * kRowLanes; i0 < L; i0 += kBatch * kRowLanes) {
            bf16x8 v[kBatch], d[BACKWARD ? kBatch : 1];
            load_batch(i0, v, d);
            gather(i0, v, d);
        }
        // combine the threads of a wave that share columns (lane bits above log2(kGroups)), then the four waves
#pragma unroll
        for (int d = kGroups; d < 64; d <<= 1)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float lo = __shfl_xor(l[e], d, 64);
                if (BACKWARD) l[e] += lo;
                else {
                    const float mo = __shfl_xor(m[e], d, 64), mn = fmaxf(m[e], mo);
                    l[e] = (mn == -INFINITY) ? 0.0f : l[e] * __expf(m[e] - mn) + lo * __expf(mo - mn);
                    m[e] = mn;
                }
            }
        if (lane < kGroups)
#pragma unroll
            for (int e = 0; e < 8; ++e) { stat_m[wave][cg * 8 + e] = m[e]; stat_l[wave][cg * 8 + e] = l[e]; }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (BACKWARD) l[e] = (stat_l[0][cg * 8 + e] + stat_l[1][cg * 8 + e]) + (stat_l[2][cg * 8 + e] + stat_l[3][cg * 8 + e]);
            else {
                float mn = fmaxf(fmaxf(stat_m[0][cg * 8 + e], stat_m[1][cg * 8 + e]), fmaxf(stat_m[2][cg * 8 + e], stat_m[3][cg * 8 + e]));
                float sum = 0.0f;
#pragma unroll
                for (int wv = 0; wv < 4; ++wv)
                    if (stat_m[wv][cg * 8 + e] != -INFINITY) sum += stat_l[wv][cg * 8 + e] * __expf(stat_m[wv][cg * 8 + e] - mn);
                m[e] = mn;
                l[e] = 1.0f / sum;
            }
        }
        bf16x8 *orow = reinterpret_cast<bf16x8 *>(out + row0 * D) + cg;
        auto emit = [&](int i0, const bf16x8 (&v)[kBatch], const bf16x8 (&d)[BACKWARD ? kBatch : 1]) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + u * kRowLanes;
                if (i >= L) break;
                bf16x8 r;
                if (BACKWARD) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) r[e] = (__bf16)((float)v[u][e] * ((float)d[u][e] - l[e]));
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) r[e] = (__bf16)(__expf((float)v[u][e] - m[e]) * l[e]);
                }
                orow[(int64_t)i * kGroups] = r;
            }
        };
        emit(rl, held, held_g);
        for (int i0 = rl + kBatch * kRowLanes; i0 < L; i0 += kBatch * kRowLanes) {
            bf16x8 v[kBatch], d[BACKWARD ? kBatch : 1];
            load_batch(i0, v, d);
            emit(i0, v, d);
        }
    }
}

#define JFA_DT_CASES(KERNEL, ...)                                                  \
    switch (D * 1000 + T) {                                                        \
        JFA_DT_CASE(KERNEL, 32, 32, __VA_ARGS__) JFA_DT_CASE(KERNEL, 32, 64, __VA_ARGS__) JFA_DT_CASE(KERNEL, 32, 128, __VA_ARGS__)   \
        JFA_DT_CASE(KERNEL, 64, 32, __VA_ARGS__) JFA_DT_CASE(KERNEL, 64, 64, __VA_ARGS__) JFA_DT_CASE(KERNEL, 64, 128, __VA_ARGS__)   \
        JFA_DT_CASE(KERNEL, 128, 32, __VA_ARGS__) JFA_DT_CASE(KERNEL, 128, 64, __VA_ARGS__) JFA_DT_CASE(KERNEL, 128, 128, __VA_ARGS__) \
        default: return hipErrorInvalidValue;                                      \
    }
#define JFA_DT_CASE(KERNEL, DD, TT, ...)                                                                         \
    case DD * 1000 + TT:                                                                                         \
        hipLaunchKernelGGL((KERNEL<DD, TT>), dim3(persistent_grid<KERNEL<DD, TT>>(kFoThreads, cus)), dim3(kFoThreads), 0, \
                           stream, __VA_ARGS__);                                                                 \
        break;

hipError_t launch_jagged_dense_bmm(const void *x, const void *w, const int64_t *offsets, int B, int D, int T, int32_t *counter,
                                   void *out, int cus, hipStream_t stream) {
    hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, stream, counter);
    JFA_DT_CASES(jagged_dense_bmm_kernel, (const __bf16 *)x, (const __bf16 *)w, offsets, B, counter, (__bf16 *)out)
    return hipGetLastError();
}

hipError_t launch_jagged_jagged_bmm(const void *x, const void *y, const int64_t *offsets, int B, int D, int T, int32_t *counter,
                                    void *out, int cus, hipStream_t stream) {
    hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, stream, counter);
    JFA_DT_CASES(jagged_jagged_bmm_kernel, (const __bf16 *)x, (const __bf16 *)y, offsets, B, counter, (__bf16 *)out)
    return hipGetLastError();
}
#undef JFA_DT_CASE
#undef JFA_DT_CASES

template <int D>
static hipError_t launch_softmax_d(bool backward, const __bf16 *a, const __bf16 *g, const int64_t *offsets, int B, int32_t *s,
                                   __bf16 *out, int cus, hipStream_t stream) {
    hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(64), 0, stream, s);
    if (backward)
        hipLaunchKernelGGL((jagged_softmax_kernel<D, true>), dim3(persistent_grid<jagged_softmax_kernel<D, true>>(kFoThreads, cus)),
                           dim3(kFoThreads), 0, stream, a, g, offsets, B, s, out);
    else
        hipLaunchKernelGGL((jagged_softmax_kernel<D, false>), dim3(persistent_grid<jagged_softmax_kernel<D, false>>(kFoThreads, cus)),
                           dim3(kFoThreads), 0, stream, a, g, offsets, B, s, out);
    return hipGetLastError();
}

hipError_t launch_jagged_softmax(bool backward, const void *a, const void *g, const int64_t *offsets, int B, int D,
                                 int32_t *s, void *out, int cus, hipStream_t stream) {
    switch (D) {
        case 32: return launch_softmax_d<32>(backward, (const __bf16 *)a, (const __bf16 *)g, offsets, B, s, (__bf16 *)out, cus, stream);
        case 64: return launch_softmax_d<64>(backward, (const __bf16 *)a, (const __bf16 *)g, offsets, B, s, (__bf16 *)out, cus, stream);
        case 128: return launch_softmax_d<128>(backward, (const __bf16 *)a, (const __bf16 *)g, offsets, B, s, (__bf16 *)out, cus, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace jfa

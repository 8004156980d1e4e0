// The UNFUSED jagged attention of the paper's Table 1 -- three separate jagged operators that write the score
// array to memory -- as the baseline its Section 3 compares the fused kernel with:
//   scores   jagged x jagged product with a jagged square output:  S[h, sq[b] + i L_b + j] = q_i . k_j / sqrt(D)
//   softmax  row softmax over each sample's L_b x L_b block of that array (in place)
//   apply    (jagged square array) x jagged product:                out_i = sum_j P[h, sq[b] + i L_b + j] v_j
// and the operators their gradients need (Section 2.2 builds forward and backward): the same product with a free
// scale (dP = dO V^T), the softmax's backward, and the transposed apply (dV = P^T dO, dK = dS^T Q).
// sq = [0, cumsum(L_b^2)] is the offsets array of the jagged square array (square_offsets_kernel).  The score
// array is fp32 [H, sq[B]]; q, k, v, out are bf16 [sum_B, H, D] as everywhere else.
//
// All of them are bound by HBM: what they measure is the cost of moving sum L_b^2 scores through memory several
// times, which is the point of the comparison.  They share the fused path's building blocks (one wave = 32 rows,
// v_mfma_f32_32x32x16_bf16, transposing LDS reads) but are organised around the score array: a key index sits on
// the lane axis wherever the array is touched, and stores cover whole 128-byte lines.
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kUfThreads = 256;   // four waves, 32 queries each
constexpr int kUfRows = 128;      // queries per work item (the schedule's row block)

// ---- offsets of the jagged square array: sq[b] = sum_{c < b} L_c^2 (one workgroup, any B) ----
__global__ __launch_bounds__(1024) void square_offsets_kernel(const int64_t *__restrict__ offsets, int B,
                                                               int64_t *__restrict__ sq) {
    __shared__ int64_t wave_sums[16];
    __shared__ int64_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { carry = 0; sq[0] = 0; }
    __syncthreads();
    for (int base = 0; base < B; base += 1024) {
        const int b = base + tid;
        int64_t x = 0;
        if (b < B) { const int64_t len = offsets[b + 1] - offsets[b]; x = len * len; }
        for (int d = 1; d < 64; d <<= 1) {   // inclusive scan inside the wave
            const int64_t y = __shfl_up(x, d, 64);
            if (lane >= d) x += y;
        }
        if (lane == 63) wave_sums[wave] = x;
        __syncthreads();
        int64_t before = carry;
        for (int w = 0; w < wave; ++w) before += wave_sums[w];
        if (b < B) sq[b + 1] = before + x;
        __syncthreads();
        if (tid == 1023) carry = before + x;
        __syncthreads();
    }
}

// All three operators keep a key index on the lane axis wherever they touch the score array: one wave-wide access
// covers 64 (or 2 x 32) consecutive keys of a row, so every load and store of the array is coalesced.

// ---- scores: S = scale * Q K^T (scale = 1 / sqrt(D) for the scores, 1 for dP = dO V^T) ----
// A workgroup takes 128 queries of one (sample, head); wave w holds queries 32 w .. 32 w + 31 as the A operand
// in registers for the whole item.  K streams through LDS in blocks of 64 keys shared by the four waves (rows padded
// by 16 bytes: the 16-byte operand reads of consecutive key rows fall into different banks); the block after the
// current one is already on its way into registers while the current one is multiplied.
template <int D>
__global__ __launch_bounds__(kUfThreads, 2) void unfused_scores_kernel(const __bf16 *__restrict__ q,
                                                                       const __bf16 *__restrict__ k,
                                                                       const int64_t *__restrict__ offsets,
                                                                       const int64_t *__restrict__ sq, int B, int H,
                                                                       Schedule s, float scale, float *__restrict__ scores) {
    constexpr int kKSteps = D / 16, kChunks = D / 8, kRowBytes = D * 2 + 16;
    constexpr int kLoads = 64 * kChunks / kUfThreads;   // 16-byte chunks of a K block per thread
    __shared__ __attribute__((aligned(16))) char kt[64 * kRowBytes];
    __shared__ int64_t slot;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t row_stride = (int64_t)H * D;
    const int64_t S2 = sq[B];
    WorkCursor cursor;
    for (;;) {
        const int64_t w = fetch_item(s.counter, cursor, total, &slot);
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const int q0 = t.block * kUfRows + wave * 32;   // first query of this wave
        const bool wave_active = q0 < L;
        bf16x8 qreg[kKSteps];
        {
            const int iq = q0 + col < L ? q0 + col : L - 1;
            const __bf16 *qrow = q + (t.row0 + iq) * row_stride + (int64_t)t.head * D + 8 * half;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
        }
        // Row rho of this wave starts at float index g0 + rho L of the score array; `first` is where that lands inside
        // a 256-byte window of memory (see the stores below).
        float *srow = scores + (int64_t)t.head * S2 + sq[t.sample] + (int64_t)q0 * L;
        const int g0 = __builtin_amdgcn_readfirstlane((int)((reinterpret_cast<uintptr_t>(srow) >> 2) & 63));
        auto first = [&](int rho) { return (g0 + rho * L) & 63; };
        float prev[2][16];   // the previous block's scores (same layout as `cur` below)
#pragma unroll
        for (int v = 0; v < 16; ++v) prev[0][v] = prev[1][v] = 0.0f;
        const __bf16 *kbase = k + t.row0 * row_stride + (int64_t)t.head * D;
        u32x4 kpre[kLoads];
        auto load_k = [&](int j0) {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int c = tid + kUfThreads * u, r = c / kChunks, ch = c % kChunks;
                const int jr = j0 + r < L ? j0 + r : L - 1;
                kpre[u] = *reinterpret_cast<const u32x4 *>(kbase + (int64_t)jr * row_stride + ch * 8);
            }
        };
        load_k(0);
        for (int j0 = 0; j0 < L; j0 += 64) {
            __syncthreads();   // the previous block has been consumed
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int c = tid + kUfThreads * u, r = c / kChunks, ch = c % kChunks;
                *reinterpret_cast<u32x4 *>(kt + r * kRowBytes + ch * 16) = kpre[u];
            }
            __syncthreads();
            if (j0 + 64 < L) load_k(j0 + 64);
            if (!wave_active) continue;
            f32x16 acc[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[mb][e] = 0.0f;
                const char *kp = kt + (mb * 32 + col) * kRowBytes + half * 16;
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) acc[mb] = mfma_32x32x16(qreg[ks], lds_read_b128(kp + ks * 32), acc[mb]);
            }
            // Register v of product mb: query 4 half + (v / 4) 8 + v % 4, key 32 mb + col.  Swapping the upper 32
            // lanes of product 0 with the lower 32 lanes of product 1 leaves, in each register, ONE query row and
            // the block's 64 consecutive keys across the wave.
            // A store that covers only part of a 128-byte line of memory makes the memory system read the line
            // first, and rows start at arbitrary float indices.  So each row is written in windows that are
            // 256-byte aligned in MEMORY: the window that ends inside this block takes its first `s` keys from
            // the previous block and the rest from this one, rotated across the lanes by s = first(row).
            int g = g0;
            asm volatile("" : "+s"(g));   // the per-row shifts are rebuilt per block: 32 lane masks kept across the loop would spill
            const bool interior = q0 + 32 <= L && j0 >= 64 && j0 + 64 <= L;   // every window of this block lies inside its row
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += 8) {   // sixteen rows at a time: rotate them all, then store them all
                float x[2][8];
#pragma unroll
                for (int v = v0; v < v0 + 8; ++v) {
                    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[0][v] * scale),
                                                                    __float_as_uint(acc[1][v] * scale), false, false);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int sft = (g + ((v >> 2) * 8 + (v & 3) + 4 * h) * L) & 63;
                        const float cur = __uint_as_float(r[h]);
                        const float sel = lane >= 64 - sft ? prev[h][v] : cur;
                        x[h][v - v0] = __int_as_float(__builtin_amdgcn_ds_bpermute(((lane - sft) & 63) << 2, __float_as_int(sel)));
                        prev[h][v] = cur;
                    }
                }
                if (interior) {
#pragma unroll
                    for (int v = v0; v < v0 + 8; ++v)
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const int rho = (v >> 2) * 8 + (v & 3) + 4 * h;
                            (srow + (int64_t)rho * L + (j0 - ((g + rho * L) & 63)))[lane] = x[h][v - v0];
                        }
                } else {
#pragma unroll
                    for (int v = v0; v < v0 + 8; ++v)
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const int rho = (v >> 2) * 8 + (v & 3) + 4 * h;
                            const int key = j0 - ((g + rho * L) & 63) + lane;   // this lane's key in the window
                            if (key >= 0 && key < L && q0 + rho < L) srow[(int64_t)rho * L + key] = x[h][v - v0];
                        }
                }
            }
        }
        if (wave_active) {   // the windows that hold the rows' last keys
            const int jend = (L + 63) & ~63;
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int rho = (v >> 2) * 8 + (v & 3) + 4 * h;
                    const int sft = first(rho);
                    if (jend - sft >= L) continue;   // wave-uniform
                    const float x = __int_as_float(__builtin_amdgcn_ds_bpermute(((lane - sft) & 63) << 2, __float_as_int(prev[h][v])));
                    const int key = jend - sft + lane;
                    if (key < L && q0 + rho < L) srow[(int64_t)rho * L + key] = x;
                }
        }
    }
}

// ---- row softmax, in place ----
// One wave per row, the row held in registers: the array is read once and written once.  The row is cut into
// windows that are 1024-byte aligned in memory (64 lanes x 16 bytes; stores that cover whole 128-byte lines need
// no read of the line): window u holds keys 256 u - s .. 256 u - s + 255 with s the position of the row's first
// element inside its window, and lane l owns four consecutive keys of it.  Only the first and the last window of
// a row have lanes that fall partly outside the row; they go element by element.  R = windows per lane, enough
// for rows of up to 256 R - 255 keys; longer rows take the three-pass loop below.
template <int R>
__device__ inline void softmax_row_cached(float *row, int L, int lane) {
    const int s = __builtin_amdgcn_readfirstlane((int)((reinterpret_cast<uintptr_t>(row) >> 2) & 255));
    float4 x[R];
#pragma unroll
    for (int u = 0; u < R; ++u) {
        x[u] = float4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (256 * u - s < L) {
            const int j = 256 * u - s + 4 * lane;
            if (j >= 0 && j + 3 < L) x[u] = *reinterpret_cast<const float4 *>(row + j);
            else {
                if (j >= 0 && j < L) x[u].x = row[j];
                if (j + 1 >= 0 && j + 1 < L) x[u].y = row[j + 1];
                if (j + 2 >= 0 && j + 2 < L) x[u].z = row[j + 2];
                if (j + 3 >= 0 && j + 3 < L) x[u].w = row[j + 3];
            }
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < R; ++u) m = fmaxf(fmaxf(m, fmaxf(x[u].x, x[u].y)), fmaxf(x[u].z, x[u].w));
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
    float sum = 0.0f;
#pragma unroll
    for (int u = 0; u < R; ++u) {   // exp(-inf) = 0 for the slots outside the row
        x[u].x = __expf(x[u].x - m); x[u].y = __expf(x[u].y - m); x[u].z = __expf(x[u].z - m); x[u].w = __expf(x[u].w - m);
        sum += (x[u].x + x[u].y) + (x[u].z + x[u].w);
    }
    for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (256 * u - s < L) {
            const int j = 256 * u - s + 4 * lane;
            const float4 y = float4{x[u].x * inv, x[u].y * inv, x[u].z * inv, x[u].w * inv};
            if (j >= 0 && j + 3 < L) *reinterpret_cast<float4 *>(row + j) = y;
            else {
                if (j >= 0 && j < L) row[j] = y.x;
                if (j + 1 >= 0 && j + 1 < L) row[j + 1] = y.y;
                if (j + 2 >= 0 && j + 2 < L) row[j + 2] = y.z;
                if (j + 3 >= 0 && j + 3 < L) row[j + 3] = y.w;
            }
        }
}

__device__ inline void softmax_row_streamed(float *row, int L, int lane) {
    float m = -INFINITY;
    for (int j = lane; j < L; j += 64) m = fmaxf(m, row[j]);
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
    float sum = 0.0f;
    for (int j = lane; j < L; j += 64) sum += __expf(row[j] - m);
    for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
    const float inv = 1.0f / sum;
    for (int j = lane; j < L; j += 64) row[j] = __expf(row[j] - m) * inv;
}

__global__ __launch_bounds__(kUfThreads) void unfused_softmax_kernel(const int64_t *__restrict__ offsets,
                                                                     const int64_t *__restrict__ sq, int B, int H,
                                                                     Schedule s, float *__restrict__ scores) {
    __shared__ int64_t slot;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t S2 = sq[B];
    WorkCursor cursor;
    for (;;) {
        const int64_t w = fetch_item(s.counter, cursor, total, &slot);
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        float *blk = scores + (int64_t)t.head * S2 + sq[t.sample];
        const int i0 = t.block * kUfRows + wave * 32;
        const int i1 = i0 + 32 < L ? i0 + 32 : L;
        if (L <= 256 * 2 - 255)       for (int i = i0; i < i1; ++i) softmax_row_cached<2>(blk + (int64_t)i * L, L, lane);
        else if (L <= 256 * 5 - 255)  for (int i = i0; i < i1; ++i) softmax_row_cached<5>(blk + (int64_t)i * L, L, lane);
        else if (L <= 256 * 17 - 255) for (int i = i0; i < i1; ++i) softmax_row_cached<17>(blk + (int64_t)i * L, L, lane);
        else                          for (int i = i0; i < i1; ++i) softmax_row_streamed(blk + (int64_t)i * L, L, lane);
    }
}

// ---- apply: out = P V ----
// Computed as out^T = V^T P^T on blocks of 64 keys.  Each wave reads its 32 probability rows with the key on the
// lane axis (one coalesced 256-byte load per row), rounds them to bf16 and parks them in LDS as a [key][query]
// matrix; V sits there as [key][feature].  Both operands of the product then come from transposing LDS reads of
// the same shape.  The next block's probabilities and V rows are in flight while the current block is multiplied.
template <int D>
__global__ __launch_bounds__(kUfThreads) void unfused_apply_kernel(const float *__restrict__ probs,
                                                                   const __bf16 *__restrict__ v,
                                                                   const int64_t *__restrict__ offsets,
                                                                   const int64_t *__restrict__ sq, int B, int H,
                                                                   Schedule s, __bf16 *__restrict__ out) {
    constexpr int kDBlocks = D / 32, kChunks = D / 8;
    constexpr int kVRowBytes = D == 32 ? 64 : D * 2 + 64;   // four consecutive key rows' 64-byte feature blocks: different banks
    constexpr int kLoads = 64 * kChunks / kUfThreads;
    __shared__ __attribute__((aligned(16))) char vt[64 * kVRowBytes];
    // P^T of each wave: key row kk holds 32 queries x bf16 = four 16-byte chunks, chunk u at position u ^ ((kk >> 2) & 3)
    __shared__ __attribute__((aligned(16))) char pt[4][64 * 64];
    __shared__ int64_t slot;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t row_stride = (int64_t)H * D;
    const int64_t S2 = sq[B];
    // Transposing read of this lane: key row 4 half + (lane & 15) / 4 (+8 for the operand's second half, +16 per
    // 16-key step); inside the row the 64-byte block of 32 features (or the 32 queries), bytes
    // 32 ((lane >> 4) & 1) + 8 (lane & 3).
    const int krow = half * 4 + ((lane & 15) >> 2);
    const int voff = krow * kVRowBytes + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
    const int pchunk = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    const int poff = krow * 64 + ((pchunk ^ half) << 4) + (lane & 1) * 8;
    const int poff8 = (poff + 8 * 64) ^ 32;   // second half of the operand: key rows + 8, whose chunk positions differ by 2
    char *mypt = pt[wave];
    WorkCursor cursor;
    for (;;) {
        const int64_t w = fetch_item(s.counter, cursor, total, &slot);
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const int q0 = t.block * kUfRows + wave * 32;
        const bool wave_active = q0 < L;
        const float *pblk = probs + (int64_t)t.head * S2 + sq[t.sample];
        const __bf16 *vbase = v + t.row0 * row_stride + (int64_t)t.head * D;
        f32x16 o[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
        u32x4 vpre[kLoads];
        float ppre[32];
        auto load_block = [&](int j0) {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int c = tid + kUfThreads * u, r = c / kChunks, ch = c % kChunks;
                const int jr = j0 + r < L ? j0 + r : L - 1;
                vpre[u] = *reinterpret_cast<const u32x4 *>(vbase + (int64_t)jr * row_stride + ch * 8);
            }
            if (wave_active) {
                const bool key_ok = j0 + lane < L;
#pragma unroll
                for (int r = 0; r < 32; ++r) {
                    const int i = q0 + r < L ? q0 + r : L - 1;
                    ppre[r] = key_ok ? pblk[(int64_t)i * L + j0 + lane] : 0.0f;
                }
            }
        };
        load_block(0);
        for (int j0 = 0; j0 < L; j0 += 64) {
            __syncthreads();   // the previous block has been consumed
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int c = tid + kUfThreads * u, r = c / kChunks, ch = c % kChunks;
                *reinterpret_cast<u32x4 *>(vt + r * kVRowBytes + ch * 16) = vpre[u];
            }
            if (wave_active) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    bf16x8 x;
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = (__bf16)ppre[8 * u + e];
                    *reinterpret_cast<bf16x8 *>(mypt + lane * 64 + ((u ^ ((lane >> 2) & 3)) << 4)) = x;
                }
            }
            __syncthreads();
            if (j0 + 64 < L) load_block(j0 + 64);
            if (!wave_active) continue;
#pragma unroll
            for (int ts = 0; ts < 4; ++ts) {
                if (j0 + ts * 16 >= L) break;
                const bf16x8 pb = concat(lds_read_tr16(mypt + ts * 16 * 64 + poff), lds_read_tr16(mypt + ts * 16 * 64 + poff8));
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *vp = vt + ts * 16 * kVRowBytes + voff + db * 64;
                    const bf16x8 va = concat(lds_read_tr16(vp), lds_read_tr16(vp + 8 * kVRowBytes));
                    o[db] = mfma_32x32x16(va, pb, o[db]);
                }
            }
        }
        const int i = q0 + col;
        if (i < L) {
            __bf16 *orow = out + (t.row0 + i) * row_stride + (int64_t)t.head * D;
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = (__bf16)o[db][4 * g + e];
                    *reinterpret_cast<bf16x4 *>(orow + db * 32 + g * 8 + half * 4) = x;
                }
        }
    }
}

// ---- backward of the row softmax: dS = scale * P o (dP - rowsum(P o dP)), written over dP ----
// Same shape as the forward: one wave per row, both rows held in registers as 1024-byte aligned windows (P and dP
// have the same element index, and both arrays are 16-byte aligned, so one alignment serves both).
template <int R>
__device__ inline void softmax_bwd_row_cached(const float *prow, float *grow, int L, float scale, int lane) {
    const int s = __builtin_amdgcn_readfirstlane((int)((reinterpret_cast<uintptr_t>(grow) >> 2) & 255));
    float4 p[R], g[R];
    float dot = 0.0f;
#pragma unroll
    for (int u = 0; u < R; ++u) {
        p[u] = g[u] = float4{0.0f, 0.0f, 0.0f, 0.0f};
        if (256 * u - s < L) {
            const int j = 256 * u - s + 4 * lane;
            if (j >= 0 && j + 3 < L) {
                p[u] = *reinterpret_cast<const float4 *>(prow + j);
                g[u] = *reinterpret_cast<const float4 *>(grow + j);
            } else {
                if (j >= 0 && j < L) { p[u].x = prow[j]; g[u].x = grow[j]; }
                if (j + 1 >= 0 && j + 1 < L) { p[u].y = prow[j + 1]; g[u].y = grow[j + 1]; }
                if (j + 2 >= 0 && j + 2 < L) { p[u].z = prow[j + 2]; g[u].z = grow[j + 2]; }
                if (j + 3 >= 0 && j + 3 < L) { p[u].w = prow[j + 3]; g[u].w = grow[j + 3]; }
            }
        }
        dot += (p[u].x * g[u].x + p[u].y * g[u].y) + (p[u].z * g[u].z + p[u].w * g[u].w);
    }
    for (int d = 32; d >= 1; d >>= 1) dot += __shfl_xor(dot, d, 64);
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (256 * u - s < L) {
            const int j = 256 * u - s + 4 * lane;
            const float4 y = float4{scale * p[u].x * (g[u].x - dot), scale * p[u].y * (g[u].y - dot),
                                    scale * p[u].z * (g[u].z - dot), scale * p[u].w * (g[u].w - dot)};
            if (j >= 0 && j + 3 < L) *reinterpret_cast<float4 *>(grow + j) = y;
            else {
                if (j >= 0 && j < L) grow[j] = y.x;
                if (j + 1 >= 0 && j + 1 < L) grow[j + 1] = y.y;
                if (j + 2 >= 0 && j + 2 < L) grow[j + 2] = y.z;
                if (j + 3 >= 0 && j + 3 < L) grow[j + 3] = y.w;
            }
        }
}

__device__ inline void softmax_bwd_row_streamed(const float *prow, float *grow, int L, float scale, int lane) {
    float dot = 0.0f;
    for (int j = lane; j < L; j += 64) dot += prow[j] * grow[j];
    for (int d = 32; d >= 1; d >>= 1) dot += __shfl_xor(dot, d, 64);
    for (int j = lane; j < L; j += 64) grow[j] = scale * prow[j] * (grow[j] - dot);
}

__global__ __launch_bounds__(kUfThreads) void unfused_softmax_bwd_kernel(const float *__restrict__ probs,
                                                                         const int64_t *__restrict__ offsets,
                                                                         const int64_t *__restrict__ sq, int B, int H,
                                                                         Schedule s, float scale, float *dprobs) {
    __shared__ int64_t slot;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t S2 = sq[B];
    WorkCursor cursor;
    for (;;) {
        const int64_t w = fetch_item(s.counter, cursor, total, &slot);
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const int64_t blk = (int64_t)t.head * S2 + sq[t.sample];
        const int i0 = t.block * kUfRows + wave * 32;
        const int i1 = i0 + 32 < L ? i0 + 32 : L;
        for (int i = i0; i < i1; ++i) {
            const float *prow = probs + blk + (int64_t)i * L;
            float *grow = dprobs + blk + (int64_t)i * L;
            if (L <= 256 * 2 - 255) softmax_bwd_row_cached<2>(prow, grow, L, scale, lane);
            else if (L <= 256 * 5 - 255) softmax_bwd_row_cached<5>(prow, grow, L, scale, lane);
            else if (L <= 256 * 17 - 255) softmax_bwd_row_cached<17>(prow, grow, L, scale, lane);
            else softmax_bwd_row_streamed(prow, grow, L, scale, lane);
        }
    }
}

// ---- transposed apply: out_j = sum_i X[i, j] x_i  (dV = P^T dO, dK = dS^T Q) ----
// Computed as out^T = x^T X on blocks of 64 rows i.  A wave owns 32 output rows j.  With the slot order of the
// transposing read that delivers x^T (row i of a 16-row step in slot order 4 half + e, 8 + 4 half + e), the
// B operand of lane (col, half) is the column j = col of exactly those rows of X: each of its loads covers 32
// consecutive j of one row (two rows per instruction), straight from memory into operand position.  x goes
// through LDS as [i][feature], shared by the four waves; the next block is in flight during the products.
template <int D>
__global__ __launch_bounds__(kUfThreads, 2) void unfused_apply_t_kernel(const float *__restrict__ X,
                                                                     const __bf16 *__restrict__ x,
                                                                     const int64_t *__restrict__ offsets,
                                                                     const int64_t *__restrict__ sq, int B, int H,
                                                                     Schedule s, __bf16 *__restrict__ out) {
    constexpr int kDBlocks = D / 32, kChunks = D / 8;
    constexpr int kRowBytes = D == 32 ? 64 : D * 2 + 64;
    constexpr int kLoads = 64 * kChunks / kUfThreads;
    __shared__ __attribute__((aligned(16))) char xt[64 * kRowBytes];
    __shared__ int64_t slot;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t total = (int64_t)s.tile_start[B] * H;
    const int64_t row_stride = (int64_t)H * D;
    const int64_t S2 = sq[B];
    const int xoff = (half * 4 + ((lane & 15) >> 2)) * kRowBytes + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
    WorkCursor cursor;
    for (;;) {
        const int64_t w = fetch_item(s.counter, cursor, total, &slot);
        if (w < 0) break;
        const Work t = decode_work(s, offsets, B, H, w);
        const int L = t.len;
        const int j = t.block * kUfRows + wave * 32 + col;   // this lane's output row
        const bool wave_active = t.block * kUfRows + wave * 32 < L;
        const bool j_ok = j < L;
        const float *xcol = X + (int64_t)t.head * S2 + sq[t.sample] + (j_ok ? j : 0);   // X[i, j] = xcol[i * L]
        const __bf16 *xbase = x + t.row0 * row_stride + (int64_t)t.head * D;
        f32x16 o[kDBlocks];
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
        u32x4 xpre[kLoads];
        float cpre[32];   // slot e of step ks: row i0 + 16 ks + (e / 4) 8 + 4 half + e % 4
        auto load_block = [&](int i0) {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int c = tid + kUfThreads * u, r = c / kChunks, ch = c % kChunks;
                const int ir = i0 + r < L ? i0 + r : L - 1;
                xpre[u] = *reinterpret_cast<const u32x4 *>(xbase + (int64_t)ir * row_stride + ch * 8);
            }
            if (wave_active) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int i = i0 + 16 * ks + (e >> 2) * 8 + 4 * half + (e & 3);
                        cpre[8 * ks + e] = (j_ok && i < L) ? xcol[(int64_t)i * L] : 0.0f;
                    }
            }
        };
        load_block(0);
        for (int i0 = 0; i0 < L; i0 += 64) {
            __syncthreads();   // the previous block of x has been consumed
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int c = tid + kUfThreads * u, r = c / kChunks, ch = c % kChunks;
                *reinterpret_cast<u32x4 *>(xt + r * kRowBytes + ch * 16) = xpre[u];
            }
            bf16x8 cb[4];
            if (wave_active) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int e = 0; e < 8; ++e) cb[ks][e] = (__bf16)cpre[8 * ks + e];
            }
            __syncthreads();
            if (i0 + 64 < L) load_block(i0 + 64);
            if (!wave_active) continue;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (i0 + ks * 16 >= L) break;
#pragma unroll
                for (int db = 0; db < kDBlocks; ++db) {
                    const char *p = xt + ks * 16 * kRowBytes + xoff + db * 64;
                    o[db] = mfma_32x32x16(concat(lds_read_tr16(p), lds_read_tr16(p + 8 * kRowBytes)), cb[ks], o[db]);
                }
            }
        }
        if (j_ok) {
            __bf16 *orow = out + (t.row0 + j) * row_stride + (int64_t)t.head * D;
#pragma unroll
            for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (__bf16)o[db][4 * g + e];
                    *reinterpret_cast<bf16x4 *>(orow + db * 32 + g * 8 + half * 4) = v;
                }
        }
    }
}

hipError_t launch_square_offsets(const int64_t *offsets, int B, int64_t *sq, hipStream_t stream) {
    hipLaunchKernelGGL(square_offsets_kernel, dim3(1), dim3(1024), 0, stream, offsets, B, sq);
    return hipGetLastError();
}

hipError_t launch_unfused_scores(const void *q, const void *k, const int64_t *offsets, const int64_t *sq, int B, int H,
                                 int D, Schedule s, float scale, float *scores, int cus, hipStream_t stream) {
#define JFA_CASE(DD)                                                                                                \
    case DD:                                                                                                        \
        hipLaunchKernelGGL(unfused_scores_kernel<DD>, dim3(persistent_grid<unfused_scores_kernel<DD>>(kUfThreads, cus)), \
                           dim3(kUfThreads), 0, stream, (const __bf16 *)q, (const __bf16 *)k, offsets, sq, B, H, s, scale, scores); \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

hipError_t launch_unfused_softmax(const int64_t *offsets, const int64_t *sq, int B, int H, Schedule s, float *scores,
                                  int cus, hipStream_t stream) {
    hipLaunchKernelGGL(unfused_softmax_kernel, dim3(persistent_grid<unfused_softmax_kernel>(kUfThreads, cus)),
                       dim3(kUfThreads), 0, stream, offsets, sq, B, H, s, scores);
    return hipGetLastError();
}

hipError_t launch_unfused_apply(const float *probs, const void *v, const int64_t *offsets, const int64_t *sq, int B,
                                int H, int D, Schedule s, void *out, int cus, hipStream_t stream) {
#define JFA_CASE(DD)                                                                                               \
    case DD:                                                                                                       \
        hipLaunchKernelGGL(unfused_apply_kernel<DD>, dim3(persistent_grid<unfused_apply_kernel<DD>>(kUfThreads, cus)), \
                           dim3(kUfThreads), 0, stream, probs, (const __bf16 *)v, offsets, sq, B, H, s, (__bf16 *)out); \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

hipError_t launch_unfused_softmax_bwd(const float *probs, const int64_t *offsets, const int64_t *sq, int B, int H,
                                      Schedule s, float scale, float *dprobs, int cus, hipStream_t stream) {
    hipLaunchKernelGGL(unfused_softmax_bwd_kernel, dim3(persistent_grid<unfused_softmax_bwd_kernel>(kUfThreads, cus)),
                       dim3(kUfThreads), 0, stream, probs, offsets, sq, B, H, s, scale, dprobs);
    return hipGetLastError();
}

hipError_t launch_unfused_apply_t(const float *X, const void *x, const int64_t *offsets, const int64_t *sq, int B, int H,
                                  int D, Schedule s, void *out, int cus, hipStream_t stream) {
#define JFA_CASE(DD)                                                                                                   \
    case DD:                                                                                                           \
        hipLaunchKernelGGL(unfused_apply_t_kernel<DD>, dim3(persistent_grid<unfused_apply_t_kernel<DD>>(kUfThreads, cus)), \
                           dim3(kUfThreads), 0, stream, X, (const __bf16 *)x, offsets, sq, B, H, s, (__bf16 *)out);     \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

}  // namespace jfa

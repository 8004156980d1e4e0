// fp32 jagged attention, forward and backward, in plain FMA arithmetic (no matrix cores): the
// small-tolerance path.  Same structure as the bf16 kernels -- persistent workgroups pull
// (sample, head, row-block) tiles from the offsets-driven schedule, stream the sample's keys
// through LDS and keep an online softmax in registers (paper Section 2.1) -- but one row is owned
// by four neighbouring lanes, each holding every fourth element of the row.
#include "jfa_common.h"

namespace jfa {

constexpr int kRows = kF32BlockRows;  // rows (queries or keys) per tile
// streamed rows per LDS stage: two [cols][D] fp32 stages stay within 32 KB
template <int D> constexpr int cols_for() { return 4096 / D < 64 ? 4096 / D : 64; }
static_assert(2 * cols_for<32>() * 32 >= kInlineScratchInts && 2 * cols_for<128>() * 128 >= kInlineScratchInts,
              "the two stage buffers double as the in-kernel scheduler's scratch");
constexpr int kThreads = kRows * 4;

__device__ inline float quad_sum(float x) {
    x += __shfl_xor(x, 1, 64);
    x += __shfl_xor(x, 2, 64);
    return x;
}

// Copy `n` rows (row0 .. row0+n-1, head h) of a [*, H, D] fp32 tensor into LDS [n][D].
template <int D>
__device__ inline void stage_rows(float *dst, const float *__restrict__ src, int64_t row0, int n, int h, int H) {
    constexpr int kVec = D / 4;
    for (int i = threadIdx.x; i < n * kVec; i += kThreads) {
        const int r = i / kVec, c = i - r * kVec;
        const float4 x = *reinterpret_cast<const float4 *>(src + ((row0 + r) * H + h) * (int64_t)D + c * 4);
        *reinterpret_cast<float4 *>(dst + r * D + c * 4) = x;
    }
}

__device__ inline int64_t fetch_work(int32_t *counters, WorkCursor &probe, int64_t total, int64_t *slot) {
    __syncthreads();
    if (threadIdx.x == 0) *slot = next_work(counters, probe, total);
    __syncthreads();
    return uniform64(*slot);
}

template <int D>
__global__ __launch_bounds__(kThreads) void fwd_f32_kernel(const float *__restrict__ q, const float *__restrict__ k,
                                                           const float *__restrict__ v,
                                                           const int64_t *__restrict__ offsets,
                                                           const int64_t *__restrict__ offsets_kv, bool causal,
                                                           int B, int H, Schedule s, float *__restrict__ out,
                                                           float *__restrict__ lse) {
    constexpr int kPer = D / 4;
    constexpr int kCols = cols_for<D>();
    __shared__ float KVs[2 * kCols * D];   // staged K rows, then V rows (the schedule build borrows all of it)
    float *const Ks = KVs, *const Vs = KVs + kCols * D;
    __shared__ int64_t slot;
    WorkCursor probe;
    const int r = threadIdx.x >> 2, c = threadIdx.x & 3;
    const float scale = 1.0f / sqrtf((float)D);
    __shared__ SmallWork mine;
    const bool small = s.build_rows != 0;   // small problem: no scheduler launch has run, the schedule is built here, in LDS
    if (small) build_small_work(offsets, offsets_kv, B, H, s.build_rows, reinterpret_cast<int *>(KVs), &mine);
    probe.static_only = s.static_only;
    const int64_t total = small ? 0 : (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];

    for (int n = 0;; ++n) {
        Work t;   // keys: rows orow0 .. orow0 + olen - 1
        if (small) {   // the workgroup's items were decoded when the schedule was built
            __syncthreads();   // the previous item's use of the staging arrays is over
            if (n >= __builtin_amdgcn_readfirstlane(mine.count) || !load_work<true>(&mine.item[n], t)) break;
        } else {
            const int64_t w = fetch_work(s.counter, probe, total, &slot);
            if (w < 0) break;
            t = decode_work(s, offsets, B, H, w, offsets_kv);
        }
        const int i = t.block * kRows + r;                    // query index inside the sample
        const int iq = i < t.len ? i : t.len - 1;             // rows past the end recompute the last row
        float qr[kPer], acc[kPer];
        for (int e = 0; e < kPer; ++e) {
            qr[e] = q[((t.row0 + iq) * H + t.head) * (int64_t)D + 4 * e + c];
            acc[e] = 0.0f;
        }
        float m = -INFINITY, l = 0.0f;
        // causal (self attention only): query i sees keys 0 .. i, so the tile needs the keys up to its last query
        const int kend = causal && (t.block + 1) * kRows < t.olen ? (t.block + 1) * kRows : t.olen;
        for (int j0 = 0; j0 < kend; j0 += kCols) {
            const int n = kend - j0 < kCols ? kend - j0 : kCols;
            __syncthreads();
            stage_rows<D>(Ks, k, t.orow0 + j0, n, t.head, H);
            stage_rows<D>(Vs, v, t.orow0 + j0, n, t.head, H);
            __syncthreads();
            for (int j = 0; j < n; ++j) {
                float part = 0.0f;
                for (int e = 0; e < kPer; ++e) part = fmaf(qr[e], Ks[j * D + 4 * e + c], part);
                const float sc = causal && j0 + j > iq ? -INFINITY : quad_sum(part) * scale;   // key 0 is never masked: m stays finite
                const float m_new = fmaxf(m, sc);
                const float a = expf(m - m_new);              // exp(-inf) = 0 on the first key
                const float p = expf(sc - m_new);
                l = fmaf(l, a, p);
                for (int e = 0; e < kPer; ++e) acc[e] = fmaf(acc[e], a, p * Vs[j * D + 4 * e + c]);
                m = m_new;
            }
        }
        if (i < t.len) {
            const float inv = l > 0.0f ? 1.0f / l : 0.0f;   // a sample without keys: out = 0, lse = -inf
            for (int e = 0; e < kPer; ++e) out[((t.row0 + i) * H + t.head) * (int64_t)D + 4 * e + c] = acc[e] * inv;
            if (c == 0) lse[(int64_t)t.head * sum_B + t.row0 + i] = m + logf(l);
        }
    }
}

// dQ: tile = 64 queries, stream the sample's keys.  The kernel is the first of the backward: it holds each query's dO
// row anyway, reads the matching row of the forward's output, and computes delta = rowsum(dO o O) for its own use
// and for the dK / dV kernel (no separate pass over dO and O, one launch less).
template <int D>
__global__ __launch_bounds__(kThreads) void dq_f32_kernel(const float *__restrict__ q, const float *__restrict__ k,
                                                          const float *__restrict__ v,
                                                          const float *__restrict__ out_fwd,
                                                          const float *__restrict__ dout,
                                                          const float *__restrict__ lse,
                                                          float *__restrict__ delta,
                                                          const int64_t *__restrict__ offsets,
                                                          const int64_t *__restrict__ offsets_kv, bool causal,
                                                          int B, int H, Schedule s, float *__restrict__ dq) {
    constexpr int kPer = D / 4;
    constexpr int kCols = cols_for<D>();
    __shared__ float KVs[2 * kCols * D];   // staged K rows, then V rows (the schedule build borrows all of it)
    float *const Ks = KVs, *const Vs = KVs + kCols * D;
    __shared__ int64_t slot;
    WorkCursor probe;
    const int r = threadIdx.x >> 2, c = threadIdx.x & 3;
    const float scale = 1.0f / sqrtf((float)D);
    __shared__ SmallWork mine;
    const bool small = s.build_rows != 0;   // small problem: no scheduler launch has run, the schedule is built here, in LDS
    if (small) build_small_work(offsets, offsets_kv, B, H, s.build_rows, reinterpret_cast<int *>(KVs), &mine);
    probe.static_only = s.static_only;
    const int64_t total = small ? 0 : (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets[B];

    for (int n = 0;; ++n) {
        Work t;
        if (small) {   // the workgroup's items were decoded when the schedule was built
            __syncthreads();   // the previous item's use of the staging arrays is over
            if (n >= __builtin_amdgcn_readfirstlane(mine.count) || !load_work<true>(&mine.item[n], t)) break;
        } else {
            const int64_t w = fetch_work(s.counter, probe, total, &slot);
            if (w < 0) break;
            t = decode_work(s, offsets, B, H, w, offsets_kv);
        }
        const int i = t.block * kRows + r;
        const int iq = i < t.len ? i : t.len - 1;
        float qr[kPer], dor[kPer], acc[kPer];
        float dot = 0.0f;
        for (int e = 0; e < kPer; ++e) {
            const int64_t idx = ((t.row0 + iq) * H + t.head) * (int64_t)D + 4 * e + c;
            qr[e] = q[idx];
            dor[e] = dout[idx];
            dot = fmaf(dor[e], out_fwd[idx], dot);
            acc[e] = 0.0f;
        }
        const float lse_i = lse[(int64_t)t.head * sum_B + t.row0 + iq];
        const float delta_i = quad_sum(dot);   // the four lanes of a row hold a quarter of its features each
        if (i < t.len && c == 0) delta[(int64_t)t.head * sum_B + t.row0 + i] = delta_i;
        // causal (self attention only): query i sees keys 0 .. i, so the tile needs the keys up to its last query
        const int kend = causal && (t.block + 1) * kRows < t.olen ? (t.block + 1) * kRows : t.olen;
        for (int j0 = 0; j0 < kend; j0 += kCols) {
            const int n = kend - j0 < kCols ? kend - j0 : kCols;
            __syncthreads();
            stage_rows<D>(Ks, k, t.orow0 + j0, n, t.head, H);
            stage_rows<D>(Vs, v, t.orow0 + j0, n, t.head, H);
            __syncthreads();
            for (int j = 0; j < n; ++j) {
                float ps = 0.0f, pd = 0.0f;
                for (int e = 0; e < kPer; ++e) {
                    ps = fmaf(qr[e], Ks[j * D + 4 * e + c], ps);
                    pd = fmaf(dor[e], Vs[j * D + 4 * e + c], pd);
                }
                const float p = causal && j0 + j > iq ? 0.0f : expf(quad_sum(ps) * scale - lse_i);
                const float ds = p * (quad_sum(pd) - delta_i);
                for (int e = 0; e < kPer; ++e) acc[e] = fmaf(ds, Ks[j * D + 4 * e + c], acc[e]);
            }
        }
        if (i < t.len)
            for (int e = 0; e < kPer; ++e) dq[((t.row0 + i) * H + t.head) * (int64_t)D + 4 * e + c] = acc[e] * scale;
    }
}

// dK, dV: tile = 64 keys, stream the sample's queries (with their dO, lse, delta).
template <int D>
__global__ __launch_bounds__(kThreads) void dkv_f32_kernel(const float *__restrict__ q, const float *__restrict__ k,
                                                           const float *__restrict__ v,
                                                           const float *__restrict__ dout,
                                                           const float *__restrict__ lse,
                                                           const float *__restrict__ delta,
                                                           const int64_t *__restrict__ offsets,   // of the keys
                                                           const int64_t *__restrict__ offsets_q, bool causal,
                                                           int B, int H, Schedule s, float *__restrict__ dk,
                                                           float *__restrict__ dv) {
    constexpr int kPer = D / 4;
    constexpr int kCols = cols_for<D>();
    __shared__ float QOs[2 * kCols * D];   // staged Q rows, then dO rows (the schedule build borrows all of it)
    float *const Qs = QOs, *const Os = QOs + kCols * D;
    __shared__ float lse_s[kCols];
    __shared__ float delta_s[kCols];
    __shared__ int64_t slot;
    WorkCursor probe;
    const int r = threadIdx.x >> 2, c = threadIdx.x & 3;
    const float scale = 1.0f / sqrtf((float)D);
    __shared__ SmallWork mine;
    const bool small = s.build_rows != 0;   // small problem: no scheduler launch has run, the schedule is built here, in LDS
    if (small) build_small_work(offsets, offsets_q, B, H, s.build_rows, reinterpret_cast<int *>(QOs), &mine);
    probe.static_only = s.static_only;
    const int64_t total = small ? 0 : (int64_t)s.tile_start[B] * H;
    const int64_t sum_B = offsets_q ? offsets_q[B] : offsets[B];   // lse and delta are indexed by query rows

    for (int n = 0;; ++n) {
        Work t;   // queries: rows orow0 .. orow0 + olen - 1
        if (small) {   // the workgroup's items were decoded when the schedule was built
            __syncthreads();   // the previous item's use of the staging arrays is over
            if (n >= __builtin_amdgcn_readfirstlane(mine.count) || !load_work<true>(&mine.item[n], t)) break;
        } else {
            const int64_t w = fetch_work(s.counter, probe, total, &slot);
            if (w < 0) break;
            t = decode_work(s, offsets, B, H, w, offsets_q);
        }
        const int j = t.block * kRows + r;
        const int jk = j < t.len ? j : t.len - 1;
        float kr[kPer], vr[kPer], acck[kPer], accv[kPer];
        for (int e = 0; e < kPer; ++e) {
            const int64_t idx = ((t.row0 + jk) * H + t.head) * (int64_t)D + 4 * e + c;
            kr[e] = k[idx];
            vr[e] = v[idx];
            acck[e] = 0.0f;
            accv[e] = 0.0f;
        }
        // causal: key j is seen by queries j .. L - 1, so the stream starts at the stage that holds the tile's first key
        const int istart = causal ? (t.block * kRows / kCols) * kCols : 0;
        for (int i0 = istart; i0 < t.olen; i0 += kCols) {
            const int n = t.olen - i0 < kCols ? t.olen - i0 : kCols;
            __syncthreads();
            stage_rows<D>(Qs, q, t.orow0 + i0, n, t.head, H);
            stage_rows<D>(Os, dout, t.orow0 + i0, n, t.head, H);
            if (threadIdx.x < n) {
                lse_s[threadIdx.x] = lse[(int64_t)t.head * sum_B + t.orow0 + i0 + threadIdx.x];
                delta_s[threadIdx.x] = delta[(int64_t)t.head * sum_B + t.orow0 + i0 + threadIdx.x];
            }
            __syncthreads();
            for (int i = 0; i < n; ++i) {
                float ps = 0.0f, pd = 0.0f;
                for (int e = 0; e < kPer; ++e) {
                    ps = fmaf(Qs[i * D + 4 * e + c], kr[e], ps);
                    pd = fmaf(Os[i * D + 4 * e + c], vr[e], pd);
                }
                const float p = causal && i0 + i < jk ? 0.0f : expf(quad_sum(ps) * scale - lse_s[i]);
                const float ds = p * (quad_sum(pd) - delta_s[i]);
                for (int e = 0; e < kPer; ++e) {
                    accv[e] = fmaf(p, Os[i * D + 4 * e + c], accv[e]);
                    acck[e] = fmaf(ds, Qs[i * D + 4 * e + c], acck[e]);
                }
            }
        }
        if (j < t.len)
            for (int e = 0; e < kPer; ++e) {
                const int64_t idx = ((t.row0 + j) * H + t.head) * (int64_t)D + 4 * e + c;
                dk[idx] = acck[e] * scale;
                dv[idx] = accv[e];
            }
    }
}

hipError_t launch_fwd_f32(const float *q, const float *k, const float *v, const int64_t *offsets,
                          const int64_t *offsets_kv, bool causal, int B, int H, int D, Schedule s, float *out, float *lse,
                          int cus, hipStream_t stream) {
#define JFA_CASE(DD)                                                                                              \
    case DD:                                                                                                      \
        hipLaunchKernelGGL(fwd_f32_kernel<DD>, dim3(persistent_grid<fwd_f32_kernel<DD>>(kThreads, cus)), dim3(kThreads), 0, stream, q, k, v, offsets, offsets_kv, causal, B, H, s, \
                           out, lse);                                                                             \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

hipError_t launch_bwd_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                          const float *lse, const int64_t *offsets, const int64_t *offsets_kv, bool causal, int B, int H,
                          int D, Schedule s_dq, Schedule s_dkv, float *dq, float *dk, float *dv, float *delta, int cus,
                          hipStream_t stream) {
#define JFA_CASE(DD)                                                                                               \
    case DD:                                                                                                       \
        hipLaunchKernelGGL(dq_f32_kernel<DD>, dim3(persistent_grid<dq_f32_kernel<DD>>(kThreads, cus)), dim3(kThreads), 0, stream, q, k, v, out, dout, lse, delta,   \
                           offsets, offsets_kv, causal, B, H, s_dq, dq);                                           \
        hipLaunchKernelGGL(dkv_f32_kernel<DD>, dim3(persistent_grid<dkv_f32_kernel<DD>>(kThreads, cus)), dim3(kThreads), 0, stream, q, k, v, dout, lse, delta,  \
                           offsets_kv ? offsets_kv : offsets, offsets_kv ? offsets : nullptr, causal, B, H, s_dkv, dk, dv);  \
        break;
    switch (D) {
        JFA_CASE(32) JFA_CASE(64) JFA_CASE(128)
        default: return hipErrorInvalidValue;
    }
#undef JFA_CASE
    return hipGetLastError();
}

}  // namespace jfa

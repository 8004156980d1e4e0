// extern "C" entry points of libjfa.so: argument validation, the private work table and the
// sequence of kernel launches of each call.  See include/jfa.h for the contract.
#include <map>
#include <mutex>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <utility>
#include <vector>

#include "../../include/jfa.h"
#include "jfa_common.h"

namespace {

thread_local char g_err[512] = "";

int fail(jfa_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return (int)st;
}

// ---- private work table: [kNumCounters counters][2 x (order[B], tile_start[B+1])] per (device, stream) ----
struct Table {
    char *base = nullptr;
    size_t bytes = 0;
};
std::mutex g_mu;
std::map<std::pair<int, hipStream_t>, Table> g_tables;
std::map<int, int> g_cu_count;

constexpr size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
constexpr size_t sched_bytes(int64_t B) { return align_up((size_t)(2 * B + 1) * sizeof(int32_t), 256); }
constexpr size_t table_bytes(int64_t B) { return (size_t)jfa::kNumCounters * sizeof(int32_t) + 2 * sched_bytes(B); }

struct Views {
    int32_t *counters;
    int32_t *order[2];
    int32_t *tile_start[2];
    int cus;
};

// [counters][order 0, tile_start 0][order 1, tile_start 1] for a batch of B samples, from `base` on
void lay_out(char *base, int64_t B, Views *v) {
    v->counters = (int32_t *)base;
    char *p = base + (size_t)jfa::kNumCounters * sizeof(int32_t);
    for (int i = 0; i < 2; ++i) {
        v->order[i] = (int32_t *)p;
        v->tile_start[i] = v->order[i] + B;
        p += sched_bytes(B);
    }
}

int get_table(int64_t B, hipStream_t stream, Views *v) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(JFA_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    std::lock_guard<std::mutex> lock(g_mu);
    auto cu = g_cu_count.find(dev);
    if (cu == g_cu_count.end()) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || n <= 0) return fail(JFA_ERR_HIP, "cannot read the compute-unit count: %s", hipGetErrorString(e));
        cu = g_cu_count.emplace(dev, n).first;
    }
    Table &t = g_tables[std::make_pair(dev, stream)];
    const size_t need = table_bytes(B);
    if (t.bytes < need) {
        // Grow.  The old table may still be in use by work enqueued earlier on this stream.
        if (t.base) {
            e = hipStreamSynchronize(stream);
            if (e != hipSuccess) return fail(JFA_ERR_HIP, "hipStreamSynchronize: %s", hipGetErrorString(e));
            (void)hipFree(t.base);
            t.base = nullptr;
            t.bytes = 0;
        }
        void *p = nullptr;
        e = hipMalloc(&p, need);
        if (e != hipSuccess) return fail(JFA_ERR_ALLOC, "hipMalloc(%zu) for the work table: %s", need, hipGetErrorString(e));
        t.base = (char *)p;
        t.bytes = need;
    }
    // Views are laid out for the table's capacity in bytes, not for this call's B: recompute from B.
    lay_out(t.base, B, v);
    v->cus = cu->second;
    return JFA_OK;
}

// ---- the work table of jfa_forward_noalloc: a fixed array in device memory, one copy per GPU ----
// In host code the array's name is only a handle for hipGetSymbolAddress; every use of its memory goes through the
// per-device pointer obtained from that call.
constexpr size_t kScratchBytes = table_bytes(JFA_NOALLOC_MAX_B);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
struct StaticTable {
    char *ptr = nullptr;   // device address of `scratch` on this device
    int cus = 0;
};
StaticTable g_static[kMaxDevices];

int get_static_table(int64_t B, Views *v) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(JFA_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(JFA_ERR_UNSUPPORTED, "device index %d is beyond the %d this call keeps a table for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_mu);
    StaticTable &t = g_static[dev];
    if (!t.ptr) {   // first call on this device (which is current): ask for this device's copy of the array
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(JFA_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || n <= 0) return fail(JFA_ERR_HIP, "cannot read the compute-unit count: %s", hipGetErrorString(e));
        t.cus = n;
        t.ptr = (char *)p;
    }
    lay_out(t.ptr, B, v);
    v->cus = t.cus;
    return JFA_OK;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

int check_common(const char *fn, int64_t B, int64_t max_len, int H, int D, const void *const *ptrs, int n_ptrs) {
    if (B < 0) return fail(JFA_ERR_INVALID_ARG, "%s: B = %lld is negative", fn, (long long)B);
    if (max_len < 0) return fail(JFA_ERR_INVALID_ARG, "%s: max_len = %lld is negative", fn, (long long)max_len);
    if (H <= 0) return fail(JFA_ERR_INVALID_ARG, "%s: H = %d must be positive", fn, H);
    if (D != 32 && D != 64 && D != 128) return fail(JFA_ERR_UNSUPPORTED, "%s: D = %d is not one of 32, 64, 128", fn, D);
    if (B >= (int64_t)1 << 30) return fail(JFA_ERR_UNSUPPORTED, "%s: B = %lld is too large", fn, (long long)B);
    if (B == 0) return JFA_OK;
    for (int i = 0; i < n_ptrs; ++i) {
        if (!ptrs[i]) return fail(JFA_ERR_INVALID_ARG, "%s: pointer argument %d is null", fn, i);
        if (misaligned(ptrs[i])) return fail(JFA_ERR_INVALID_ARG, "%s: pointer argument %d is not 16-byte aligned", fn, i);
    }
    return JFA_OK;
}

// ---- optional per-kernel timing (see jfa_timing_enable) ----
struct TimedLaunch {
    const char *name;
    hipEvent_t e0, e1;
};
thread_local bool g_timing = false;
thread_local bool g_timing_suppressed = false;   // inside jfa_forward_noalloc: creating events would allocate
thread_local std::vector<TimedLaunch> g_timed;

// Brackets one kernel launch with events when timing is on; a no-op otherwise.
struct ScopedTimer {
    TimedLaunch t{nullptr, nullptr, nullptr};
    hipStream_t stream;
    ScopedTimer(const char *name, hipStream_t s) : stream(s) {
        if (!g_timing || g_timing_suppressed) return;
        if (hipEventCreate(&t.e0) != hipSuccess) return;
        if (hipEventCreate(&t.e1) != hipSuccess) { (void)hipEventDestroy(t.e0); return; }
        t.name = name;
        (void)hipEventRecord(t.e0, stream);
    }
    ~ScopedTimer() {
        if (!t.name) return;
        (void)hipEventRecord(t.e1, stream);
        g_timed.push_back(t);
    }
};

void drop_timed() {
    for (auto &t : g_timed) { (void)hipEventDestroy(t.e0); (void)hipEventDestroy(t.e1); }
    g_timed.clear();
}

// Forward variant: the direct-to-LDS kernel for long samples at D = 128, the register-staged one otherwise.
enum FwdVariant { kNarrow = 0, kDma = 2 };
FwdVariant forward_variant(int64_t max_len, int D, int H) {
    if (D != 128 || (int64_t)H * D > (1 << 20)) return kNarrow;   // the direct-to-LDS kernels keep 32-bit row offsets
    return max_len > 256 ? kDma : kNarrow;   // 256-query tiles only pay off when samples can be long
}

// Small problems skip the scheduler launch: the attention kernels build the schedule themselves and deal the work
// statically (see build_small_work).  max_len bounds every sample's length, so B * blocks(max_len) * H bounds
// the number of work items; at most four per workgroup is the size up to which static dealing is used anyway.
bool small_problem(int64_t B, int64_t max_len, int H, int block_rows, int cus) {
    if (B > jfa::kInlineCap) return false;
    const int64_t blocks = (max_len + block_rows - 1) / block_rows;
    return B * (blocks > 0 ? blocks : 1) * (int64_t)H <= 4 * (int64_t)cus;
}

int hip_fail(const char *what, hipError_t e) { return fail(JFA_ERR_HIP, "%s: %s", what, hipGetErrorString(e)); }

}  // namespace

extern "C" {

const char *jfa_last_error(void) { return g_err; }

int jfa_timing_enable(int on) {
    drop_timed();
    g_timing = on != 0;
    return JFA_OK;
}

int jfa_timing_read(int capacity, const char **names, float *total_ms, int *launches) {
    if (capacity < 0 || (capacity > 0 && (!names || !total_ms || !launches)))
        return fail(JFA_ERR_INVALID_ARG, "jfa_timing_read: null output array");
    int n = 0;
    for (auto &t : g_timed) {
        hipError_t e = hipEventSynchronize(t.e1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.e0, t.e1);
        if (e != hipSuccess) { drop_timed(); return hip_fail("timing events", e); }
        int i = 0;
        while (i < n && strcmp(names[i], t.name) != 0) ++i;
        if (i == n) {
            if (n == capacity) continue;
            names[n] = t.name; total_ms[n] = 0.0f; launches[n] = 0; ++n;
        }
        total_ms[i] += ms;
        launches[i] += 1;
    }
    drop_timed();
    return n;
}
int jfa_version(void) { return 100; }

size_t jfa_workspace_bytes(int64_t B, int64_t max_len, int H, int D, int pass) {
    (void)max_len; (void)H; (void)D; (void)pass;
    return B > 0 ? table_bytes(B) : 0;
}

int jfa_build_schedule(const int64_t *offsets, int64_t B, int block_rows, int32_t *order, int32_t *tile_start,
                       void *stream) {
    if (B < 0 || B >= (int64_t)1 << 30) return fail(JFA_ERR_INVALID_ARG, "jfa_build_schedule: bad B");
    if (block_rows <= 0 || block_rows % 32) return fail(JFA_ERR_INVALID_ARG, "jfa_build_schedule: block_rows = %d must be a positive multiple of 32", block_rows);
    if (!offsets || !tile_start || (B > 0 && !order)) return fail(JFA_ERR_INVALID_ARG, "jfa_build_schedule: null pointer");
    Views v;
    int st = get_table(B, (hipStream_t)stream, &v);
    if (st != JFA_OK) return st;
    hipError_t e = jfa::launch_schedule(offsets, nullptr, (int)B, block_rows, order, tile_start, v.counters, jfa::kNumCounters, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail("schedule kernel", e);
    return JFA_OK;
}

int jfa_check_offsets(const int64_t *offsets, int64_t B, int64_t max_len, void *stream, int *host_flags) {
    if (!host_flags) return fail(JFA_ERR_INVALID_ARG, "jfa_check_offsets: host_flags is null");
    if (B < 0 || B >= (int64_t)1 << 30) return fail(JFA_ERR_INVALID_ARG, "jfa_check_offsets: bad B");
    if (!offsets) return fail(JFA_ERR_INVALID_ARG, "jfa_check_offsets: offsets is null");
    Views v;
    int st = get_table(B, (hipStream_t)stream, &v);
    if (st != JFA_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    int *flag = v.counters + jfa::kNumCounters - 1;
    hipError_t e = hipMemsetAsync(flag, 0, sizeof(int), s);
    if (e != hipSuccess) return hip_fail("hipMemsetAsync", e);
    e = jfa::launch_check_offsets(offsets, (int)B, max_len, flag, s);
    if (e != hipSuccess) return hip_fail("check kernel", e);
    e = hipMemcpyAsync(host_flags, flag, sizeof(int), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail("hipMemcpyAsync", e);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail("hipStreamSynchronize", e);
    return JFA_OK;
}

}  // extern "C"

namespace {
// Forward and backward behind the self- and cross-attention entry points.  offsets_kv == nullptr: self attention
// (keys and values share the queries' offsets).  Work schedules are built over the offsets of the rows a kernel's
// work items are blocks of: the queries' for the forward and dQ, the keys' for dK and dV.
hipError_t schedule(const int64_t *offsets, const int64_t *offsets_other, int64_t B, int block_rows, const Views &w, int which,
                    hipStream_t s) {
    ScopedTimer tm("schedule", s);
    return jfa::launch_schedule(offsets, offsets_other, (int)B, block_rows, w.order[which], w.tile_start[which], w.counters, jfa::kNumCounters, s);
}

// Cross attention with few queries per sample against their keys (target attention: at most kFewqRows queries,
// D = 128, bf16) has one kernel per direction, bound by one pass over K and V.  Their work items are whole
// (sample, head) pairs, claimed longest key list first: only the schedule's sample order is used (sorted by the keys'
// 32-row block count).  Small problems are dealt in sample order without it.
bool few_queries(bool f32, int D, int H, const int64_t *offsets_kv, int64_t max_len_q) {
    return !f32 && D == 128 && (int64_t)H * D <= (1 << 20) && offsets_kv && max_len_q <= jfa::kFewqRows;   // 32-bit row offsets inside a block
}
int few_queries_schedule(const int64_t *offsets, const int64_t *offsets_kv, int64_t B, int H, const Views &w, hipStream_t s,
                         jfa::Schedule *sc) {
    *sc = jfa::Schedule{w.order[0], w.tile_start[0], w.counters};
    if (B * H <= 4 * (int64_t)w.cus) {
        sc->order = nullptr;
        sc->static_only = true;
        return JFA_OK;
    }
    const hipError_t e = schedule(offsets, offsets_kv, B, jfa::kFewqRows, w, 0, s);
    return e == hipSuccess ? JFA_OK : hip_fail("schedule kernel", e);
}

int forward_impl(const char *who, bool f32, bool causal, const void *q, const void *k, const void *v, const int64_t *offsets,
                 const int64_t *offsets_kv, int64_t B, int64_t max_len, int64_t max_len_kv, int H, int D, void *out,
                 float *lse, hipStream_t s, bool static_table = false) {
    const void *ptrs[] = {q, k, v, offsets, out, lse};
    int st = check_common(who, B, max_len, H, D, ptrs, 6);
    if (st != JFA_OK || B == 0) return st;
    if (max_len_kv < 0) return fail(JFA_ERR_INVALID_ARG, "%s: max_len_kv = %lld is negative", who, (long long)max_len_kv);
    Views w;
    if ((st = static_table ? get_static_table(B, &w) : get_table(B, s, &w)) != JFA_OK) return st;
    hipError_t e;
    if (few_queries(f32, D, H, offsets_kv, max_len)) {
        jfa::Schedule sc;
        if ((st = few_queries_schedule(offsets, offsets_kv, B, H, w, s, &sc)) != JFA_OK) return st;
        ScopedTimer tm("fwd_cross_fewq", s);
        e = jfa::launch_fwd_cross_fewq(q, k, v, offsets, offsets_kv, (int)B, H, D, sc, out, lse, w.cus, s);
        return e == hipSuccess ? JFA_OK : hip_fail("fwd_cross_fewq", e);
    }
    const FwdVariant variant = f32 ? kNarrow : forward_variant(max_len > max_len_kv ? max_len : max_len_kv, D, H);
    const int block_rows = f32 ? jfa::kF32BlockRows : (variant == kNarrow ? jfa::kFwdBlockRows : jfa::kDmaBlockRows);
    jfa::Schedule sc{w.order[0], w.tile_start[0], w.counters};
    if (variant == kNarrow && small_problem(B, max_len, H, block_rows, w.cus)) {
        sc.build_rows = block_rows;
        sc.static_only = true;
    } else {
        e = schedule(offsets, offsets_kv, B, block_rows, w, 0, s);
        if (e != hipSuccess) return hip_fail("schedule kernel", e);
    }
    if (f32) { ScopedTimer tm("fwd_f32", s); e = jfa::launch_fwd_f32((const float *)q, (const float *)k, (const float *)v, offsets, offsets_kv, causal, (int)B, H, D, sc, (float *)out, lse, w.cus, s); }
    else if (variant == kDma) { ScopedTimer tm("fwd_bf16_dma", s); e = jfa::launch_fwd_bf16_dma(q, k, v, offsets, offsets_kv, causal, (int)B, H, D, sc, out, lse, w.cus, s); }
    else { ScopedTimer tm("fwd_bf16", s); e = jfa::launch_fwd_bf16(q, k, v, offsets, offsets_kv, causal, (int)B, H, D, sc, out, lse, w.cus, s); }
    if (e != hipSuccess) return hip_fail("forward kernel", e);
    return JFA_OK;
}

int backward_impl(const char *who, bool f32, bool causal, const void *q, const void *k, const void *v, const void *out,
                  const void *dout, const float *lse, const int64_t *offsets, const int64_t *offsets_kv, int64_t B,
                  int64_t max_len, int64_t max_len_kv, int H, int D, void *dq, void *dk, void *dv, float *delta,
                  hipStream_t s) {
    const void *ptrs[] = {q, k, v, out, dout, lse, offsets, dq, dk, dv, delta};
    int st = check_common(who, B, max_len, H, D, ptrs, 11);
    if (st != JFA_OK || B == 0) return st;
    if (max_len_kv < 0) return fail(JFA_ERR_INVALID_ARG, "%s: max_len_kv = %lld is negative", who, (long long)max_len_kv);
    Views w;
    if ((st = get_table(B, s, &w)) != JFA_OK) return st;
    hipError_t e;
    if (few_queries(f32, D, H, offsets_kv, max_len)) {
        jfa::Schedule sc;
        if ((st = few_queries_schedule(offsets, offsets_kv, B, H, w, s, &sc)) != JFA_OK) return st;
        ScopedTimer tm("bwd_cross_fewq", s);
        e = jfa::launch_bwd_cross_fewq(q, k, v, out, dout, lse, delta, offsets, offsets_kv, (int)B, H, D, sc, dq, dk, dv, w.cus, s);
        return e == hipSuccess ? JFA_OK : hip_fail("bwd_cross_fewq", e);
    }
    const bool dma = !f32 && D == 128 && forward_variant(max_len > max_len_kv ? max_len : max_len_kv, D, H) != kNarrow;
    const int block_rows = f32 ? jfa::kF32BlockRows : (dma ? jfa::kDmaBlockRows : jfa::kBwdBlockRows);
    // Schedule 0: blocks of queries.  Schedule 1: blocks of keys, only different from schedule 0 for cross attention.
    // Both launches clear all work counters, and both run before the first kernel that uses one.  Small problems on
    // the register-staged and fp32 kernels have no scheduler launch: those kernels build their schedule themselves.
    const bool in_kernel = !dma && small_problem(B, max_len > max_len_kv ? max_len : max_len_kv, H, block_rows, w.cus);
    if (!in_kernel) {
        e = schedule(offsets, offsets_kv, B, block_rows, w, 0, s);
        if (e == hipSuccess && offsets_kv && !dma) e = schedule(offsets_kv, offsets, B, block_rows, w, 1, s);
        if (e != hipSuccess) return hip_fail("schedule kernel", e);
    }
    const int kv = offsets_kv ? 1 : 0;
    const int64_t *const offsets_k = offsets_kv ? offsets_kv : offsets;   // the keys' offsets
    const int64_t *const offsets_q_other = offsets_kv ? offsets : nullptr;   // the queries', as the second array of dK / dV
    if (f32) {
        jfa::Schedule s_dq{w.order[0], w.tile_start[0], w.counters};
        jfa::Schedule s_dkv{w.order[kv], w.tile_start[kv], w.counters + jfa::kXcds};
        if (in_kernel) {   // every kernel builds the schedule of its own work items, in LDS
            s_dq.static_only = s_dkv.static_only = true;
            s_dq.build_rows = block_rows;
            s_dkv.build_rows = block_rows;
        }
        ScopedTimer tm_bwd("bwd_f32", s);
        e = jfa::launch_bwd_f32((const float *)q, (const float *)k, (const float *)v, (const float *)out, (const float *)dout, lse,
                                offsets, offsets_kv, causal, (int)B, H, D, s_dq, s_dkv, (float *)dq, (float *)dk, (float *)dv, delta, w.cus, s);
        if (e != hipSuccess) return hip_fail("fp32 backward kernels", e);
        return JFA_OK;
    }
    if (dma) {
        // long samples at D = 128: dQ (which also fills both statistics planes) on schedule 0, then dK and dV together on
        // 128-key blocks (schedule 1: blocks of keys, for cross attention from the keys' offsets)
        e = schedule(offsets_k, offsets_q_other, B, jfa::kDkvBlockRows, w, 1, s);
        if (e != hipSuccess) return hip_fail("schedule kernel", e);
        jfa::Schedule s_dq{w.order[0], w.tile_start[0], w.counters};
        jfa::Schedule s_dkv{w.order[1], w.tile_start[1], w.counters + jfa::kXcds};
        { ScopedTimer tm("dq_bf16_dma", s); e = jfa::launch_bwd_dq_dma(q, k, v, out, dout, lse, delta, offsets, offsets_kv, causal, (int)B, H, D, s_dq, dq, w.cus, s); }
        if (e != hipSuccess) return hip_fail("dq_bf16_dma", e);
        { ScopedTimer tm("dkv_bf16_dma", s); e = jfa::launch_bwd_dkv_dma(q, k, v, dout, delta, offsets_k, offsets_q_other, causal, (int)B, H, D, s_dkv, dk, dv, w.cus, s); }
        if (e != hipSuccess) return hip_fail("dkv_bf16_dma", e);
        return JFA_OK;
    }
    jfa::Schedule s_dq{w.order[0], w.tile_start[0], w.counters};
    jfa::Schedule s_dkv{w.order[kv], w.tile_start[kv], w.counters + jfa::kXcds};
    if (in_kernel) {   // every kernel builds the schedule of its own work items, in LDS
        s_dq.static_only = s_dkv.static_only = true;
        s_dq.build_rows = block_rows;
        s_dkv.build_rows = block_rows;
    }
    // the dQ kernel goes first: it computes delta = rowsum(dO o O) for its own rows and leaves it for the dK / dV kernel
    { ScopedTimer tm("dq_bf16", s); e = jfa::launch_dq_bf16(q, k, v, out, dout, lse, delta, offsets, offsets_kv, causal, (int)B, H, D, s_dq, dq, w.cus, s); }
    if (e != hipSuccess) return hip_fail("bf16 dQ kernel", e);
    { ScopedTimer tm("dkv_bf16", s); e = jfa::launch_dkv_bf16(q, k, v, dout, lse, delta, offsets_k, offsets_q_other, causal, (int)B, H, D, s_dkv, dk, dv, w.cus, s); }
    if (e != hipSuccess) return hip_fail("bf16 dK/dV kernel", e);
    return JFA_OK;
}

int need_kv(const char *who, const int64_t *offsets_kv, int64_t B) {
    if (B > 0 && !offsets_kv) return fail(JFA_ERR_INVALID_ARG, "%s: offsets_kv is null", who);
    if (B > 0 && misaligned(offsets_kv)) return fail(JFA_ERR_INVALID_ARG, "%s: offsets_kv is not 16-byte aligned", who);
    return JFA_OK;
}
}  // namespace

extern "C" {

int jfa_forward_f32(const float *q, const float *k, const float *v, const int64_t *offsets, int64_t B,
                    int64_t max_len, int H, int D, float *out, float *lse, void *stream) {
    return forward_impl("jfa_forward_f32", true, false, q, k, v, offsets, nullptr, B, max_len, max_len, H, D, out, lse, (hipStream_t)stream);
}

int jfa_backward_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                     const float *lse, const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, float *dq,
                     float *dk, float *dv, float *delta, void *stream) {
    return backward_impl("jfa_backward_f32", true, false, q, k, v, out, dout, lse, offsets, nullptr, B, max_len, max_len, H, D, dq, dk, dv, delta, (hipStream_t)stream);
}

int jfa_forward(const void *q, const void *k, const void *v, const int64_t *offsets, int64_t B, int64_t max_len,
                int H, int D, void *out, float *lse, void *stream) {
    return forward_impl("jfa_forward", false, false, q, k, v, offsets, nullptr, B, max_len, max_len, H, D, out, lse, (hipStream_t)stream);
}

int jfa_forward_noalloc(const void *q, const void *k, const void *v, const int64_t *offsets, int64_t B, int64_t max_len,
                        int H, int D, void *out, float *lse, void *stream) {
    if (B > JFA_NOALLOC_MAX_B)
        return fail(JFA_ERR_UNSUPPORTED, "jfa_forward_noalloc: B = %lld exceeds JFA_NOALLOC_MAX_B = %d, the batch the fixed work table holds",
                    (long long)B, JFA_NOALLOC_MAX_B);
    g_timing_suppressed = true;
    const int st = forward_impl("jfa_forward_noalloc", false, false, q, k, v, offsets, nullptr, B, max_len, max_len, H, D, out, lse,
                                (hipStream_t)stream, true);
    g_timing_suppressed = false;
    return st;
}

int jfa_backward(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                 const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, void *dq, void *dk, void *dv,
                 float *delta, void *stream) {
    return backward_impl("jfa_backward", false, false, q, k, v, out, dout, lse, offsets, nullptr, B, max_len, max_len, H, D, dq, dk, dv, delta, (hipStream_t)stream);
}

// ---- cross attention: queries and keys of a sample come from two offsets arrays ----

int jfa_forward_cross(const void *q, const void *k, const void *v, const int64_t *offsets_q, const int64_t *offsets_kv,
                      int64_t B, int64_t max_len_q, int64_t max_len_kv, int H, int D, void *out, float *lse, void *stream) {
    int st = need_kv("jfa_forward_cross", offsets_kv, B);
    if (st != JFA_OK) return st;
    return forward_impl("jfa_forward_cross", false, false, q, k, v, offsets_q, offsets_kv, B, max_len_q, max_len_kv, H, D, out, lse, (hipStream_t)stream);
}

int jfa_forward_cross_f32(const float *q, const float *k, const float *v, const int64_t *offsets_q,
                          const int64_t *offsets_kv, int64_t B, int64_t max_len_q, int64_t max_len_kv, int H, int D,
                          float *out, float *lse, void *stream) {
    int st = need_kv("jfa_forward_cross_f32", offsets_kv, B);
    if (st != JFA_OK) return st;
    return forward_impl("jfa_forward_cross_f32", true, false, q, k, v, offsets_q, offsets_kv, B, max_len_q, max_len_kv, H, D, out, lse, (hipStream_t)stream);
}

int jfa_backward_cross(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                       const int64_t *offsets_q, const int64_t *offsets_kv, int64_t B, int64_t max_len_q,
                       int64_t max_len_kv, int H, int D, void *dq, void *dk, void *dv, float *delta, void *stream) {
    int st = need_kv("jfa_backward_cross", offsets_kv, B);
    if (st != JFA_OK) return st;
    return backward_impl("jfa_backward_cross", false, false, q, k, v, out, dout, lse, offsets_q, offsets_kv, B, max_len_q, max_len_kv, H, D, dq, dk, dv, delta, (hipStream_t)stream);
}

int jfa_backward_cross_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                           const float *lse, const int64_t *offsets_q, const int64_t *offsets_kv, int64_t B,
                           int64_t max_len_q, int64_t max_len_kv, int H, int D, float *dq, float *dk, float *dv,
                           float *delta, void *stream) {
    int st = need_kv("jfa_backward_cross_f32", offsets_kv, B);
    if (st != JFA_OK) return st;
    return backward_impl("jfa_backward_cross_f32", true, false, q, k, v, out, dout, lse, offsets_q, offsets_kv, B, max_len_q, max_len_kv, H, D, dq, dk, dv, delta, (hipStream_t)stream);
}

// ---- causal self attention: row i attends to rows 0 .. i of its sample ----

int jfa_forward_causal(const void *q, const void *k, const void *v, const int64_t *offsets, int64_t B, int64_t max_len,
                       int H, int D, void *out, float *lse, void *stream) {
    return forward_impl("jfa_forward_causal", false, true, q, k, v, offsets, nullptr, B, max_len, max_len, H, D, out, lse, (hipStream_t)stream);
}

int jfa_forward_causal_f32(const float *q, const float *k, const float *v, const int64_t *offsets, int64_t B,
                           int64_t max_len, int H, int D, float *out, float *lse, void *stream) {
    return forward_impl("jfa_forward_causal_f32", true, true, q, k, v, offsets, nullptr, B, max_len, max_len, H, D, out, lse, (hipStream_t)stream);
}

int jfa_backward_causal(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                        const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, void *dq, void *dk, void *dv,
                        float *delta, void *stream) {
    return backward_impl("jfa_backward_causal", false, true, q, k, v, out, dout, lse, offsets, nullptr, B, max_len, max_len, H, D, dq, dk, dv, delta, (hipStream_t)stream);
}

int jfa_backward_causal_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                            const float *lse, const int64_t *offsets, int64_t B, int64_t max_len, int H, int D, float *dq,
                            float *dk, float *dv, float *delta, void *stream) {
    return backward_impl("jfa_backward_causal_f32", true, true, q, k, v, out, dout, lse, offsets, nullptr, B, max_len, max_len, H, D, dq, dk, dv, delta, (hipStream_t)stream);
}

// ---- unfused jagged attention (paper Table 1): the baseline of Section 3 ----

int jfa_square_offsets(const int64_t *offsets, int64_t B, int64_t *sq_offsets, void *stream) {
    if (B < 0 || B >= (int64_t)1 << 30) return fail(JFA_ERR_INVALID_ARG, "jfa_square_offsets: bad B");
    if (!offsets || !sq_offsets) return fail(JFA_ERR_INVALID_ARG, "jfa_square_offsets: null pointer");
    hipError_t e = jfa::launch_square_offsets(offsets, (int)B, sq_offsets, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail("square offsets kernel", e);
    return JFA_OK;
}

namespace {
// Common front end of the three operators: validation, work table, schedule (row blocks of 128 queries).
int unfused_begin(const char *who, int64_t B, int64_t max_len, int H, int D, const void *const *ptrs, int n_ptrs,
                  const int64_t *offsets, hipStream_t s, Views *w, jfa::Schedule *sc) {
    int st = check_common(who, B, max_len, H, D, ptrs, n_ptrs);
    if (st != JFA_OK || B == 0) return st;
    if ((st = get_table(B, s, w)) != JFA_OK) return st;
    hipError_t e;
    { ScopedTimer tm("schedule", s); e = jfa::launch_schedule(offsets, nullptr, (int)B, 128, w->order[0], w->tile_start[0], w->counters, jfa::kNumCounters, s); }
    if (e != hipSuccess) return hip_fail("schedule kernel", e);
    *sc = jfa::Schedule{w->order[0], w->tile_start[0], w->counters};
    return JFA_OK;
}
}  // namespace

int jfa_unfused_scores(const void *q, const void *k, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                       int64_t max_len, int H, int D, float *scores, void *stream) {
    const void *ptrs[] = {q, k, offsets, sq_offsets, scores};
    hipStream_t s = (hipStream_t)stream;
    Views w;
    jfa::Schedule sc;
    int st = unfused_begin("jfa_unfused_scores", B, max_len, H, D, ptrs, 5, offsets, s, &w, &sc);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("unfused_scores", s); e = jfa::launch_unfused_scores(q, k, offsets, sq_offsets, (int)B, H, D, sc, 1.0f / sqrtf((float)D), scores, w.cus, s); }
    if (e != hipSuccess) return hip_fail("unfused scores kernel", e);
    return JFA_OK;
}

int jfa_unfused_softmax(const int64_t *offsets, const int64_t *sq_offsets, int64_t B, int64_t max_len, int H,
                        float *scores, void *stream) {
    const void *ptrs[] = {offsets, sq_offsets, scores};
    hipStream_t s = (hipStream_t)stream;
    Views w;
    jfa::Schedule sc;
    int st = unfused_begin("jfa_unfused_softmax", B, max_len, H, 128, ptrs, 3, offsets, s, &w, &sc);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("unfused_softmax", s); e = jfa::launch_unfused_softmax(offsets, sq_offsets, (int)B, H, sc, scores, w.cus, s); }
    if (e != hipSuccess) return hip_fail("unfused softmax kernel", e);
    return JFA_OK;
}

int jfa_unfused_product(const void *a, const void *b, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                        int64_t max_len, int H, int D, float scale, float *out, void *stream) {
    const void *ptrs[] = {a, b, offsets, sq_offsets, out};
    hipStream_t s = (hipStream_t)stream;
    Views w;
    jfa::Schedule sc;
    int st = unfused_begin("jfa_unfused_product", B, max_len, H, D, ptrs, 5, offsets, s, &w, &sc);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("unfused_product", s); e = jfa::launch_unfused_scores(a, b, offsets, sq_offsets, (int)B, H, D, sc, scale, out, w.cus, s); }
    if (e != hipSuccess) return hip_fail("unfused product kernel", e);
    return JFA_OK;
}

int jfa_unfused_softmax_backward(const float *probs, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                                 int64_t max_len, int H, float scale, float *dprobs, void *stream) {
    const void *ptrs[] = {probs, offsets, sq_offsets, dprobs};
    hipStream_t s = (hipStream_t)stream;
    Views w;
    jfa::Schedule sc;
    int st = unfused_begin("jfa_unfused_softmax_backward", B, max_len, H, 128, ptrs, 4, offsets, s, &w, &sc);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("unfused_softmax_bwd", s); e = jfa::launch_unfused_softmax_bwd(probs, offsets, sq_offsets, (int)B, H, sc, scale, dprobs, w.cus, s); }
    if (e != hipSuccess) return hip_fail("unfused softmax backward kernel", e);
    return JFA_OK;
}

int jfa_unfused_apply_transposed(const float *array, const void *x, const int64_t *offsets, const int64_t *sq_offsets,
                                 int64_t B, int64_t max_len, int H, int D, void *out, void *stream) {
    const void *ptrs[] = {array, x, offsets, sq_offsets, out};
    hipStream_t s = (hipStream_t)stream;
    Views w;
    jfa::Schedule sc;
    int st = unfused_begin("jfa_unfused_apply_transposed", B, max_len, H, D, ptrs, 5, offsets, s, &w, &sc);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("unfused_apply_t", s); e = jfa::launch_unfused_apply_t(array, x, offsets, sq_offsets, (int)B, H, D, sc, out, w.cus, s); }
    if (e != hipSuccess) return hip_fail("unfused transposed apply kernel", e);
    return JFA_OK;
}

int jfa_unfused_apply(const float *probs, const void *v, const int64_t *offsets, const int64_t *sq_offsets, int64_t B,
                      int64_t max_len, int H, int D, void *out, void *stream) {
    const void *ptrs[] = {probs, v, offsets, sq_offsets, out};
    hipStream_t s = (hipStream_t)stream;
    Views w;
    jfa::Schedule sc;
    int st = unfused_begin("jfa_unfused_apply", B, max_len, H, D, ptrs, 5, offsets, s, &w, &sc);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("unfused_apply", s); e = jfa::launch_unfused_apply(probs, v, offsets, sq_offsets, (int)B, H, D, sc, out, w.cus, s); }
    if (e != hipSuccess) return hip_fail("unfused apply kernel", e);
    return JFA_OK;
}

// ---- jagged <-> padded-dense conversion (paper Section 2.2) ----

namespace {
int convert(const char *who, bool to_dense, const void *src, void *dst, const int64_t *offsets, int64_t B,
            int64_t max_len, int64_t row_bytes, uint32_t pad, hipStream_t s) {
    if (B < 0 || B >= (int64_t)1 << 30) return fail(JFA_ERR_INVALID_ARG, "%s: bad B = %lld", who, (long long)B);
    if (max_len < 0 || max_len >= (int64_t)1 << 30) return fail(JFA_ERR_INVALID_ARG, "%s: bad max_len = %lld", who, (long long)max_len);
    if (row_bytes <= 0 || row_bytes % 16 != 0 || row_bytes > (int64_t)1 << 24)
        return fail(JFA_ERR_UNSUPPORTED, "%s: row_bytes = %lld must be a positive multiple of 16, at most 2^24", who, (long long)row_bytes);
    if (B == 0 || max_len == 0) return JFA_OK;
    if (!src || !dst || !offsets) return fail(JFA_ERR_INVALID_ARG, "%s: null pointer", who);
    if (misaligned(src) || misaligned(dst)) return fail(JFA_ERR_INVALID_ARG, "%s: tensors must be 16-byte aligned", who);
    Views w;   // only the compute-unit count is used
    int st = get_table(B, s, &w);
    if (st != JFA_OK) return st;
    hipError_t e;
    { ScopedTimer tm(to_dense ? "jagged_to_dense" : "dense_to_jagged", s); e = jfa::launch_convert(to_dense, src, dst, offsets, (int)B, max_len, row_bytes / 16, pad, w.cus, s); }
    if (e != hipSuccess) return hip_fail("conversion kernel", e);
    return JFA_OK;
}
}  // namespace

int jfa_jagged_to_dense(const void *values, const int64_t *offsets, int64_t B, int64_t max_len, int64_t row_bytes,
                        uint32_t pad_pattern, void *dense, void *stream) {
    return convert("jfa_jagged_to_dense", true, values, dense, offsets, B, max_len, row_bytes, pad_pattern, (hipStream_t)stream);
}

int jfa_dense_to_jagged(const void *dense, const int64_t *offsets, int64_t B, int64_t max_len, int64_t row_bytes,
                        void *values, void *stream) {
    return convert("jfa_dense_to_jagged", false, dense, values, offsets, B, max_len, row_bytes, 0, (hipStream_t)stream);
}

// ---- jagged feature operators (paper Table 1) ----

namespace {
bool dim_ok(int d) { return d == 32 || d == 64 || d == 128; }

int feature_begin(const char *who, int64_t B, int64_t max_len, int D, int T, const void *const *ptrs, int n_ptrs,
                  hipStream_t s, Views *w) {
    if (!dim_ok(T)) return fail(JFA_ERR_UNSUPPORTED, "%s: T = %d is not one of 32, 64, 128", who, T);
    int st = check_common(who, B, max_len, 1, D, ptrs, n_ptrs);
    if (st != JFA_OK || B == 0) return st;
    return get_table(B, s, w);   // for the work counter and the compute-unit count
}
}  // namespace

int jfa_jagged_dense_bmm(const void *x, const void *w, const int64_t *offsets, int64_t B, int64_t max_len, int D, int T,
                         void *out, void *stream) {
    const void *ptrs[] = {x, w, offsets, out};
    hipStream_t s = (hipStream_t)stream;
    Views v;
    int st = feature_begin("jfa_jagged_dense_bmm", B, max_len, D, T, ptrs, 4, s, &v);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("jagged_dense_bmm", s); e = jfa::launch_jagged_dense_bmm(x, w, offsets, (int)B, D, T, v.counters, out, v.cus, s); }
    if (e != hipSuccess) return hip_fail("jagged_dense_bmm kernel", e);
    return JFA_OK;
}

int jfa_jagged_jagged_bmm(const void *x, const void *y, const int64_t *offsets, int64_t B, int64_t max_len, int D, int T,
                          void *out, void *stream) {
    const void *ptrs[] = {x, y, offsets, out};
    hipStream_t s = (hipStream_t)stream;
    Views v;
    int st = feature_begin("jfa_jagged_jagged_bmm", B, max_len, D, T, ptrs, 4, s, &v);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("jagged_jagged_bmm", s); e = jfa::launch_jagged_jagged_bmm(x, y, offsets, (int)B, D, T, v.counters, out, v.cus, s); }
    if (e != hipSuccess) return hip_fail("jagged_jagged_bmm kernel", e);
    return JFA_OK;
}

int jfa_jagged_softmax(const void *x, const int64_t *offsets, int64_t B, int64_t max_len, int D, void *y, void *stream) {
    const void *ptrs[] = {x, offsets, y};
    hipStream_t s = (hipStream_t)stream;
    Views v;
    int st = feature_begin("jfa_jagged_softmax", B, max_len, D, 32, ptrs, 3, s, &v);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("jagged_softmax", s); e = jfa::launch_jagged_softmax(false, x, nullptr, offsets, (int)B, D, v.counters, y, v.cus, s); }
    if (e != hipSuccess) return hip_fail("jagged_softmax kernel", e);
    return JFA_OK;
}

int jfa_jagged_softmax_backward(const void *y, const void *dy, const int64_t *offsets, int64_t B, int64_t max_len, int D,
                                void *dx, void *stream) {
    const void *ptrs[] = {y, dy, offsets, dx};
    hipStream_t s = (hipStream_t)stream;
    Views v;
    int st = feature_begin("jfa_jagged_softmax_backward", B, max_len, D, 32, ptrs, 4, s, &v);
    if (st != JFA_OK || B == 0) return st;
    hipError_t e;
    { ScopedTimer tm("jagged_softmax_bwd", s); e = jfa::launch_jagged_softmax(true, y, dy, offsets, (int)B, D, v.counters, dx, v.cus, s); }
    if (e != hipSuccess) return hip_fail("jagged_softmax backward kernel", e);
    return JFA_OK;
}

}  // extern "C"

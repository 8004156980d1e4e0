// Internal declarations shared by the HIP translation units of libjfa.so (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace jfa {

// Number of int32 work counters at the head of the private work table.
constexpr int kNumCounters = 64;
// Histogram bins of the scheduler's counting sort (samples with >= kSchedBins-1 row blocks share the top bin).
constexpr int kSchedBins = 1024;

// Device view of one work schedule (see jfa_build_schedule in jfa.h for the meaning of the arrays).
struct Schedule {
    const int32_t *order;       // [B]
    const int32_t *tile_start;  // [B+1]
    int32_t *counter;           // kXcds zeroed work counters (one queue per XCD), bumped by the persistent workgroups
    // Small problems (see build_small_work) run without a scheduler launch: the counters are then not valid
    // and work is dealt statically (static_only); build_rows > 0 tells the kernel to build the schedule itself, in LDS, for
    // row blocks of that many rows (order and tile_start are then not looked at), 0 that the scheduler kernel has filled them.
    int build_rows = 0;
    bool static_only = false;
};

// The chip has 8 accelerator dies (XCDs), each with its own L2, and workgroups are dealt to them round-robin
// by workgroup id.  Work ids are cut into groups of kWorkGroup consecutive ids -- consecutive ids are row
// blocks of the same (sample, head), which stream the same K/V -- and group g belongs to the queue of XCD
// g % 8, so the blocks that share K/V run on the die whose L2 already holds it.  A workgroup drains its own
// die's queue first and then helps the others, so the assumption about placement only affects locality.
constexpr int kXcds = 8;
constexpr int kWorkGroup = 32;

// Work id of local index t of queue y.
__device__ inline int64_t work_id(int y, int t) {
    return ((int64_t)(t / kWorkGroup) * kXcds + y) * kWorkGroup + t % kWorkGroup;
}

// Per-workgroup claim state (kept by the one thread that claims).
struct WorkCursor {
    bool first = true;
    bool home_done = false;
    bool static_only = false;   // the counters are not valid (schedule built in the kernel): deal statically whatever the size
    int64_t next = -1;   // small problems: next statically assigned id
    int grid = 0;        // gridDim.x, read once: the dispatch packet it comes from is a slow place to read
};

__device__ inline int cursor_grid(WorkCursor &cur) {
    if (cur.grid == 0) {
        int g = (int)gridDim.x;
        asm volatile("" : "+v"(g));   // a value, not a load the compiler may repeat wherever it is needed
        cur.grid = g;
    }
    return cur.grid;
}

// Next work id for this workgroup, or -1 when nothing is left.  Called by one thread.
//   * The first item is assigned statically (queue blockIdx % 8, local index blockIdx / 8): no memory traffic,
//     and on problems smaller than the grid the surplus workgroups leave at once.
//   * Further items of the home queue are claimed with one atomic add (local indices continue after the
//     static ones, hence the gridDim / 8 base; the grid is a multiple of 8).
//   * Once the home queue is empty the workgroup looks at all eight counters with plain loads and only
//     spends an atomic on a queue that still shows work.
//   * Problems of at most four items per workgroup skip all of this (see below).
__device__ inline int64_t next_work(int32_t *counters, WorkCursor &cur, int64_t total) {
    // Small problems (at most four items per workgroup) are dealt round-robin with no atomics at all: the
    // items are sorted longest-first, so the deal is even, and the claim traffic would dominate the run time.
    const int grid = cursor_grid(cur);
    if (cur.static_only || total <= 4 * (int64_t)grid) {
        cur.next = cur.next < 0 ? blockIdx.x : cur.next + grid;
        return cur.next < total ? cur.next : -1;
    }
    const int home = blockIdx.x % kXcds;
    const int base = grid / kXcds;
    if (cur.first) {
        cur.first = false;
        const int64_t id = work_id(home, blockIdx.x / kXcds);
        if (id < total) return id;
        cur.home_done = true;  // ids grow with the local index: nothing later in this queue is valid either
    }
    if (!cur.home_done) {
        const int64_t id = work_id(home, base + atomicAdd(&counters[home], 1));
        if (id < total) return id;
        cur.home_done = true;
    }
    for (;;) {
        int seen[kXcds];  // all eight counters in one round of independent loads
#pragma unroll
        for (int y = 0; y < kXcds; ++y) seen[y] = __atomic_load_n(&counters[y], __ATOMIC_RELAXED);
        bool any = false;
#pragma unroll
        for (int d = 1; d < kXcds; ++d) {
            const int y = (home + d) % kXcds;
            int c = 0;
#pragma unroll
            for (int z = 0; z < kXcds; ++z) c = z == y ? seen[z] : c;
            if (work_id(y, base + c) >= total) continue;
            any = true;
            const int64_t id = work_id(y, base + atomicAdd(&counters[y], 1));
            if (id < total) return id;
        }
        if (!any) return -1;  // counters only grow, so this loop ends
    }
}

// The work id is the same for every lane; saying so lets the tile parameters derived from it live in scalar
// registers and be fetched with scalar loads.
__device__ inline int64_t uniform64(int64_t x) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)x >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Next work id for the whole workgroup (thread 0 claims, `slot` in LDS hands it to the others), or -1.
__device__ inline int64_t fetch_item(int32_t *counters, WorkCursor &cur, int64_t total, int64_t *slot) {
    __syncthreads();
    if (threadIdx.x == 0) *slot = next_work(counters, cur, total);
    __syncthreads();
    return uniform64(*slot);
}

// One decoded work item.
struct Work {
    int sample;   // sample id b
    int head;     // head h
    int block;    // row-block index inside the sample
    int64_t row0; // offsets[b]
    int len;      // L_b
    // Cross attention: the sample's rows on the other side (the rows that stream past the block: keys for a
    // block of queries, queries for a block of keys), from a second offsets array.  Equal to row0 / len otherwise.
    int64_t orow0;
    int olen;
};

// Largest p in [0, B) with tile_start[p] * H <= w, found by one wave: 64 probes per round instead of one.
__device__ inline int find_position_wave(const int32_t *tile_start, int B, int H, int64_t w) {
    const int lane = threadIdx.x & 63;
    int lo = 0, hi = B;  // invariant: tile_start[lo]*H <= w < tile_start[hi]*H
    while (hi - lo > 1) {
        const int step = (hi - lo + 63) / 64;
        const int idx = lo + (lane + 1) * step;
        const bool ok = idx < hi && (int64_t)tile_start[idx] * H <= w;   // true for a prefix of the lanes
        const int cnt = __popcll(__builtin_amdgcn_ballot_w64(ok));
        lo += cnt * step;
        hi = hi < lo + step ? hi : lo + step;
    }
    return lo;
}

// Work item w -> (sample, head, row block).  Called by whole waves (each wave searches for itself, 64 probes per
// round: two or three dependent loads instead of log2(B)).
__device__ inline Work decode_work(const Schedule &s, const int64_t *offsets, int B, int H, int64_t w,
                                   const int64_t *offsets_other = nullptr) {
    Work t;
    const int p = find_position_wave(s.tile_start, B, H, w);   // every lane of the calling wave must be active
    const int t0 = s.tile_start[p];
    const int n = s.tile_start[p + 1] - t0;
    const int r = (int)(w - (int64_t)t0 * H);
    t.sample = s.order[p];
    t.head = r / n;
    t.block = r - t.head * n;
    t.row0 = offsets[t.sample];
    t.len = (int)(offsets[t.sample + 1] - t.row0);
    t.orow0 = t.row0;
    t.olen = t.len;
    if (offsets_other) {
        t.orow0 = offsets_other[t.sample];
        t.olen = (int)(offsets_other[t.sample + 1] - t.orow0);
    }
    return t;
}

// A decoded work item parked in LDS for the whole workgroup.
struct WorkSlot {
    int valid;   // 0: nothing left
    int sample, head, block, len;
    int row0_lo, row0_hi;
    int olen, orow0_lo, orow0_hi;   // the other side's rows (cross attention only)
};

// The schedule of a small problem, built inside the attention kernel instead of by a launch of its own (a launch and
// the scheduler kernel's chain of dependent trips to memory cost more than these problems' whole arithmetic), and
// kept in LDS: every workgroup computes the same schedule -- samples in descending order of their stream's block
// count, equal counts in sample order, the order the scheduler kernel produces (samples in their own order when there
// is at most one item per workgroup) -- and decodes from it the at most
// kSmallItems work items that the static deal gives it (item blockIdx + n * gridDim), so that nothing of the
// schedule is written to or read back from memory: after the one trip for the lengths, an item costs one more for
// its sample's offsets.  Lengths are fetched once, by all threads at once, into LDS; one wave then runs a counting
// sort over at most kInlineBins keys, in which the ranks inside a bin come from ballots, a scan of the block counts
// in sorted order, and the search for the workgroup's items.
// `scratch`: kInlineScratchInts ints of LDS that nothing else uses until the call returns (the kernels lend a stage
// buffer); `mine` is LDS that lasts.  Called by every thread of the workgroup; B <= kInlineCap; ends with a barrier.
constexpr int kInlineCap = 1024;
constexpr int kInlineBins = 64;
constexpr int kSmallItems = 4;
constexpr int kInlineScratchInts = 2 * kInlineBins + kInlineCap + kInlineCap / 4 + kInlineCap / 2 + kInlineCap + 4;   // 11.6 KB
struct SmallWork {
    int count;                     // items of this workgroup
    WorkSlot item[kSmallItems];
};
__device__ inline void build_small_work(const int64_t *offsets, const int64_t *offsets_other, int B, int H, int block_rows,
                                        int *scratch, SmallWork *mine) {
    int *const bins = scratch;                                    // [kInlineBins] counts, then [kInlineBins] next free positions
    int *const nblk = scratch + 2 * kInlineBins;                  // [kInlineCap] row blocks of sample b
    uint8_t *const keys = reinterpret_cast<uint8_t *>(nblk + kInlineCap);               // [kInlineCap] sort key of sample b
    uint16_t *const sorted = reinterpret_cast<uint16_t *>(nblk + kInlineCap + kInlineCap / 4);   // [kInlineCap] sample at position p
    int *const start = nblk + kInlineCap + kInlineCap / 4 + kInlineCap / 2;             // [kInlineCap + 1] first tile of position p
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int64_t len = offsets[b + 1] - offsets[b];
        const int64_t stream = offsets_other ? offsets_other[b + 1] - offsets_other[b] : len;
        const int64_t key = (stream + block_rows - 1) / block_rows;
        nblk[b] = (int)((len + block_rows - 1) / block_rows);
        keys[b] = (uint8_t)(key < kInlineBins - 1 ? key : kInlineBins - 1);
    }
    if (threadIdx.x < 2 * kInlineBins) bins[threadIdx.x] = 0;
    __syncthreads();
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        // inclusive scan of the block counts, samples taken in the order `at(p)`, into start[1 .. B]; returns the total
        auto scan_blocks = [&](auto at) {
            int carry = 0;
            if (lane == 0) start[0] = 0;
            for (int p0 = 0; p0 < B; p0 += 64) {
                const int p = p0 + lane;
                int incl = p < B ? nblk[at(p)] : 0;
                for (int d = 1; d < 64; d <<= 1) {
                    const int y = __shfl_up(incl, d, 64);
                    if (lane >= d) incl += y;
                }
                incl += carry;
                if (p < B) start[p + 1] = incl;
                carry = __shfl(incl, 63, 64);
            }
            return carry;
        };
        // 0. With at most one item per workgroup the order of the deal is of no consequence: the samples stay in their
        //    own order and the sort (steps 1 to 3, most of this function's time) is skipped.
        int blocks = scan_blocks([](int p) { return p; });
        const bool in_sample_order = (int64_t)blocks * H <= (int64_t)gridDim.x;
        if (!in_sample_order) {
        // 1. samples per key
        for (int b0 = 0; b0 < B; b0 += 64) {
            const bool valid = b0 + lane < B;
            const int key = valid ? keys[b0 + lane] : -1;
            uint64_t todo = __builtin_amdgcn_ballot_w64(valid);
            while (todo) {
                const int leader = __builtin_amdgcn_readfirstlane(__builtin_ctzll(todo));
                const int kk = __builtin_amdgcn_readlane(key, leader);
                const uint64_t same = __builtin_amdgcn_ballot_w64(key == kk);
                if (lane == leader) bins[kk] += __popcll(same);
                todo &= ~same;
            }
        }
        // 2. first position of each key, keys in descending order: lane l owns key kInlineBins - 1 - l
        {
            const int cnt = bins[kInlineBins - 1 - lane];
            int incl = cnt;
            for (int d = 1; d < 64; d <<= 1) {
                const int y = __shfl_up(incl, d, 64);
                if (lane >= d) incl += y;
            }
            bins[kInlineBins + (kInlineBins - 1 - lane)] = incl - cnt;
        }
        // 3. scatter in sample order
        for (int b0 = 0; b0 < B; b0 += 64) {
            const bool valid = b0 + lane < B;
            const int b = valid ? b0 + lane : 0;
            const int key = valid ? keys[b] : -1;
            uint64_t todo = __builtin_amdgcn_ballot_w64(valid);
            while (todo) {
                const int leader = __builtin_amdgcn_readfirstlane(__builtin_ctzll(todo));
                const int kk = __builtin_amdgcn_readlane(key, leader);
                const uint64_t same = __builtin_amdgcn_ballot_w64(key == kk);
                const int base = bins[kInlineBins + kk];
                if (key == kk) sorted[base + __popcll(same & ((1ull << lane) - 1))] = (uint16_t)b;
                if (lane == leader) bins[kInlineBins + kk] = base + __popcll(same);
                todo &= ~same;
            }
        }
        // 4. inclusive scan of the block counts in sorted order
        blocks = scan_blocks([&](int p) { return (int)sorted[p]; });
        }
        // 5. this workgroup's items: the position of each in the sorted order (64 probes per round), then, a lane per
        //    item, the sample's offsets -- the only trip to memory, all items at once
        const int64_t total = (int64_t)blocks * H;
        int my_p = 0, my_r = 0, n_items = 0;
        for (int n = 0; n < kSmallItems; ++n) {
            const int64_t w = (int64_t)blockIdx.x + (int64_t)n * gridDim.x;
            if (w >= total) break;
            int lo = 0, hi = B;   // invariant: start[lo] * H <= w < start[hi] * H
            while (hi - lo > 1) {
                const int step = (hi - lo + 63) / 64;
                const int idx = lo + (lane + 1) * step;
                const bool ok = idx < hi && (int64_t)start[idx] * H <= w;   // true for a prefix of the lanes
                const int cnt = __popcll(__builtin_amdgcn_ballot_w64(ok));
                lo += cnt * step;
                hi = hi < lo + step ? hi : lo + step;
            }
            if (lane == n) {
                my_p = lo;
                my_r = (int)(w - (int64_t)start[lo] * H);
            }
            n_items = n + 1;
        }
        if (lane == 0) mine->count = n_items;
        if (lane < n_items) {
            const int sample = in_sample_order ? my_p : (int)sorted[my_p];
            const int per_head = start[my_p + 1] - start[my_p];
            const int64_t row0 = offsets[sample];
            WorkSlot *slot = &mine->item[lane];
            slot->valid = 1;
            slot->sample = sample;
            slot->head = my_r / per_head;
            slot->block = my_r - (my_r / per_head) * per_head;
            slot->len = (int)(offsets[sample + 1] - row0);
            slot->row0_lo = (int)(uint32_t)row0;
            slot->row0_hi = (int)(uint32_t)((uint64_t)row0 >> 32);
            const int64_t *const oo = offsets_other ? offsets_other : offsets;   // the other side's rows: the same without a second array
            const int64_t orow0 = oo[sample];
            slot->olen = (int)(oo[sample + 1] - orow0);
            slot->orow0_lo = (int)(uint32_t)orow0;
            slot->orow0_hi = (int)(uint32_t)((uint64_t)orow0 >> 32);
        }
    }
    __syncthreads();
}

// Persistent-grid size for `kernel`: every compute unit filled to the kernel's occupancy, no more
// (extra workgroups would only find the work counter exhausted).  Queried once per kernel.
template <auto Kernel>
inline int persistent_grid(int threads, int cus) {
    static int per_cu = 0;  // one instance per kernel function
    if (per_cu == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, Kernel, threads, 0) != hipSuccess || n < 1) n = 1;
        per_cu = n;
    }
    const int grid = cus * per_cu;
    return (grid + kXcds - 1) / kXcds * kXcds;  // next_work() relies on a multiple of 8
}


// Claim the next work item and decode it into `slot`.  Called by every lane of ONE wave (the claim itself is
// made by its lane 0, whose registers hold `cur`); meant to be issued right after a tile's first loads so
// that its latency chain (atomic, search, offsets) overlaps with theirs.
__device__ inline void claim_and_decode(WorkSlot *slot, const Schedule &s, const int64_t *offsets, int B, int H,
                                        int64_t total, WorkCursor &cur, const int64_t *offsets_other = nullptr) {
    const int lane = threadIdx.x & 63;
    int64_t w = -1;
    if (lane == 0) w = next_work(s.counter, cur, total);
    w = uniform64(w);
    if (w < 0) {
        if (lane == 0) slot->valid = 0;
        return;
    }
    const int p = find_position_wave(s.tile_start, B, H, w);
    const int t0 = s.tile_start[p];
    const int n = s.tile_start[p + 1] - t0;
    const int r = (int)(w - (int64_t)t0 * H);
    const int sample = s.order[p];
    const int64_t row0 = offsets[sample];
    const int len = (int)(offsets[sample + 1] - row0);
    if (offsets_other) {
        const int64_t orow0 = offsets_other[sample];
        const int olen = (int)(offsets_other[sample + 1] - orow0);
        if (lane == 0) {
            slot->olen = olen;
            slot->orow0_lo = (int)(uint32_t)orow0;
            slot->orow0_hi = (int)(uint32_t)((uint64_t)orow0 >> 32);
        }
    }
    if (lane == 0) {
        slot->valid = 1;
        slot->sample = sample;
        slot->head = r / n;
        slot->block = r - (r / n) * n;
        slot->len = len;
        slot->row0_lo = (int)(uint32_t)row0;
        slot->row0_hi = (int)(uint32_t)((uint64_t)row0 >> 32);
    }
}

// A workgroup's LDS copy of a schedule of at most kTabCap samples (position p of the sorted order: first tile,
// sample, rows): decoding a claimed work id then costs a few LDS reads instead of a chain of dependent global loads.
// Declare it __shared__; CROSS adds the other side's rows.
constexpr int kTabCap = 1024;
template <bool CROSS>
struct LdsSchedule {
    int32_t start[kTabCap + 1];
    int32_t sample[kTabCap], len[kTabCap], row0[kTabCap][2];
    int32_t olen[CROSS ? kTabCap : 1], orow0[CROSS ? kTabCap : 1][2];

    // Called by every thread of the workgroup, B <= kTabCap; a barrier must follow before decode().
    __device__ void fill(const Schedule &s, const int64_t *offsets, const int64_t *offsets_other, int B) {
        for (int p = threadIdx.x; p <= B; p += blockDim.x) start[p] = s.tile_start[p];
        for (int p = threadIdx.x; p < B; p += blockDim.x) {
            const int b = s.order[p];
            const int64_t r0 = offsets[b];
            sample[p] = b;
            len[p] = (int)(offsets[b + 1] - r0);
            row0[p][0] = (int)(uint32_t)r0;
            row0[p][1] = (int)(uint32_t)((uint64_t)r0 >> 32);
            if (CROSS) {
                const int64_t o0 = offsets_other[b];
                olen[p] = (int)(offsets_other[b + 1] - o0);
                orow0[p][0] = (int)(uint32_t)o0;
                orow0[p][1] = (int)(uint32_t)((uint64_t)o0 >> 32);
            }
        }
    }

    // Work id w (the same in every lane; < 0: nothing left) -> slot.  Called by every lane of one wave.
    __device__ void decode(WorkSlot *slot, int B, int H, int64_t w) const {
        const int lane = threadIdx.x & 63;
        if (w < 0) {
            if (lane == 0) slot->valid = 0;
            return;
        }
        int lo = 0, hi = B;   // invariant: start[lo] * H <= w < start[hi] * H
        while (hi - lo > 1) {
            const int step = (hi - lo + 63) / 64;
            const int idx = lo + (lane + 1) * step;
            const bool ok = idx < hi && (int64_t)start[idx] * H <= w;   // true for a prefix of the lanes
            const int cnt = __popcll(__builtin_amdgcn_ballot_w64(ok));
            lo += cnt * step;
            hi = hi < lo + step ? hi : lo + step;
        }
        if (lane == 0) {
            const int t0 = start[lo];
            const int n = start[lo + 1] - t0;
            const int r = (int)(w - (int64_t)t0 * H);
            slot->valid = 1;
            slot->sample = sample[lo];
            slot->head = r / n;
            slot->block = r - (r / n) * n;
            slot->len = len[lo];
            slot->row0_lo = row0[lo][0];
            slot->row0_hi = row0[lo][1];
            if (CROSS) {
                slot->olen = olen[lo];
                slot->orow0_lo = orow0[lo][0];
                slot->orow0_hi = orow0[lo][1];
            }
        }
    }
};

// Read the parked work item into scalar registers; returns false when nothing is left.  CROSS: the slot also holds
// the other side's rows.
template <bool CROSS = false>
__device__ inline bool load_work(const WorkSlot *slot, Work &t) {
    if (__builtin_amdgcn_readfirstlane(slot->valid) == 0) return false;
    t.sample = __builtin_amdgcn_readfirstlane(slot->sample);
    t.head = __builtin_amdgcn_readfirstlane(slot->head);
    t.block = __builtin_amdgcn_readfirstlane(slot->block);
    t.len = __builtin_amdgcn_readfirstlane(slot->len);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane(slot->row0_lo);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane(slot->row0_hi);
    t.row0 = (int64_t)(((uint64_t)hi << 32) | lo);
    t.orow0 = t.row0;
    t.olen = t.len;
    if (CROSS) {
        t.olen = __builtin_amdgcn_readfirstlane(slot->olen);
        const uint32_t olo = (uint32_t)__builtin_amdgcn_readfirstlane(slot->orow0_lo);
        const uint32_t ohi = (uint32_t)__builtin_amdgcn_readfirstlane(slot->orow0_hi);
        t.orow0 = (int64_t)(((uint64_t)ohi << 32) | olo);
    }
    return true;
}

// ---- launchers (each enqueues on `stream` and returns the launch status; `cus` = compute units of the device) ----

// Scheduler: fills order / tile_start for the given row-block size and zeroes `n_counters` counters.  Blocks are
// counted over `offsets`; samples are ordered by the length of the rows that stream past a block (offsets_other:
// cross attention; nullptr: the sample's own length).
hipError_t launch_schedule(const int64_t *offsets, const int64_t *offsets_other, int B, int block_rows, int32_t *order,
                           int32_t *tile_start, int32_t *counters, int n_counters, hipStream_t stream);
hipError_t launch_check_offsets(const int64_t *offsets, int B, int64_t max_len, int *flags, hipStream_t stream);

// fp32 path
constexpr int kF32BlockRows = 64;
// Cross attention: offsets = the queries' offsets, offsets_kv = the keys' (nullptr: the same array); schedules are
// built over the stationary side's offsets (s, s_dq: queries; s_dkv: keys).
// causal (self attention only, offsets_kv == nullptr): row i attends to rows 0 .. i of its sample.
hipError_t launch_fwd_f32(const float *q, const float *k, const float *v, const int64_t *offsets,
                          const int64_t *offsets_kv, bool causal, int B, int H, int D, Schedule s, float *out, float *lse,
                          int cus, hipStream_t stream);
hipError_t launch_bwd_f32(const float *q, const float *k, const float *v, const float *out, const float *dout,
                          const float *lse, const int64_t *offsets, const int64_t *offsets_kv, bool causal, int B, int H,
                          int D, Schedule s_dq, Schedule s_dkv, float *dq, float *dk, float *dv, float *delta, int cus,
                          hipStream_t stream);
// (the dQ kernel of every path runs first and computes delta[h, row] = sum_d dout * out for the kernels after it)

// bf16 attention, register-staged kernels (any supported D, short samples)
constexpr int kFwdBlockRows = 128;
constexpr int kBwdBlockRows = 128;
// In all bf16 launchers `offsets` belongs to the rows the schedule `s` was built over (queries for the forward and
// dQ, keys for dK / dV) and the second array to the rows that stream past them (cross attention; nullptr: the same).
// causal: self attention in which row i attends to rows 0 .. i of its sample (not together with a second array).
hipError_t launch_fwd_bf16(const void *q, const void *k, const void *v, const int64_t *offsets,
                           const int64_t *offsets_kv, bool causal, int B, int H, int D, Schedule s, void *out, float *lse,
                           int cus, hipStream_t stream);
hipError_t launch_dkv_bf16(const void *q, const void *k, const void *v, const void *dout, const float *lse,
                           const float *delta, const int64_t *offsets, const int64_t *offsets_q, bool causal, int B, int H,
                           int D, Schedule s, void *dk, void *dv, int cus, hipStream_t stream);
// out != nullptr: the kernel computes delta = rowsum(dO o O) itself and stores it in `delta` (launch it before the
// dK / dV kernel); out == nullptr: `delta` has been filled before.
hipError_t launch_dq_bf16(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                          float *delta, const int64_t *offsets, const int64_t *offsets_kv, bool causal, int B, int H,
                          int D, Schedule s, void *dq, int cus, hipStream_t stream);

// bf16 attention, direct-to-LDS kernels (D = 128, long samples; work items are blocks of kDmaBlockRows rows)
constexpr int kDmaBlockRows = 256;
hipError_t launch_fwd_bf16_dma(const void *q, const void *k, const void *v, const int64_t *offsets,
                               const int64_t *offsets_kv, bool causal, int B, int H, int D, Schedule s, void *out, float *lse,
                               int cus, hipStream_t stream);
// The dQ launch has to come first: with `out` given (the forward's output) it computes delta = rowsum(dout o out) and
// -lse * sqrt(D) itself and leaves them in `delta` [2, H, sum_B] for the dK / dV kernel.
hipError_t launch_bwd_dq_dma(const void *q, const void *k, const void *v, const void *out, const void *dout, const float *lse,
                             float *delta, const int64_t *offsets, const int64_t *offsets_other, bool causal, int B, int H,
                             int D, Schedule s, void *dq, int cus, hipStream_t stream);

// dK and dV of self attention in one kernel (pairs of waves share 32 keys; work items are blocks of kDkvBlockRows keys);
// `stats` is the [2, H, sum_B] buffer the dQ launch has filled.
constexpr int kDkvBlockRows = 128;
// Cross attention with at most 32 queries per sample, D = 128: a forward kernel bound by reading K and V once, and the
// whole backward (statistics, dQ, dK, dV) in one kernel and one pass over K and V.  `sched`: only `order` (the samples by their number of 32-key blocks, longest
// first; nullptr = sample order), `counter` and `static_only` are used; a work item is a whole (sample, head).
constexpr int kFewqRows = 32;
hipError_t launch_fwd_cross_fewq(const void *q, const void *k, const void *v, const int64_t *offsets_q,
                                 const int64_t *offsets_kv, int B, int H, int D, Schedule sched, void *out, float *lse, int cus,
                                 hipStream_t stream);
hipError_t launch_bwd_cross_fewq(const void *q, const void *k, const void *v, const void *out, const void *dout,
                                 const float *lse, float *stats, const int64_t *offsets_q, const int64_t *offsets_kv, int B,
                                 int H, int D, Schedule sched, void *dq, void *dk, void *dv, int cus, hipStream_t stream);
hipError_t launch_bwd_dkv_dma(const void *q, const void *k, const void *v, const void *dout, const float *stats,
                              const int64_t *offsets, const int64_t *offsets_other, bool causal, int B, int H, int D, Schedule s, void *dk,
                              void *dv, int cus,
                              hipStream_t stream);

// Unfused jagged attention (Table 1): offsets of the jagged square array, then the three operators.
hipError_t launch_square_offsets(const int64_t *offsets, int B, int64_t *sq, hipStream_t stream);
hipError_t launch_unfused_scores(const void *q, const void *k, const int64_t *offsets, const int64_t *sq, int B, int H,
                                 int D, Schedule s, float scale, float *scores, int cus, hipStream_t stream);
hipError_t launch_unfused_softmax_bwd(const float *probs, const int64_t *offsets, const int64_t *sq, int B, int H,
                                      Schedule s, float scale, float *dprobs, int cus, hipStream_t stream);
hipError_t launch_unfused_apply_t(const float *X, const void *x, const int64_t *offsets, const int64_t *sq, int B, int H,
                                  int D, Schedule s, void *out, int cus, hipStream_t stream);
hipError_t launch_unfused_softmax(const int64_t *offsets, const int64_t *sq, int B, int H, Schedule s, float *scores,
                                  int cus, hipStream_t stream);
hipError_t launch_unfused_apply(const float *probs, const void *v, const int64_t *offsets, const int64_t *sq, int B,
                                int H, int D, Schedule s, void *out, int cus, hipStream_t stream);

// Jagged <-> padded-dense conversion (Section 2.2); rows are row_chunks 16-byte chunks long.
hipError_t launch_convert(bool to_dense, const void *src, void *dst, const int64_t *offsets, int B, int64_t max_len,
                          int64_t row_chunks, uint32_t pad, int cus, hipStream_t stream);

// Jagged feature operators (Table 1); `counter` is one work counter, reset by the launcher.
hipError_t launch_jagged_dense_bmm(const void *x, const void *w, const int64_t *offsets, int B, int D, int T,
                                   int32_t *counter, void *out, int cus, hipStream_t stream);
hipError_t launch_jagged_jagged_bmm(const void *x, const void *y, const int64_t *offsets, int B, int D, int T,
                                    int32_t *counter, void *out, int cus, hipStream_t stream);
hipError_t launch_jagged_softmax(bool backward, const void *a, const void *b, const int64_t *offsets, int B, int D,
                                 int32_t *counter, void *out, int cus, hipStream_t stream);

}  // namespace jfa

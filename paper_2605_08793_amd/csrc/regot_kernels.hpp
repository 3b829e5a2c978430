// Streaming kernels over the cost matrix M (gfx950).
//
// Work decomposition (all stage-1 kernels): the n x m matrix is cut into column
// panels of kPanel = 512 columns and g_r row chunks of (almost) equal height.  One
// workgroup (4 waves) owns one (row chunk, panel) pair for its whole life, and the
// grid is sized so that every workgroup is resident at once: all of them stream at
// the same time and finish together.  Inside a panel a lane owns 8 fixed columns
// (4 x 16-byte loads per row, lanes adjacent in memory), so column reductions stay
// in the lane's registers for all rows of the chunk and only row reductions cross
// lanes.  Waves take groups of kRB = 4 rows round-robin.  Each matrix entry is read
// once and nothing is accumulated with floating-point atomics: partial results go
// to a workspace and a small second kernel combines them in a fixed order.
//
// This replaces the tiling of the paper's fused gradient kernel (Sec. 4.4: 32 x D
// thread blocks, one column per thread, shuffle tree per 32-column segment, shared-
// memory atomics for the column sums): the same single-read fusion, re-cut for
// 64-wide waves and 128-bit loads.
#pragma once

#include <type_traits>

#include "regot_device.hpp"

namespace regot {

// resident waves per SIMD the stage-1 kernels are compiled for (register budget 512 / N); a
// workgroup is one wave per SIMD, so this is also the number of resident workgroups per CU
#ifndef REGOT_PLAN_WAVES_PER_EU
#define REGOT_PLAN_WAVES_PER_EU 2
#endif
#ifndef REGOT_ROWLSE_WAVES_PER_EU
#define REGOT_ROWLSE_WAVES_PER_EU 2
#endif
#ifndef REGOT_COLLSE_WAVES_PER_EU
#define REGOT_COLLSE_WAVES_PER_EU 2
#endif
#define REGOT_WAVES_ATTR(N) __attribute__((amdgpu_waves_per_eu(N, N)))

// ints at the start of the workspace
enum { HDR_SLOT_NEXT = 0, HDR_RANGE_NEXT = 1, HDR_POOL_OVERFLOW = 2, HDR_INTS = 64 };

constexpr double kDblMax = 1.7976931348623157e308;
constexpr int kFinRows = 64;                     // rows per finalize workgroup
constexpr int kFinThreads = 1024;                // its size: one lane per row, one wave per share of the panels
constexpr int kFinSub = kFinThreads / kFinRows;  // partial sums per row (one wave each)
constexpr int kFinRegs = 8;                      // partials a thread fetches in one batch

// Writes to HBM while the matrix is streaming are far more expensive than their byte count: at
// the 20000^2 workload 20 MB of stores spread over the pass cost 80 us of a 470 us kernel, the
// same bytes written after the last load 15 us (probe kernels).  So a wave keeps everything it
// produces per row -- partial row sums, hit counts, the selected entries themselves -- in LDS and
// writes it out when its rows are done; only a buffer that fills up is flushed earlier.
#ifndef REGOT_ROW_BUF
#define REGOT_ROW_BUF 448
#endif
#ifndef REGOT_REC_CAP
#define REGOT_REC_CAP 1216
#endif
constexpr int kRowBuf = REGOT_ROW_BUF;  // rows of per-row results a wave can hold next to its staged entries
// Kernels that stage no entries have the LDS to themselves: their waves hold the results of this many rows before
// anything has to be written while the matrix still streams (a chunk of up to 4 x as many rows; taller chunks flush
// in mid-stream, which costs far more than its bytes, see flush_rows)
constexpr int kRowBufWide = 2432;       // 8-byte results (partial row sums)
constexpr int kRowBufPairs = 1216;      // 16-byte results ((max, sum) pairs of the row log-sum-exp)
constexpr int kRecCap = REGOT_REC_CAP;  // selected entries a wave can hold
constexpr int kSlot = 64;             // pool allocation unit, in records
constexpr int kMaxChunkRows = 16384;  // a record stores its row relative to the chunk in 14 bits
static_assert(kRowBuf % kRB == 0 && kRowBufWide % kRB == 0 && kRowBufPairs % kRB == 0 && kRecCap >= kPanel &&
                  kRecCap % kSlot == 0,
              "buffer sizes");

// A selected entry on its way to the CSR arrays: its value and one packed word
//   bits 0-8 column inside the panel | bits 9-17 rank inside its (row, panel) segment |
//   bits 18-31 row relative to the first row of the workgroup's chunk
// (append_records builds the word, scatter_kernel takes it apart)
static_assert(kPanel == 512, "the packed word holds a 9-bit column and a 9-bit rank");

// A run of records in the pool, written by one flush of one wave.
struct PoolRange {
    int start;    // first record (multiple of kSlot)
    int count;    // records in the run
    int panel;    // panel of the wave
    int r_begin;  // first row of the wave's chunk
};

struct Stage1Args {
    int n, m;
    int64_t ldM;
    const double *M;
    const double *alpha;
    const double *beta;
    int g_c;          // number of column panels
    int g_r;          // number of row chunks
    // Workgroups [0, wide_blocks) own one (row chunk, panel) task each, over the first wide_gc panels; with
    // wide_gc = g_c - 1 the narrow last panel is a strip that the strip_blocks workgroups behind them share,
    // rows across lanes (plan_pass_strip, row_lse_strip, col_lse_strip, read_probe_strip).  Else wide_gc = g_c.
    int wide_gc;
    int wide_blocks;
    int strip_blocks;
    // > 0 if the whole grid is resident at once with several workgroups per compute unit, b, b + pair_stride,
    // b + 2 pair_stride ... sharing one.  They then keep each other's pace (PaceKeeper).
    int pair_stride;
    int *progress;  // [grid][kWaves] groups of rows done so far, as last published
    int *cu_table;  // kernels compiled with HWPACE: [kCuKeys] CuSlot, pace keeping by hardware ids (PaceKeeperHw)
    double *rowpart;  // [g_c][n]   (LSE kernels: [g_c][n][2])
    double *colpart;  // [g_r][m]   (LSE kernels: [g_r][m][2])
    // sparsify
    double delta;
    const double *delta_dev;  // plan_pass_candidates_kernel: the threshold is read from here when the kernel starts
    int *seg_count;   // [g_c][n]: entries >= delta of row i inside panel p
    int *header;
    int pool_slots;   // capacity of the pool in units of kSlot records
    int max_ranges;
    int fixed_runs;         // g_r * g_c * kWaves: the run of a wave's last flush has the id (workgroup, wave)
    PoolRange *ranges;      // [max_ranges]: fixed_runs runs with fixed ids, then the runs of earlier flushes
    double *pool_val;       // [pool_slots * kSlot]
    unsigned *pool_packed;  // [pool_slots * kSlot]
    ExpParams ex;
};

// Workgroup id -> (row chunk g, panel p): panels of one row chunk are neighbours in the grid.
__device__ __forceinline__ void block_task(int bid, int g_c, int &g, int &p)
{
    g = bid / g_c;
    p = bid - g * g_c;
}

__device__ __forceinline__ int block_panel(int bid, int g_c)
{
    int g, p;
    block_task(bid, g_c, g, p);
    return p;
}

// rows [begin, end) of chunk g: boundaries are multiples of kRB, heights differ by at most kRB
__host__ __device__ __forceinline__ void chunk_rows(int g, int g_r, int n, int &begin, int &end)
{
    begin = (int)(((int64_t)g * n / g_r) & ~(int64_t)(kRB - 1));
    end = g == g_r - 1 ? n : (int)(((int64_t)(g + 1) * n / g_r) & ~(int64_t)(kRB - 1));
}

__global__ void init_header_kernel(int *header)
{
    if (threadIdx.x < HDR_INTS) header[threadIdx.x] = 0;
}


// A few workgroups share a compute unit for the whole pass (the grid is resident at once), one wave of
// each per SIMD.  The instruction arbiter prefers the older wave, so left alone the workgroup that was
// placed first runs ahead and finishes early, and its neighbours then have the compute unit to themselves
// at a fraction of the occupancy: measured with time stamps per workgroup, the two workgroups of a compute
// unit in the fused pass finished after 0.38 and 0.52 ms (and four per compute unit, as the row log-sum-exp
// pass used to run, after 0.27, 0.32, 0.42 and 0.47 ms; priorities did not even that out, two per compute
// unit did, which is why all streaming kernels now run that way).  The waves therefore keep pace: every kPaceEvery groups of rows a wave publishes
// how far it is, reads how far the same wave of each neighbouring workgroup was (the values arrive while
// the next rows are worked on and are used one period later), and sets its priority to the number of
// neighbours that are ahead of it.  Only the order in which the hardware issues instructions changes; which
// wave adds up what stays fixed, so results do not depend on it.  That workgroups b, b + pair_stride,
// b + 2 pair_stride ... are neighbours is an assumption about the dispatcher; if it does not hold the
// priorities are noise and nothing else.  K: workgroups per compute unit the kernel is compiled for.
constexpr int kPaceEvery = 8;

template <int K>
struct PaceKeeper {
    static_assert(K >= 2 && K <= 4, "priorities 0 .. K - 1");
    int *mine;
    const int *theirs[K - 1];  // nullptr: no such neighbour
    int seen[K - 1];           // the neighbours' progress as read one period ago ...
    int then;                  // ... and this wave's own at that moment
    // progress: [grid][kWaves] ints of the workspace; pair_stride: 0 = no pace keeping; live_blocks: workgroups of
    // the grid that take part
    __device__ __forceinline__ PaceKeeper(int *progress, int pair_stride, int w, int live_blocks)
    {
        mine = nullptr;
        then = 0;
#pragma unroll
        for (int j = 0; j < K - 1; ++j) {
            theirs[j] = nullptr;
            seen[j] = 0;
        }
        if (pair_stride > 0) {
            const int b = (int)blockIdx.x;
            mine = progress + (size_t)b * kWaves + w;
#pragma unroll
            for (int j = 0; j < K - 1; ++j) {
                const int nb = (b + (j + 1) * pair_stride) % (K * pair_stride);
                if (nb < live_blocks) theirs[j] = progress + (size_t)nb * kWaves + w;
            }
        }
    }
    // it: groups of rows this wave has finished (the same in all lanes)
    __device__ __forceinline__ void tick(int it, int lane)
    {
        if (mine == nullptr || (it % kPaceEvery) != 0) return;
        if (lane == 0) __hip_atomic_store(mine, it, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (it > 0) {
            int ahead = 0;
#pragma unroll
            for (int j = 0; j < K - 1; ++j)
                if (theirs[j] != nullptr && __builtin_amdgcn_readfirstlane(seen[j]) > then) ++ahead;
            if (ahead == 0) __builtin_amdgcn_s_setprio(0);
            else if (ahead == 1) __builtin_amdgcn_s_setprio(1);
            else if (ahead == 2) __builtin_amdgcn_s_setprio(2);
            else __builtin_amdgcn_s_setprio(3);
        }
#pragma unroll
        for (int j = 0; j < K - 1; ++j)
            if (theirs[j] != nullptr) seen[j] = __hip_atomic_load(theirs[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        then = it;
    }
};

// Pace keeping by hardware ids, for grids that run in several rounds (kernels compiled with HWPACE): a workgroup finds the compute unit it runs on in the hardware-id registers, takes one of
// two places in that unit's record and keeps pace with whoever holds the other place, whenever that workgroup was
// started.  What is compared is the work LEFT (groups of rows still to do), so that a workgroup that starts beside one
// that is almost done goes first and the workgroups of the last round finish together.  (For a grid that is resident
// at once the pairing by workgroup id above does the same with less: measured 2 % faster there; here this one is
// 5 % faster at 50000 x 50000.)  The records are cleared by finalize_kernel for the next call; on a workspace's first
// use they hold whatever was there, and a compute unit whose places look taken is simply left alone for that call.
struct CuSlot {
    int mask;                   // bit s: place s is taken
    int remaining[2][kWaves];   // groups of rows left, per place and wave, as last published
    int pad[7];
};
constexpr int kCuKeys = 2048;

__device__ __forceinline__ int cu_key()
{
    const unsigned hw = __builtin_amdgcn_s_getreg((31 << 11) | 4), xcc = __builtin_amdgcn_s_getreg((31 << 11) | 20);
    return (int)(((((xcc & 0xFu) * 8u + ((hw >> 13) & 7u)) * 2u + ((hw >> 12) & 1u)) * 16u + ((hw >> 8) & 0xFu)) & (kCuKeys - 1));
}

struct PaceKeeperHw {
    CuSlot *cu;
    int slot, w, total;
    int seen_mask, seen_rem, then_rem;
    // every thread of the workgroup calls this (it synchronises); lds2: two ints
    __device__ __forceinline__ PaceKeeperHw(int *table, bool on, int wave, int total_its, int *lds2)
    {
        cu = nullptr;
        slot = -1;
        w = wave;
        total = total_its;
        seen_mask = seen_rem = then_rem = 0;
        if (!on) return;
        if (threadIdx.x == 0) {
            const int key = cu_key();
            CuSlot *c = reinterpret_cast<CuSlot *>(table) + key;
            int s = -1;
            if ((atomicOr(&c->mask, 1) & 1) == 0) s = 0;
            else if ((atomicOr(&c->mask, 2) & 2) == 0) s = 1;
            lds2[0] = key;
            lds2[1] = s;
        }
        __syncthreads();
        cu = reinterpret_cast<CuSlot *>(table) + lds2[0];
        slot = lds2[1];
    }
    __device__ __forceinline__ void tick(int it, int lane)
    {
        if (slot < 0 || (it % kPaceEvery) != 0) return;
        const int rem = total - it;
        if (lane == 0) __hip_atomic_store(&cu->remaining[slot][w], rem, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (it > 0) {
            const bool mate = ((__builtin_amdgcn_readfirstlane(seen_mask) >> (1 - slot)) & 1) != 0;
            if (mate && then_rem > __builtin_amdgcn_readfirstlane(seen_rem)) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        seen_mask = __hip_atomic_load(&cu->mask, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        seen_rem = __hip_atomic_load(&cu->remaining[1 - slot][w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        then_rem = rem;
    }
    // after the workgroup's last barrier
    __device__ __forceinline__ void release()
    {
        if (threadIdx.x == 0 && slot >= 0) atomicAnd(&cu->mask, ~(1 << slot));
    }
};

// Per-wave LDS buffers of the plan pass.
template <bool REDUCE, bool SPARSIFY>
struct WaveBuffers {
    static constexpr int kRows = SPARSIFY ? kRowBuf : kRowBufWide;  // rows whose results the wave can hold
    static constexpr int kSumBytes = REDUCE ? kRows * 8 : 0;
    static constexpr int kValBytes = SPARSIFY ? kRecCap * 8 : 0;
    static constexpr int kPackedBytes = SPARSIFY ? kRecCap * 4 : 0;
    static constexpr int kCntBytes = SPARSIFY ? kRows * 4 : 0;
    static constexpr int kBytes = kSumBytes + kValBytes + kPackedBytes + kCntBytes;
    double *rsum;      // [kRows] partial row sums, entry = 4 * group + row inside the group
    double *val;       // [kRecCap]
    unsigned *packed;  // [kRecCap]
    int *rcnt;         // [kRows]
    __device__ __forceinline__ WaveBuffers(char *lds_raw, int w)
    {
        char *base = lds_raw + w * kBytes;
        rsum = reinterpret_cast<double *>(base);
        val = reinterpret_cast<double *>(base + kSumBytes);
        packed = reinterpret_cast<unsigned *>(base + kSumBytes + kValBytes);
        rcnt = reinterpret_cast<int *>(base + kSumBytes + kValBytes + kPackedBytes);
    }
};

// The pool's two counters (next free slot, next run beyond the fixed ones) sit side by side in the
// header and are advanced together by one 64-bit atomic: low word slots, high word runs.
__device__ __forceinline__ void pool_allocate(const Stage1Args &A, int nslots, int nruns, int &slot0, int &run0)
{
    static_assert(HDR_SLOT_NEXT == 0 && HDR_RANGE_NEXT == 1, "the two counters form one 64-bit word");
    const unsigned long long add = (unsigned long long)(unsigned)nslots | ((unsigned long long)(unsigned)nruns << 32);
    const unsigned long long old = atomicAdd(reinterpret_cast<unsigned long long *>(A.header), add);
    slot0 = (int)(unsigned)(old & 0xffffffffull);
    run0 = (int)(unsigned)(old >> 32);
}

// copy a wave's staged records to the pool at record `start` (-1: no room) and forget them
template <typename Buf>
__device__ __forceinline__ void copy_records(const Stage1Args &A, const Buf &B, int &staged, int lane, int start)
{
    if (start >= 0) {
        for (int k = lane; k < staged; k += kLanes) {
            A.pool_val[(size_t)start + k] = B.val[k];
            A.pool_packed[(size_t)start + k] = B.packed[k];
        }
    }
    staged = 0;
}

// lane 0: register run `rid` of `staged` records in `nslots` slots from slot s0; returns the first record or -1
__device__ __forceinline__ int register_run(const Stage1Args &A, int s0, int nslots, int64_t rid, int staged,
                                            int panel, int r_begin)
{
    const bool fits = s0 >= 0 && s0 + nslots <= A.pool_slots;
    if (rid < A.max_ranges) A.ranges[rid] = PoolRange{fits ? s0 * kSlot : 0, fits ? staged : 0, panel, r_begin};
    if (fits && rid < A.max_ranges) return s0 * kSlot;
    A.header[HDR_POOL_OVERFLOW] = 1;
    return -1;
}

// Write a wave's staged records to the pool as one run and register the run (when its buffer is full).
// These runs take the ids after the fixed ones, in the order in which the waves get here.
template <typename Buf>
__device__ __forceinline__ void flush_records(const Stage1Args &A, const Buf &B, int &staged, int lane, int panel,
                                              int r_begin)
{
    if (staged == 0) return;
    const int nslots = (staged + kSlot - 1) / kSlot;
    int start = -1;
    if (lane == 0) {
        int s0, extra;
        pool_allocate(A, nslots, 1, s0, extra);
        start = register_run(A, s0, nslots, (int64_t)A.fixed_runs + extra, staged, panel, r_begin);
    }
    start = __builtin_amdgcn_readfirstlane(start);
    copy_records(A, B, staged, lane, start);
}

// The last flush of all waves of a workgroup (a workgroup-wide call): one allocation for the four runs.
// All workgroups finish at about the same time, and thousands of waves adding to one counter would
// queue up on it.  The run of wave w of workgroup b gets the fixed id b * kWaves + w (written even
// when it is empty), so that the scatter kernel knows which part of the matrix a run id stands for
// without reading it.
// task: the id of the (row chunk, panel) task, g * g_c + p.
template <typename Buf>
__device__ __forceinline__ void flush_records_workgroup(const Stage1Args &A, const Buf &B, int &staged, int lane,
                                                        int w, int panel, int r_begin, int task,
                                                        int *lds_alloc /* [kWaves + 1] */)
{
    const int nslots = (staged + kSlot - 1) / kSlot;
    __syncthreads();  // a workgroup that runs several tasks: the previous call's reads of lds_alloc are done
    if (lane == 0) lds_alloc[w] = nslots;
    __syncthreads();
    if (threadIdx.x == 0) {
        int slots = 0;
        for (int q = 0; q < kWaves; ++q) slots += lds_alloc[q];
        int s0 = 0, unused = 0;
        if (slots > 0) pool_allocate(A, slots, 0, s0, unused);
        lds_alloc[kWaves] = s0;
    }
    __syncthreads();
    int start = -1;
    if (lane == 0) {
        const int64_t rid = (int64_t)task * kWaves + w;
        if (staged > 0) {
            int s0 = lds_alloc[kWaves];
            for (int q = 0; q < w; ++q) s0 += lds_alloc[q];
            start = register_run(A, s0, nslots, rid, staged, panel, r_begin);
        } else if (rid < A.max_ranges) {
            A.ranges[rid] = PoolRange{0, 0, panel, r_begin};
        }
    }
    start = __builtin_amdgcn_readfirstlane(start);
    copy_records(A, B, staged, lane, start);
}

// Append the entries of one 128-column group of a (row, panel) segment that passed the threshold.
// h0, h1: this lane's two entries; m0, m1: the same as wave-wide masks; before: hits of the segment in the
// groups before this one.  Each record carries its rank in ascending column order inside the segment, so
// the scatter kernel can place it without knowing where in the pool it landed.
template <typename Buf>
__device__ __forceinline__ void append_group(const Buf &B, int at /* first record of the row */, int before,
                                             unsigned word /* column of e = 0 | row bits */, uint64_t m0, uint64_t m1,
                                             bool h0, bool h1, double t0, double t1)
{
    // rank = hits in earlier groups, then hits of lower lanes in this group, then this lane's own two in
    // column order; a record's place in the buffer is the row's first place + its rank
    int rk0 = __builtin_amdgcn_mbcnt_hi((uint32_t)(m0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m0, (uint32_t)before));
    rk0 = __builtin_amdgcn_mbcnt_hi((uint32_t)(m1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m1, (uint32_t)rk0));
    if (h0) {
        B.val[at + rk0] = t0;
        B.packed[at + rk0] = word | ((unsigned)rk0 << 9);
    }
    if (h1) {
        const int rk1 = rk0 + (h0 ? 1 : 0);
        B.val[at + rk1] = t1;
        B.packed[at + rk1] = (word + 1u) | ((unsigned)rk1 << 9);
    }
}

// ---------------------------------------------------------------------------
// Fused pass: plan entries -> row partials, column partials, threshold hits.
// REDUCE: produce row / column partial sums.  SPARSIFY: count and stage T_ij >= delta.
// ---------------------------------------------------------------------------
// HWPACE: the grid runs in several rounds and the workgroups pair up by hardware id (PaceKeeperHw); else by workgroup id
template <bool REDUCE, bool SPARSIFY, bool ALIGNED, int MODE, bool HWPACE>
__device__ __forceinline__ void plan_pass(const Stage1Args &A, char *lds_raw, int *lds_alloc)
{
    constexpr bool FULL = MODE == kPanelFull;
    constexpr bool VEC16 = ALIGNED && (FULL || MODE == kPanelOverlapEven);
    constexpr bool GUARDED = MODE == kPanelPartial;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int g, p;
    block_task(blockIdx.x, A.wide_gc, g, p);
    int r_begin, r_end;
    chunk_rows(g, A.g_r, A.n, r_begin, r_end);

    const PanelCols<MODE> pc(p, A.m, lane);
    const int col0 = pc.col0;
    const bool(&cv)[kU][2] = pc.cv;
    double bet[kU][2];
    double cacc[kU][2];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = u * (2 * kLanes) + 2 * lane + e;
            bet[u][e] = cv[u][e] ? A.beta[col0 + c] : 0.0;
            cacc[u][e] = 0.0;
        }
    const double *Mlane = A.M + col0 + 2 * lane;
    const WaveBuffers<REDUCE, SPARSIFY> B(lds_raw, w);
    int staged = 0;  // records waiting in B.val / B.packed

    const ExpParams &ex = A.ex;
    // A group of rows is worked on in two phases, all exponentials first and the threshold work after them,
    // so that the constants of the exponential (26 scalar registers) and the masks, counts and addresses of
    // the threshold work are not all alive at the same time.
    // Phase 1, one row: v <- the plan entries (in place); returns the lane's partial row sum.
    auto plan_row = [&](double al, double (&v)[kU][2]) -> double {
        double sv[kU][2];
        double racc = 0.0;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) {  // a group of a ragged panel that owns no column: nothing to compute
                v[u][0] = v[u][1] = sv[u][0] = sv[u][1] = 0.0;
                continue;
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                sv[u][e] = (al + bet[u][e]) - v[u][e];
                double t = exp_eta(sv[u][e], ex);
                if constexpr (!FULL) t = cv[u][e] ? t : 0.0;
                v[u][e] = t;
                racc += t;
            }
        }
        // An infinite cost (or anything else outside the range reduction of exp_eta) shows up as a sum that is
        // not finite: only then are the row's entries formed again, with the IEEE limits (T = 0 for M = +inf).
        if (__ballot(not_finite(racc)) != 0) {
            racc = 0.0;
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                if (!pc.live(u)) continue;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    double t = exp_eta_any(sv[u][e], ex);
                    if constexpr (!FULL) t = cv[u][e] ? t : 0.0;
                    v[u][e] = t;
                    racc += t;
                }
            }
        }
        if constexpr (REDUCE) {
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) cacc[u][e] += v[u][e];
        }
        return racc;
    };
    // Phase 2, one row: stages the entries T >= delta; returns their number.
    // (the threshold is kept in a vector register: as a scalar it would be evicted and fetched again for
    // every comparison)
    double delta_v = A.delta;
    asm volatile("" : "+v"(delta_v));
    auto threshold_row = [&](int row, const double (&T)[kU][2]) -> int {
        auto is_hit = [&](int u, int e) -> bool {
            bool h = T[u][e] >= delta_v;
            if constexpr (!FULL) h = h && cv[u][e];
            return h;
        };
        // The records of a row stay inside one run.  While a whole row of hits would still fit the buffer
        // nothing has to be known in advance; otherwise the row's hits are counted first.
        if (staged + kPanel > kRecCap) {
            int c = 0;
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) c += __builtin_popcountll(__ballot(is_hit(u, e)));
            if (staged + c > kRecCap) flush_records(A, B, staged, lane, p, r_begin);
        }
        const unsigned row_bits = (unsigned)(row - r_begin) << 18;  // wave-uniform part of the packed word
        int cnt = 0;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const bool h0 = is_hit(u, 0), h1 = is_hit(u, 1);
            const uint64_t m0 = __ballot(h0), m1 = __ballot(h1);
            if ((m0 | m1) != 0) {
                append_group(B, staged, cnt, (unsigned)(u * (2 * kLanes) + 2 * lane) | row_bits, m0, m1, h0, h1, T[u][0], T[u][1]);
                cnt += __builtin_popcountll(m0) + __builtin_popcountll(m1);
            }
        }
        staged += cnt;
        return cnt;
    };

    // per-row results wait in LDS: entry 4*t + r belongs to row buf_row0 + 16*t + r
    int buffered = 0;  // entries in B.rsum / B.rcnt
    int buf_row0 = 0;
    auto flush_rows = [&]() {
        for (int e = lane; e < buffered; e += kLanes) {
            const size_t k = (size_t)p * A.n + buf_row0 + (kRB * kWaves) * (e >> 2) + (e & 3);
            if constexpr (REDUCE) A.rowpart[k] = B.rsum[e];
            if constexpr (SPARSIFY) A.seg_count[k] = B.rcnt[e];
        }
        buffered = 0;
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    static_assert(kRB == 4, "wave_reduce4 handles four rows per group");
    PaceKeeper<REGOT_PLAN_WAVES_PER_EU> pace(A.progress, HWPACE ? 0 : A.pair_stride, w, A.wide_blocks);
    PaceKeeperHw pace_hw(A.cu_table, HWPACE, w, (ngroups - w + kWaves - 1) / kWaves, lds_alloc);
    int it = 0;
    for (int q = w; q < ngroups; q += kWaves, ++it) {
        const int row0 = r_begin + q * kRB;
        if constexpr (HWPACE) pace_hw.tick(it, lane);
        else pace.tick(it, lane);
        double v[kRB][kU][2];
        load_rows<VEC16, GUARDED, kRB>(Mlane, A.ldM, row0, cv, pc.u_lo, pc.u_hi, v);
        double al[kRB], racc[kRB];
        int cnt[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) al[r] = A.alpha[row0 + r];
        if (buffered == WaveBuffers<REDUCE, SPARSIFY>::kRows) flush_rows();  // only chunks taller than 4 x that get here
        if (buffered == 0) buf_row0 = row0;
#ifdef REGOT_INTERLEAVE
#pragma unroll
        for (int r = 0; r < kRB; ++r) {
            racc[r] = plan_row(al[r], v[r]);
            if constexpr (SPARSIFY) cnt[r] = threshold_row(row0 + r, v[r]);
        }
#else
#pragma unroll
        for (int r = 0; r < kRB; ++r) racc[r] = plan_row(al[r], v[r]);
#endif
        if constexpr (REDUCE) {
            const double rs = wave_reduce4<OpSum>(racc[0], racc[1], racc[2], racc[3]);
            if ((lane & 15) == 0) B.rsum[buffered + quad_row(lane)] = rs;
        }
        if constexpr (SPARSIFY) {
#ifndef REGOT_INTERLEAVE
#pragma unroll
            for (int r = 0; r < kRB; ++r) cnt[r] = threshold_row(row0 + r, v[r]);
#endif
            if (lane < kRB) B.rcnt[buffered + lane] = lane == 0 ? cnt[0] : lane == 1 ? cnt[1] : lane == 2 ? cnt[2] : cnt[3];
        }
        buffered += kRB;
    }
    // all loads of this wave are done: everything it kept on chip goes out now
    flush_rows();
    // leftover rows (fewer than kRB; only the last chunk has any), spread over the waves
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        const int row = r_begin + ngroups * kRB + t;
        double v[1][kU][2];
        load_rows<VEC16, GUARDED, 1>(Mlane, A.ldM, row, cv, pc.u_lo, pc.u_hi, v);
        const double racc = plan_row(A.alpha[row], v[0]);
        int cnt = 0;
        if constexpr (SPARSIFY) cnt = threshold_row(row, v[0]);
        if constexpr (REDUCE) {
            const double rs = wave_reduce1<OpSum>(racc);
            if (lane == 0) A.rowpart[(size_t)p * A.n + row] = rs;
        }
        if constexpr (SPARSIFY) {
            if (lane == 0) A.seg_count[(size_t)p * A.n + row] = cnt;
        }
    }
    if constexpr (SPARSIFY) flush_records_workgroup(A, B, staged, lane, w, p, r_begin, g * A.g_c + p, lds_alloc);
    if constexpr (REDUCE) {
        // the wave buffers are done with: reuse the LDS to add up the four waves' column sums
        double(*lds_col)[kPanel] = reinterpret_cast<double(*)[kPanel]>(lds_raw);
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            lds_col[w][u * (2 * kLanes) + 2 * lane] = cacc[u][0];
            lds_col[w][u * (2 * kLanes) + 2 * lane + 1] = cacc[u][1];
        }
        __syncthreads();
        for (int c = threadIdx.x; c < kPanel; c += kThreads) {
            if (!PanelCols<MODE>::owns(c, p, A.m)) continue;
            double s = lds_col[0][c];
#pragma unroll
            for (int ww = 1; ww < kWaves; ++ww) s += lds_col[ww][c];
            A.colpart[(size_t)g * A.m + col0 + c] = s;
        }
    }
    if constexpr (HWPACE) {
        __syncthreads();
        pace_hw.release();
    }
}


// ---------------------------------------------------------------------------
// A narrow last panel shared by a few extra workgroups.
// A ragged last panel of few columns costs a (row chunk, panel) workgroup far more than its share of
// the bytes: one load per row in flight instead of four and most lanes idle, so it waits for the same
// memory latency per group of rows as a full panel.  When the last panel has at most kStripCols = 32
// columns, the grid is instead filled with the tasks of the full panels only, and the few workgroups
// that still fit on the chip beside them (strip_blocks) share the narrow panel's tasks: workgroup sb
// takes the row chunks g = sb, sb + strip_blocks, ...  A wave covers FOUR rows with one load: lane
// 16 r + c owns columns 2c, 2c + 1 of row r of the four, so row sums are sums over the 16 lanes of a DPP
// row, and kStripRows = 32 rows (eight loads) are in flight at a time.  Everything a strip workgroup
// leaves behind (partial sums, counts, runs of records under the fixed ids of the tasks (g, last panel),
// the records of a row next to each other in column order) is what one workgroup per task would have
// left, and every plan entry is formed by the same expression: identical bits.
// ---------------------------------------------------------------------------
constexpr int kStripCols = 32;                          // widest last panel that is run this way
constexpr int kStripLanes = kStripCols / 2;             // lanes per row
constexpr int kStripRowsPerLoad = kLanes / kStripLanes; // 4
constexpr int kStripLoads = 8;                          // loads a wave keeps in flight
constexpr int kStripRows = kStripLoads * kStripRowsPerLoad;
static_assert(kStripLanes == 16, "a row of the strip is one DPP row of lanes");

// What a lane of a strip workgroup is and holds: row `rsub` of the four rows of a load, column pair `cp` of the panel.
struct StripLane {
    int p, first, ncol, rsub, cp;
    bool cv[2];
    __device__ __forceinline__ StripLane(const Stage1Args &A, int lane)
    {
        p = A.g_c - 1;
        first = p * kPanel;   // first column of the panel (even)
        ncol = A.m - first;   // 1 .. kStripCols
        rsub = lane / kStripLanes;
        cp = lane % kStripLanes;
        cv[0] = 2 * cp < ncol;
        cv[1] = 2 * cp + 1 < ncol;
    }
};

// NL loads of four rows each, rows [row0, row0 + 4 NL); entries of rows at or beyond r_end and of columns beyond the
// panel come back as 0 with live[i] / L.cv[e] false
template <bool ALIGNED, int NL>
__device__ __forceinline__ void strip_load(const Stage1Args &A, const StripLane &L, int row0, int r_end, double (&v)[NL][2],
                                           bool (&live)[NL])
{
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int row = row0 + kStripRowsPerLoad * i + L.rsub;
        live[i] = row < r_end;
        const double *ptr = A.M + (int64_t)row * A.ldM + L.first + 2 * L.cp;
        v[i][0] = v[i][1] = 0.0;
        if (ALIGNED && (L.ncol % 2 == 0)) {
            if (live[i] && L.cv[1]) {
                const dbl2 x = __builtin_nontemporal_load(reinterpret_cast<const dbl2 *>(ptr));
                v[i][0] = x.x;
                v[i][1] = x.y;
            }
        } else {
            if (live[i] && L.cv[0]) v[i][0] = __builtin_nontemporal_load(ptr);
            if (live[i] && L.cv[1]) v[i][1] = __builtin_nontemporal_load(ptr + 1);
        }
    }
}

// the rows of chunk [r_begin, r_end) by the waves of a strip workgroup: full groups of kStripRows rows, then the rest
// four at a time (a short last four masked); fn(tag<NL>, row0)
template <typename Fn>
__device__ __forceinline__ void strip_rows(int r_begin, int r_end, int w, Fn fn)
{
    const int nrows = r_end - r_begin;
    const int nbig = nrows / kStripRows;
    for (int q = w; q < nbig; q += kWaves) fn(std::integral_constant<int, kStripLoads>{}, r_begin + q * kStripRows);
    const int done = nbig * kStripRows;
    const int nquad = (nrows - done + kStripRowsPerLoad - 1) / kStripRowsPerLoad;
    for (int q = w; q < nquad; q += kWaves) fn(std::integral_constant<int, 1>{}, r_begin + done + q * kStripRowsPerLoad);
}

template <bool REDUCE, bool SPARSIFY, bool ALIGNED>
__device__ __forceinline__ void plan_pass_strip(const Stage1Args &A, char *lds_raw, int *lds_alloc)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = A.g_c - 1;
    const int first = p * kPanel;   // first column of the panel (even)
    const int ncol = A.m - first;   // 1 .. kStripCols
    const int rsub = lane / kStripLanes, cp = lane % kStripLanes;  // row of the four, column pair
    bool cv[2];
    double bet[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        cv[e] = 2 * cp + e < ncol;
        bet[e] = cv[e] ? A.beta[first + 2 * cp + e] : 0.0;
    }
    // a ragged last panel counts its columns from m - kPanel (see plan_pass and the scatter kernel)
    const unsigned col_word = (unsigned)(kPanel - ncol + 2 * cp);
    const uint64_t rows_below = rsub == 0 ? 0ull : (~0ull >> (kLanes - kStripLanes * rsub));  // lanes of the rows before this lane's
    const uint64_t row_lanes = 0xffffull << (kStripLanes * rsub);
    const int sb = (int)blockIdx.x - A.wide_blocks;
    const WaveBuffers<REDUCE, SPARSIFY> B(lds_raw, w);
    const ExpParams &ex = A.ex;
    double delta_v = A.delta;
    asm volatile("" : "+v"(delta_v));
    int staged = 0;
    // A strip workgroup is the youngest on its compute unit, and the instruction arbiter prefers older waves:
    // left at that it would get what its neighbour leaves and finish last.  Its work is light, so it goes first
    // instead and is done well before the neighbour.
    __builtin_amdgcn_s_setprio(3);

    for (int g = sb; g < A.g_r; g += A.strip_blocks) {
        int r_begin, r_end;
        chunk_rows(g, A.g_r, A.n, r_begin, r_end);
        double cacc[2] = {0.0, 0.0};
        // rows [row0, row0 + NL * 4) of the chunk, those at or beyond r_end masked out
        auto rows = [&](auto nl_tag, int row0) {
            constexpr int NL = decltype(nl_tag)::value;
            double v[NL][2];
            double al[NL];
            bool live[NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int row = row0 + kStripRowsPerLoad * i + rsub;
                live[i] = row < r_end;
                const double *ptr = A.M + (int64_t)row * A.ldM + first + 2 * cp;
                v[i][0] = v[i][1] = 0.0;
                if (ALIGNED && (ncol % 2 == 0)) {
                    if (live[i] && cv[1]) {
                        const dbl2 x = __builtin_nontemporal_load(reinterpret_cast<const dbl2 *>(ptr));
                        v[i][0] = x.x;
                        v[i][1] = x.y;
                    }
                } else {
                    if (live[i] && cv[0]) v[i][0] = __builtin_nontemporal_load(ptr);
                    if (live[i] && cv[1]) v[i][1] = __builtin_nontemporal_load(ptr + 1);
                }
                al[i] = live[i] ? A.alpha[row] : 0.0;
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int row = row0 + kStripRowsPerLoad * i + rsub;
                double racc = 0.0;
                double sv[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    sv[e] = (al[i] + bet[e]) - v[i][e];
                    double t = exp_eta(sv[e], ex);
                    t = (live[i] && cv[e]) ? t : 0.0;
                    v[i][e] = t;
                    racc += t;
                }
                if (__ballot(not_finite(racc)) != 0) {  // as in plan_pass: the IEEE limits for what exp_eta cannot reduce
                    racc = 0.0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        double t = exp_eta_any(sv[e], ex);
                        t = (live[i] && cv[e]) ? t : 0.0;
                        v[i][e] = t;
                        racc += t;
                    }
                }
                if constexpr (REDUCE) {
                    cacc[0] += v[i][0];
                    cacc[1] += v[i][1];
                }
                // per-row results go straight to memory: a strip workgroup's are few
                if constexpr (REDUCE) {
                    const double rs = row16_reduce<OpSum>(racc);
                    if (cp == 0 && live[i]) A.rowpart[(size_t)p * A.n + row] = rs;
                }
                if constexpr (SPARSIFY) {
                    const bool h0 = v[i][0] >= delta_v && live[i] && cv[0], h1 = v[i][1] >= delta_v && live[i] && cv[1];
                    const uint64_t m0 = __ballot(h0), m1 = __ballot(h1);
                    const int all = __builtin_popcountll(m0) + __builtin_popcountll(m1);
                    if (all != 0) {
                        if (staged + all > kRecCap) flush_records(A, B, staged, lane, p, r_begin);
                        // place in the buffer: hits of all lower lanes (earlier rows, then lower columns of the same
                        // row) come first; rank inside the row: without those of the earlier rows
                        const int before_rows = __builtin_popcountll(m0 & rows_below) + __builtin_popcountll(m1 & rows_below);
                        append_group(B, staged + before_rows, -before_rows, col_word | ((unsigned)(row - r_begin) << 18), m0, m1,
                                     h0, h1, v[i][0], v[i][1]);
                        staged += all;
                    }
                    if (cp == 0 && live[i])
                        A.seg_count[(size_t)p * A.n + row] = __builtin_popcountll(m0 & row_lanes) + __builtin_popcountll(m1 & row_lanes);
                }
            }
        };
        const int nrows = r_end - r_begin;
        const int nbig = nrows / kStripRows;
        for (int q = w; q < nbig; q += kWaves) rows(std::integral_constant<int, kStripLoads>{}, r_begin + q * kStripRows);
        // the rows beyond the last full group, four at a time (a short last four masked)
        const int done = nbig * kStripRows;
        const int nquad = (nrows - done + kStripRowsPerLoad - 1) / kStripRowsPerLoad;
        for (int q = w; q < nquad; q += kWaves) rows(std::integral_constant<int, 1>{}, r_begin + done + q * kStripRowsPerLoad);

        if constexpr (SPARSIFY) flush_records_workgroup(A, B, staged, lane, w, p, r_begin, g * A.g_c + p, lds_alloc);
        if constexpr (REDUCE) {
            // column sums of the task: over the four rows of the lanes and the four waves (the slots for partial
            // row sums are free in a strip workgroup)
            B.rsum[2 * lane] = cacc[0];
            B.rsum[2 * lane + 1] = cacc[1];
            __syncthreads();
            const int c = (int)threadIdx.x;
            if (c < ncol) {
                double sum = 0.0;
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww)
#pragma unroll
                    for (int r = 0; r < kStripRowsPerLoad; ++r)
                        sum += WaveBuffers<REDUCE, SPARSIFY>(lds_raw, ww).rsum[2 * (kStripLanes * r) + c];
                A.colpart[(size_t)g * A.m + first + c] = sum;
            }
            __syncthreads();
        }
    }
}

constexpr int plan_lds_bytes(bool reduce, bool sparsify)
{
    const int rows = sparsify ? kRowBuf : kRowBufWide;
    const int bufs = kWaves * ((reduce ? rows * 8 : 0) + (sparsify ? kRecCap * 12 + rows * 4 : 0));
    const int cols = reduce ? kWaves * kPanel * (int)sizeof(double) : 16;
    return bufs > cols ? bufs : cols;
}

template <bool REDUCE, bool SPARSIFY, bool ALIGNED, bool HWPACE = false>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_PLAN_WAVES_PER_EU) void plan_pass_kernel(Stage1Args A)
{
    __shared__ __attribute__((aligned(16))) char lds_raw[plan_lds_bytes(REDUCE, SPARSIFY)];
    __shared__ int lds_alloc[kWaves + 1];
    static_assert((plan_lds_bytes(REDUCE, SPARSIFY) + 64) * REGOT_PLAN_WAVES_PER_EU <= 160 * 1024, "LDS per CU");
    if ((int)blockIdx.x >= A.wide_blocks) {
        plan_pass_strip<REDUCE, SPARSIFY, ALIGNED>(A, lds_raw, lds_alloc);
        return;
    }
    switch (panel_mode(block_panel(blockIdx.x, A.wide_gc), A.m)) {
    case kPanelFull: plan_pass<REDUCE, SPARSIFY, ALIGNED, kPanelFull, HWPACE>(A, lds_raw, lds_alloc); break;
    case kPanelOverlap: plan_pass<REDUCE, SPARSIFY, ALIGNED, kPanelOverlap, HWPACE>(A, lds_raw, lds_alloc); break;
    case kPanelOverlapEven: plan_pass<REDUCE, SPARSIFY, ALIGNED, kPanelOverlapEven, HWPACE>(A, lds_raw, lds_alloc); break;
    default: plan_pass<REDUCE, SPARSIFY, ALIGNED, kPanelPartial, HWPACE>(A, lds_raw, lds_alloc); break;
    }
}

// The fused pass with a threshold that an earlier kernel of the stream has computed: read from
// A.delta_dev when the kernel starts.  (A kernel of its own, so that the one above keeps its code.)
template <bool ALIGNED, bool HWPACE = false>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_PLAN_WAVES_PER_EU) void plan_pass_candidates_kernel(Stage1Args A)
{
    __shared__ __attribute__((aligned(16))) char lds_raw[plan_lds_bytes(true, true)];
    __shared__ int lds_alloc[kWaves + 1];
    A.delta = *A.delta_dev;
    if ((int)blockIdx.x >= A.wide_blocks) {
        plan_pass_strip<true, true, ALIGNED>(A, lds_raw, lds_alloc);
        return;
    }
    switch (panel_mode(block_panel(blockIdx.x, A.wide_gc), A.m)) {
    case kPanelFull: plan_pass<true, true, ALIGNED, kPanelFull, HWPACE>(A, lds_raw, lds_alloc); break;
    case kPanelOverlap: plan_pass<true, true, ALIGNED, kPanelOverlap, HWPACE>(A, lds_raw, lds_alloc); break;
    case kPanelOverlapEven: plan_pass<true, true, ALIGNED, kPanelOverlapEven, HWPACE>(A, lds_raw, lds_alloc); break;
    default: plan_pass<true, true, ALIGNED, kPanelPartial, HWPACE>(A, lds_raw, lds_alloc); break;
    }
}

// ---------------------------------------------------------------------------
// Measurement aid: where the dispatcher puts the workgroups of a grid that is launched like the plan pass (same
// workgroup size, same LDS, two per compute unit).  ids[2 b] = HW_ID register of workgroup b's first wave
// (compute unit [11:8], shader array [12], shader engine [15:13]), ids[2 b + 1] = XCC_ID register (die [3:0]).
// Every workgroup stays for about 20 us so that the whole grid is placed before any of it leaves.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_PLAN_WAVES_PER_EU) void placement_probe_kernel(unsigned *ids)
{
    __shared__ __attribute__((aligned(16))) char lds_raw[plan_lds_bytes(true, true)];
    if (threadIdx.x == 0) {
        lds_raw[0] = 0;  // (the array must be used for its size to count)
        ids[2 * blockIdx.x] = __builtin_amdgcn_s_getreg((31 << 11) | 4);
        ids[2 * blockIdx.x + 1] = __builtin_amdgcn_s_getreg((31 << 11) | 20);
    }
    const unsigned long long t0 = wall_clock64();  // 100 MHz
    while (wall_clock64() - t0 < 2000ull) __builtin_amdgcn_s_sleep(32);
    if (threadIdx.x == 1 && lds_raw[0] != 0) ids[0] = 0u;  // never true
}

// ---------------------------------------------------------------------------
// Measurement aid: the same cut of the matrix and the same loads as the plan pass, and nothing else
// (every entry is added to one sum per lane).  Its duration is what this tiling can stream from memory
// on the device at hand, the figure the streaming kernels are to be compared with.
// ---------------------------------------------------------------------------
template <bool ALIGNED, int MODE>
__device__ __forceinline__ double read_probe_pass(const Stage1Args &A)
{
    constexpr bool FULL = MODE == kPanelFull;
    constexpr bool VEC16 = ALIGNED && (FULL || MODE == kPanelOverlapEven);
    constexpr bool GUARDED = MODE == kPanelPartial;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int g, p;
    block_task(blockIdx.x, A.wide_gc, g, p);
    int r_begin, r_end;
    chunk_rows(g, A.g_r, A.n, r_begin, r_end);
    const PanelCols<MODE> pc(p, A.m, lane);
    const bool(&cv)[kU][2] = pc.cv;
    const double *Mlane = A.M + pc.col0 + 2 * lane;
    double acc = 0.0;
    auto add = [&](const double (&v)[kU][2]) {
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) acc += (FULL || cv[u][e]) ? v[u][e] : 0.0;
    };
    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) {
        double v[kRB][kU][2];
        load_rows<VEC16, GUARDED, kRB>(Mlane, A.ldM, r_begin + q * kRB, cv, pc.u_lo, pc.u_hi, v);
#pragma unroll
        for (int r = 0; r < kRB; ++r) add(v[r]);
    }
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        double v[1][kU][2];
        load_rows<VEC16, GUARDED, 1>(Mlane, A.ldM, r_begin + ngroups * kRB + t, cv, pc.u_lo, pc.u_hi, v);
        add(v[0]);
    }
    return acc;
}

// the narrow last panel by strip workgroups, as in plan_pass_strip
template <bool ALIGNED>
__device__ __forceinline__ double read_probe_strip(const Stage1Args &A)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const StripLane L(A, lane);
    double acc = 0.0;
    for (int g = (int)blockIdx.x - A.wide_blocks; g < A.g_r; g += A.strip_blocks) {
        int r_begin, r_end;
        chunk_rows(g, A.g_r, A.n, r_begin, r_end);
        strip_rows(r_begin, r_end, w, [&](auto nl_tag, int row0) {
            constexpr int NL = decltype(nl_tag)::value;
            double v[NL][2];
            bool live[NL];
            strip_load<ALIGNED, NL>(A, L, row0, r_end, v, live);
#pragma unroll
            for (int i = 0; i < NL; ++i) acc += v[i][0] + v[i][1];
        });
    }
    return acc;
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_PLAN_WAVES_PER_EU) void read_probe_kernel(Stage1Args A)
{
    __shared__ double lds[kWaves];
    double acc;
    if ((int)blockIdx.x >= A.wide_blocks) acc = read_probe_strip<ALIGNED>(A);
    else
    switch (panel_mode(block_panel(blockIdx.x, A.wide_gc), A.m)) {
    case kPanelFull: acc = read_probe_pass<ALIGNED, kPanelFull>(A); break;
    case kPanelOverlap: acc = read_probe_pass<ALIGNED, kPanelOverlap>(A); break;
    case kPanelOverlapEven: acc = read_probe_pass<ALIGNED, kPanelOverlapEven>(A); break;
    default: acc = read_probe_pass<ALIGNED, kPanelPartial>(A); break;
    }
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) A.colpart[blockIdx.x] = s;  // (the region for column partials holds at least one double per task)
}

// one workgroup: the tasks' sums in a fixed order
__global__ __launch_bounds__(kThreads) void read_probe_sum_kernel(const double *part, int nparts, double *out)
{
    __shared__ double lds[kWaves];
    double s = 0.0;
    for (int k = threadIdx.x; k < nparts; k += kThreads) s += part[k];
    s = block_sum(s, lds);
    if (threadIdx.x == 0) *out = s;
}

// ---------------------------------------------------------------------------
// Second stage of the fused pass: combine partials, gradient, per-row CSR offsets.
// Row workgroups: kFinRows rows, one wave per share of the panels (coalesced over rows).
// Column workgroups: 64 columns, one wave per share of the row chunks.
// The kernel is a chain of memory latencies, not of bytes: with 16 waves per row block a thread has
// at most kFinRegs partials to fetch unless the matrix has more than 128 panels (or row chunks), and
// it asks for all of them at once and keeps the counts for the prefix in registers.
// ---------------------------------------------------------------------------
struct FinalizeArgs {
    int n, m, g_c, g_r;
    const double *rowpart;
    const double *colpart;
    const double *a, *b, *alpha, *beta;
    double eta;
    double *obj, *grad_alpha, *grad_beta, *row_sum, *col_sum;
    double *objpart;     // [gridDim.x][3]
    int nblk_rows;       // workgroups [0, nblk_rows) own rows, the rest own columns
    int *header;
    int *seg_count;      // [g_c][n] in: counts; out: exclusive prefix over panels inside the row
    int64_t *row_excl;   // [n] exclusive prefix of the row's nnz inside its workgroup (64 rows x m columns can pass 2^31)
    int64_t *blk_nnz;    // [nblk_rows] nnz of the workgroup's rows (epilogue_kernel, when it runs, turns it into offsets)
    int64_t capacity;
    int64_t *info;
    int *cu_table;       // PaceKeeperHw's records: cleared for the next call (nullptr: not used by this call)
};

// sum of part[p * stride + idx] over p in [p0, p1), fetched in one batch when there are at most kFinRegs
__device__ __forceinline__ double sum_partials(const double *part, size_t stride, int64_t idx, int p0, int p1,
                                               bool live)
{
    double r = 0.0;
    if (p1 - p0 <= kFinRegs) {
        double v[kFinRegs];
#pragma unroll
        for (int j = 0; j < kFinRegs; ++j) v[j] = (live && p0 + j < p1) ? part[(size_t)(p0 + j) * stride + idx] : 0.0;
#pragma unroll
        for (int j = 0; j < kFinRegs; ++j) r += v[j];
    } else if (live) {
#pragma unroll 4
        for (int p = p0; p < p1; ++p) r += part[(size_t)p * stride + idx];
    }
    return r;
}

template <bool REDUCE, bool SPARSIFY>
__global__ __launch_bounds__(kFinThreads) void finalize_kernel(FinalizeArgs F)
{
    __shared__ double lds_part[kFinSub][kLanes];
    __shared__ int lds_cnt[kFinSub][kLanes];
    const int tid = threadIdx.x;
    const int l = tid & (kLanes - 1), sub = tid >> 6;
    static_assert(kFinRows == kLanes, "one lane per row");
    if (blockIdx.x == gridDim.x - 1 && F.cu_table != nullptr)
        for (int i = tid; i < kCuKeys * (int)(sizeof(CuSlot) / sizeof(int)); i += kFinThreads) F.cu_table[i] = 0;
    double pS = 0.0, pA = 0.0, pB = 0.0;
    if ((int)blockIdx.x < F.nblk_rows) {
        const int64_t i = (int64_t)blockIdx.x * kFinRows + l;
        const bool live = i < F.n;
        const int per = (F.g_c + kFinSub - 1) / kFinSub;
        const int p0 = min(F.g_c, sub * per), p1 = min(F.g_c, p0 + per);
        const bool batch = per <= kFinRegs;  // the same in every workgroup
        int c[kFinRegs];
        int mine = 0;
        if constexpr (SPARSIFY) {
            if (batch) {
#pragma unroll
                for (int j = 0; j < kFinRegs; ++j) c[j] = (live && p0 + j < p1) ? F.seg_count[(size_t)(p0 + j) * F.n + i] : 0;
            }
        }
        if constexpr (REDUCE) lds_part[sub][l] = sum_partials(F.rowpart, (size_t)F.n, i, p0, p1, live);
        if constexpr (SPARSIFY) {
            if (batch) {
#pragma unroll
                for (int j = 0; j < kFinRegs; ++j) mine += c[j];
            } else if (live) {
#pragma unroll 4
                for (int p = p0; p < p1; ++p) mine += F.seg_count[(size_t)p * F.n + i];
            }
            lds_cnt[sub][l] = mine;
        }
        __syncthreads();
        if constexpr (REDUCE) {
            if (sub == 0 && live) {
                double r = lds_part[0][l];
#pragma unroll
                for (int s = 1; s < kFinSub; ++s) r += lds_part[s][l];
                const double ai = F.a[i];
                if (F.row_sum) F.row_sum[i] = r;
                F.grad_alpha[i] = ai - r;
                pS = r;
                pA = F.alpha[i] * ai;
            }
        }
        if constexpr (SPARSIFY) {
            int run = 0;
            for (int s = 0; s < sub; ++s) run += lds_cnt[s][l];
            if (batch) {
#pragma unroll
                for (int j = 0; j < kFinRegs; ++j)
                    if (live && p0 + j < p1) {
                        F.seg_count[(size_t)(p0 + j) * F.n + i] = run;
                        run += c[j];
                    }
            } else if (live) {
                for (int p = p0; p < p1; ++p) {
                    const size_t k = (size_t)p * F.n + i;
                    const int cnt = F.seg_count[k];
                    F.seg_count[k] = run;
                    run += cnt;
                }
            }
            if (sub == 0) {
                // nnz of each of the 64 rows, then their exclusive scan across the wave
                int v = 0;
#pragma unroll
                for (int s = 0; s < kFinSub; ++s) v += lds_cnt[s][l];
                if (!live) v = 0;
                long long inc = v;
#pragma unroll
                for (int d = 1; d < kLanes; d <<= 1) {
                    const long long up = __shfl_up(inc, d, kLanes);
                    if (l >= d) inc += up;
                }
                if (live) F.row_excl[i] = inc - v;
                if (l == kLanes - 1) F.blk_nnz[blockIdx.x] = inc;
            }
        }
    } else if constexpr (REDUCE) {
        const int64_t j = (int64_t)((int)blockIdx.x - F.nblk_rows) * kLanes + l;
        const int per = (F.g_r + kFinSub - 1) / kFinSub;
        const int g0 = min(F.g_r, sub * per), g1 = min(F.g_r, g0 + per);
        lds_part[sub][l] = sum_partials(F.colpart, (size_t)F.m, j, g0, g1, j < F.m);
        __syncthreads();
        if (sub == 0 && j < F.m) {
            double c = lds_part[0][l];
#pragma unroll
            for (int s = 1; s < kFinSub; ++s) c += lds_part[s][l];
            const double bj = F.b[j];
            if (F.col_sum) F.col_sum[j] = c;
            F.grad_beta[j] = bj - c;
            pB = F.beta[j] * bj;
        }
    }
    if constexpr (REDUCE) {
        // only the first wave holds terms of the objective
        if (sub == 0) {
            const double bS = wave_reduce1<OpSum>(pS), bA = wave_reduce1<OpSum>(pA), bB = wave_reduce1<OpSum>(pB);
            if (l == 0) {
                F.objpart[(size_t)blockIdx.x * 3 + 0] = bS;
                F.objpart[(size_t)blockIdx.x * 3 + 1] = bA;
                F.objpart[(size_t)blockIdx.x * 3 + 2] = bB;
            }
        }
    }
}

// Objective from the per-workgroup partials of finalize_kernel (one workgroup, fixed order).
__device__ __forceinline__ void write_objective(const FinalizeArgs &F, int nparts, double *lds)
{
    double S = 0.0, dA = 0.0, dB = 0.0;
    for (int k = threadIdx.x; k < nparts; k += kThreads) {
        S += F.objpart[(size_t)k * 3 + 0];
        dA += F.objpart[(size_t)k * 3 + 1];
        dB += F.objpart[(size_t)k * 3 + 2];
    }
    S = block_sum(S, lds);
    dA = block_sum(dA, lds);
    dB = block_sum(dB, lds);
    if (threadIdx.x == 0) *F.obj = -F.eta * S + (dA + dB);
}

// Third stage, one workgroup: objective from the per-workgroup partials, and the exclusive scan of
// the per-workgroup nnz that turns row-local offsets into row_ptr.  (A separate launch rather than a
// "last workgroup done" epilogue: a kernel boundary makes the partials visible once, where a
// device-scope fence in every workgroup would write the L2 back hundreds of times.)
// Sparsify calls with at most kFoldBlocks row workgroups skip this launch: there the scatter kernel
// scans the counts itself (see scatter_kernel).
template <bool REDUCE, bool SPARSIFY>
__global__ __launch_bounds__(kThreads) void epilogue_kernel(FinalizeArgs F, int nparts)
{
    __shared__ double lds[kWaves];
    __shared__ long long lds_scan[kThreads];
    const int tid = threadIdx.x;
    if constexpr (REDUCE) write_objective(F, nparts, lds);
    if constexpr (SPARSIFY) {
        // each thread owns a contiguous range of row workgroups
        const int per = (F.nblk_rows + kThreads - 1) / kThreads;
        const int lo = min(F.nblk_rows, per * tid), hi = min(F.nblk_rows, lo + per);
        long long mine = 0;
        for (int k = lo; k < hi; ++k) mine += F.blk_nnz[k];
        lds_scan[tid] = mine;
        __syncthreads();
        for (int d = 1; d < kThreads; d <<= 1) {
            const long long up = tid >= d ? lds_scan[tid - d] : 0;
            __syncthreads();
            lds_scan[tid] += up;
            __syncthreads();
        }
        long long run = lds_scan[tid] - mine;
        for (int k = lo; k < hi; ++k) {
            const long long c = F.blk_nnz[k];
            F.blk_nnz[k] = run;
            run += c;
        }
        if (tid == kThreads - 1) {
            const long long total = lds_scan[tid];
            F.info[0] = total;
            F.info[1] = (total > F.capacity || F.header[HDR_POOL_OVERFLOW] != 0) ? 1 : 0;
        }
    }
}

// Write row_ptr and place every staged record at its CSR position.
struct ScatterArgs {
    int n, m, g_c, g_r;
    const int *header;
    int max_ranges;
    int fixed_runs;           // g_r * g_c * kWaves
    const PoolRange *ranges;
    const double *pool_val;
    const unsigned *pool_packed;
    const int *seg_rel;       // [g_c][n] exclusive prefix inside the row
    const int64_t *row_excl;  // [n]
    int64_t capacity;         // entries of col_idx / val
    const int64_t *blk_off;   // [ceil(n / kFinRows)]: offsets after the epilogue; FOLD: still the counts
    int nblk;                 // ceil(n / kFinRows)
    int64_t *info;
    int64_t *row_ptr;
    int32_t *col_idx;
    double *val;
    // FILTER: the runs hold candidates; only those with a value >= *delta_dev are entries of the CSR
    const double *delta_dev;
    const int64_t *select_info;  // [2] of the selection that found *delta_dev; negative: it failed
};

constexpr int kFoldBlocks = 1024;  // row workgroups up to which the scatter kernel does the scan itself
static_assert(kFoldBlocks % kThreads == 0, "each thread scans the same number of counts");

constexpr int kFoldPerThread = kFoldBlocks / kThreads;

// Exclusive scan of the nblk <= kFoldBlocks per-workgroup entry counts (c: this thread's
// kFoldPerThread consecutive counts) into lds_off; returns their sum.
__device__ __forceinline__ long long fold_offsets(const long long (&c)[kFoldPerThread], long long *lds_off,
                                                  long long *lds_wave)
{
    const int tid = threadIdx.x, lane = tid & (kLanes - 1), wave = tid >> 6;
    long long mine = 0;
#pragma unroll
    for (int j = 0; j < kFoldPerThread; ++j) mine += c[j];
    long long inc = mine;
#pragma unroll
    for (int d = 1; d < kLanes; d <<= 1) {
        const long long up = __shfl_up(inc, d, kLanes);
        if (lane >= d) inc += up;
    }
    if (lane == kLanes - 1) lds_wave[wave] = inc;
    __syncthreads();
    long long run = inc - mine, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave) run += lds_wave[w];
        total += lds_wave[w];
    }
#pragma unroll
    for (int j = 0; j < kFoldPerThread; ++j) {
        lds_off[tid * kFoldPerThread + j] = run;
        run += c[j];
    }
    __syncthreads();
    return total;
}

constexpr int kXcds = 8;  // accelerator dies; workgroups b of a grid with equal b % kXcds are placed on one die

// Work item t of the scatter kernel -> the run it places (-1: none).
// The pieces of one CSR row come from the g_c runs of one (row chunk, wave) pair, a few entries from
// each panel, so the runs of a pair write into the same cache lines.  Every die has its own L2: the
// items are ordered so that a pair's runs are taken by workgroups of one die at about the same time,
// which lets that L2 put the lines together before they go to memory.  (The order only matters for
// speed; the dispatcher's placement rule is an assumption, not something the result depends on.)
// Items beyond the fixed runs are the runs of earlier flushes, in the order of their ids.
__device__ __forceinline__ int64_t scatter_item_run(const ScatterArgs &S, int64_t t, int64_t n_runs)
{
    const int pairs = S.g_r * kWaves;
    const int64_t fixed_items = (int64_t)kXcds * S.g_c * ((pairs + kXcds - 1) / kXcds);
    int64_t rid;
    if (t < fixed_items) {
        const int die = (int)(t % kXcds);
        const int64_t q = t / kXcds;
        const int pair = die + kXcds * (int)(q / S.g_c), p = (int)(q % S.g_c);
        if (pair >= pairs) return -1;
        rid = ((int64_t)(pair / kWaves) * S.g_c + p) * kWaves + pair % kWaves;
    } else {
        rid = S.fixed_runs + (t - fixed_items);
    }
    return rid < n_runs ? rid : -1;
}

__host__ __device__ inline int64_t scatter_fixed_items(int g_r, int g_c)
{
    return (int64_t)kXcds * g_c * (((int64_t)g_r * kWaves + kXcds - 1) / kXcds);
}

// FOLD: launched straight after finalize_kernel, with one workgroup more than the records need.
// Every workgroup scans the per-workgroup counts itself (a few KB from the L2) instead of waiting
// for a one-workgroup launch to do it, and the extra workgroup writes the scalars of the call
// (entry count, overflow flag and, with REDUCE, the objective).
// The number of workgroups that place records is a multiple of kXcds (see scatter_item_run).
// FILTER: the runs hold candidates of a threshold that was only found after the pass (*delta_dev): records
// below it are skipped (the ranks of the others have been renumbered by then, regot_refresh.hpp).
// A failed selection (select_info negative, threshold NaN) places nothing and sets bit 1 of info[1].
template <bool FOLD, bool REDUCE, bool FILTER = false>
__global__ __launch_bounds__(kThreads) void scatter_kernel(ScatterArgs S, FinalizeArgs F, int nparts)
{
    __shared__ long long lds_off[FOLD ? kFoldBlocks : 1];
    __shared__ long long lds_wave[kWaves];
    __shared__ double lds[kWaves];
    // Everything whose address is known at launch is requested first, so that these loads overlap
    // instead of forming a chain: the header, the counts to scan, and the workgroup's first run
    // (read even if the header then says that the run does not exist: the array does).
    const int work_blocks = FOLD ? gridDim.x - 1 : gridDim.x;
    const int hdr_runs = S.header[HDR_RANGE_NEXT];
    const int hdr_overflow = S.header[HDR_POOL_OVERFLOW];
    const int64_t first = scatter_item_run(S, blockIdx.x, S.max_ranges);
    PoolRange R = S.ranges[first >= 0 ? first : 0];
    long long cnt[kFoldPerThread];
    if constexpr (FOLD) {
#pragma unroll
        for (int j = 0; j < kFoldPerThread; ++j) {
            const int k = threadIdx.x * kFoldPerThread + j;
            cnt[j] = k < S.nblk ? S.blk_off[k] : 0;
        }
    }
    const int64_t n_runs = min((int64_t)S.fixed_runs + hdr_runs, (int64_t)S.max_ranges);
    const int64_t n_items = scatter_fixed_items(S.g_r, S.g_c) + max(n_runs - S.fixed_runs, (int64_t)0);
    long long total;
    bool overflow;
    if constexpr (FOLD) {
        const bool extra = blockIdx.x == gridDim.x - 1;
        if (!extra && (int64_t)blockIdx.x >= n_items && (int64_t)blockIdx.x * kThreads > S.n) return;
        if (extra) {
            if constexpr (REDUCE) write_objective(F, nparts, lds);
        }
        total = fold_offsets(cnt, lds_off, lds_wave);
        overflow = total > S.capacity || hdr_overflow != 0;
        if (extra) {
            if (threadIdx.x == 0) {
                S.info[0] = total;
                long long flags = overflow ? 1 : 0;
                if constexpr (FILTER) flags |= S.select_info[0] < 0 ? 2 : 0;
                S.info[1] = flags;
            }
            return;
        }
    } else {
        // epilogue_kernel has written the scalars of the call; bit 1 of info[1] is added here
        total = S.info[0];
        overflow = (S.info[1] & 1) != 0;
        if constexpr (FILTER) {
            if (blockIdx.x == 0 && threadIdx.x == 0 && S.select_info[0] < 0)
                atomicOr(reinterpret_cast<unsigned long long *>(&S.info[1]), 2ull);
        }
    }
    double delta = 0.0;
    if constexpr (FILTER) delta = *S.delta_dev;
    auto block_offset = [&](int row) -> int64_t {
        if constexpr (FOLD) return lds_off[row / kFinRows];
        else return S.blk_off[row / kFinRows];
    };
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i <= S.n; i += (int64_t)work_blocks * kThreads)
        S.row_ptr[i] = i < S.n ? block_offset((int)i) + S.row_excl[i] : total;
    if (overflow) return;
    constexpr int kPer = (kRecCap + kThreads - 1) / kThreads;  // records per thread of one run
    for (int64_t t = blockIdx.x; t < n_items; t += work_blocks) {
        const int64_t r = scatter_item_run(S, t, n_runs);
        if (r < 0) continue;
        if (t != (int64_t)blockIdx.x) R = S.ranges[r];
        if (R.count == 0) continue;
        // the ragged last panel of a wide matrix is shifted to start at m - kPanel
        const int col0 = (R.panel == S.g_c - 1 && S.m >= kPanel) ? S.m - kPanel : R.panel * kPanel;
        const int *seg = S.seg_rel + (size_t)R.panel * S.n;
        // all loads of a thread's records first, then the gathers, then the stores
        unsigned pk[kPer];
        double v[kPer];
        int64_t dest[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int k = threadIdx.x + j * kThreads;
            pk[j] = k < R.count ? S.pool_packed[(size_t)R.start + k] : 0u;
            v[j] = k < R.count ? S.pool_val[(size_t)R.start + k] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int k = threadIdx.x + j * kThreads;
            const int row = min(R.r_begin + (int)(pk[j] >> 18), S.n - 1);
            bool keep = k < R.count;
            if constexpr (FILTER) keep = keep && v[j] >= delta;
            dest[j] = keep ? block_offset(row) + S.row_excl[row] + seg[row] + (int)((pk[j] >> 9) & 511) : -1;
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (dest[j] >= 0 && dest[j] < S.capacity) {  // (always below the capacity without overflow)
                S.col_idx[dest[j]] = col0 + (int)(pk[j] & 511);
                S.val[dest[j]] = v[j];
            }
    }
}

// ---------------------------------------------------------------------------
// Sinkhorn half-steps in the log domain.  Quantities are kept in units of s
// (= eta * x): a partial log-sum-exp is the pair (smax, sum exp((s - smax)/eta)).
// ---------------------------------------------------------------------------

// which = 0: per row i, over the columns of one panel, s_ij = beta_j - M_ij.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void row_lse_pass(const Stage1Args &A, dbl2 *lds_pairs)
{
    constexpr bool FULL = MODE == kPanelFull;
    constexpr bool VEC16 = ALIGNED && (FULL || MODE == kPanelOverlapEven);
    constexpr bool GUARDED = MODE == kPanelPartial;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int g, p;
    block_task(blockIdx.x, A.wide_gc, g, p);
    int r_begin, r_end;
    chunk_rows(g, A.g_r, A.n, r_begin, r_end);

    const PanelCols<MODE> pc(p, A.m, lane);
    const int col0 = pc.col0;
    const bool(&cv)[kU][2] = pc.cv;
    double bet[kU][2];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = u * (2 * kLanes) + 2 * lane + e;
            bet[u][e] = cv[u][e] ? A.beta[col0 + c] : 0.0;
        }
    const double *Mlane = A.M + col0 + 2 * lane;

    // v <- s = beta - M; returns the lane's maximum over its valid columns
    auto to_s = [&](double (&v)[kU][2]) -> double {
        double lmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                v[u][e] = bet[u][e] - v[u][e];
                if (FULL || cv[u][e]) lmax = fmax(lmax, v[u][e]);
            }
        return lmax;
    };
    // (wmax: the row's maximum over the panel, at least -DBL_MAX so that a panel of infinite costs only gives
    // s - wmax = -inf, a term 0, and an empty partial sum)
    auto sum_exp = [&](const double (&s)[kU][2], double wmax) -> double {
        double acc = 0.0;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) continue;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double t = exp_eta(s[u][e] - wmax, A.ex);
                if constexpr (!FULL) t = cv[u][e] ? t : 0.0;
                acc += t;
            }
        }
        if (__ballot(not_finite(acc)) != 0) {  // an infinite cost in the row: its term is 0 (IEEE limits of exp)
            acc = 0.0;
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                if (!pc.live(u)) continue;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    double t = exp_eta_any(s[u][e] - wmax, A.ex);
                    if constexpr (!FULL) t = cv[u][e] ? t : 0.0;
                    acc += t;
                }
            }
        }
        return acc;
    };

    // (max, sum) pairs wait in LDS until the wave's rows are done, as in the plan pass:
    // entry 4*t + r belongs to row buf_row0 + 16*t + r
    dbl2 *buf = lds_pairs + w * kRowBufPairs;
    dbl2 *part = reinterpret_cast<dbl2 *>(A.rowpart);
    int buffered = 0, buf_row0 = 0;
    auto flush_rows = [&]() {
        for (int e = lane; e < buffered; e += kLanes)
            part[(size_t)p * A.n + buf_row0 + (kRB * kWaves) * (e >> 2) + (e & 3)] = buf[e];
        buffered = 0;
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) {
        const int row0 = r_begin + q * kRB;
        double v[kRB][kU][2];
        load_rows<VEC16, GUARDED, kRB>(Mlane, A.ldM, row0, cv, pc.u_lo, pc.u_hi, v);
        if (buffered == kRowBufPairs) flush_rows();
        if (buffered == 0) buf_row0 = row0;
        double lmax[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) lmax[r] = to_s(v[r]);
        // the maximum of every row is finite: every panel owns at least one column
        const double mx = wave_reduce4<OpMax>(lmax[0], lmax[1], lmax[2], lmax[3]);
        const double wmax[kRB] = {fmax(read_lane(mx, 0), -kDblMax), fmax(read_lane(mx, 32), -kDblMax),
                                  fmax(read_lane(mx, 16), -kDblMax), fmax(read_lane(mx, 48), -kDblMax)};
        double acc[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) acc[r] = sum_exp(v[r], wmax[r]);
        const double sm = wave_reduce4<OpSum>(acc[0], acc[1], acc[2], acc[3]);
        if ((lane & 15) == 0) buf[buffered + quad_row(lane)] = dbl2{mx, sm};
        buffered += kRB;
    }
    flush_rows();
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        const int row = r_begin + ngroups * kRB + t;
        double v[1][kU][2];
        load_rows<VEC16, GUARDED, 1>(Mlane, A.ldM, row, cv, pc.u_lo, pc.u_hi, v);
        const double wmax = fmax(wave_reduce1<OpMax>(to_s(v[0])), -kDblMax);
        const double wsum = wave_reduce1<OpSum>(sum_exp(v[0], wmax));
        if (lane == 0) part[(size_t)p * A.n + row] = dbl2{wmax, wsum};
    }
}

// The narrow last panel by strip workgroups (see plan_pass_strip): the partial log-sum-exp of a row over the panel's
// columns is a reduction over the 16 lanes of a DPP row; the pairs go straight to memory (a strip workgroup's are few).
template <bool ALIGNED>
__device__ __forceinline__ void row_lse_strip(const Stage1Args &A)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const StripLane L(A, lane);
    double bet[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) bet[e] = L.cv[e] ? A.beta[L.first + 2 * L.cp + e] : 0.0;
    dbl2 *part = reinterpret_cast<dbl2 *>(A.rowpart);
    __builtin_amdgcn_s_setprio(3);  // light work beside an older workgroup: go first (see plan_pass_strip)
    for (int g = (int)blockIdx.x - A.wide_blocks; g < A.g_r; g += A.strip_blocks) {
        int r_begin, r_end;
        chunk_rows(g, A.g_r, A.n, r_begin, r_end);
        strip_rows(r_begin, r_end, w, [&](auto nl_tag, int row0) {
            constexpr int NL = decltype(nl_tag)::value;
            double v[NL][2];
            bool live[NL];
            strip_load<ALIGNED, NL>(A, L, row0, r_end, v, live);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int row = row0 + kStripRowsPerLoad * i + L.rsub;
                double sv[2], lmax = -INFINITY;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    sv[e] = bet[e] - v[i][e];
                    if (L.cv[e]) lmax = fmax(lmax, sv[e]);
                }
                // (at least -DBL_MAX, so that a panel of infinite costs gives terms 0 and an empty partial sum)
                const double wmax = fmax(row16_reduce<OpMax>(lmax), -kDblMax);
                double acc = 0.0;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const double t = exp_eta(L.cv[e] ? sv[e] - wmax : 0.0, A.ex);
                    acc += L.cv[e] ? t : 0.0;
                }
                if (__ballot(not_finite(acc)) != 0) {  // an infinite cost in the row: its term is 0 (IEEE limits of exp)
                    acc = 0.0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const double t = exp_eta_any(L.cv[e] ? sv[e] - wmax : 0.0, A.ex);
                        acc += L.cv[e] ? t : 0.0;
                    }
                }
                const double sm = row16_reduce<OpSum>(acc);
                if (L.cp == 0 && live[i]) part[(size_t)L.p * A.n + row] = dbl2{wmax, sm};
            }
        });
    }
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_ROWLSE_WAVES_PER_EU) void row_lse_kernel(Stage1Args A)
{
    __shared__ dbl2 lds_pairs[kWaves * kRowBufPairs];
    static_assert(sizeof(dbl2) * kWaves * kRowBufPairs * REGOT_ROWLSE_WAVES_PER_EU <= 160 * 1024, "LDS per CU");
    if ((int)blockIdx.x >= A.wide_blocks) {
        row_lse_strip<ALIGNED>(A);
        return;
    }
    switch (panel_mode(block_panel(blockIdx.x, A.wide_gc), A.m)) {
    case kPanelFull: row_lse_pass<ALIGNED, kPanelFull>(A, lds_pairs); break;
    case kPanelOverlap: row_lse_pass<ALIGNED, kPanelOverlap>(A, lds_pairs); break;
    case kPanelOverlapEven: row_lse_pass<ALIGNED, kPanelOverlapEven>(A, lds_pairs); break;
    default: row_lse_pass<ALIGNED, kPanelPartial>(A, lds_pairs); break;
    }
}

// which = 1: per column j, over the rows of one chunk, s_ij = alpha_i - M_ij.
// Each lane carries a running (cmax, csum) per owned column; the sum is rescaled
// only in the rare groups of rows where some column's maximum moves.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void col_lse_pass(const Stage1Args &A, double (*lds_max)[kPanel],
                                             double (*lds_sum)[kPanel])
{
    constexpr bool VEC16 = ALIGNED && (MODE == kPanelFull || MODE == kPanelOverlapEven);
    constexpr bool GUARDED = MODE == kPanelPartial;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int g, p;
    block_task(blockIdx.x, A.wide_gc, g, p);
    int r_begin, r_end;
    chunk_rows(g, A.g_r, A.n, r_begin, r_end);

    const PanelCols<MODE> pc(p, A.m, lane);
    const int col0 = pc.col0;
    const bool(&cv)[kU][2] = pc.cv;
    // Running maximum and sum per owned column.  The maximum starts at (and never falls below) -DBL_MAX: a
    // column that has only seen infinite costs then gives s - cmax = -inf, terms 0 and a sum 0, which marks a
    // partial result as empty.
    double cmax[kU][2], csum[kU][2];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            cmax[u][e] = -kDblMax;
            csum[u][e] = 0.0;
        }
    const double *Mlane = A.M + col0 + 2 * lane;

    auto group = [&](auto nr_tag, int row0) {
        constexpr int NR = decltype(nr_tag)::value;
        double v[NR][kU][2];
        load_rows<VEC16, GUARDED, NR>(Mlane, A.ldM, row0, cv, pc.u_lo, pc.u_hi, v);
        double al[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) al[r] = A.alpha[row0 + r];
        bool moved = false;
        double nmax[kU][2];
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double mx = cmax[u][e];
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    v[r][u][e] = al[r] - v[r][u][e];
                    mx = fmax(mx, v[r][u][e]);
                }
                nmax[u][e] = mx;
                moved = moved || (mx != cmax[u][e]);
            }
        if (__ballot(moved) != 0) {
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    csum[u][e] *= exp_eta_any(cmax[u][e] - nmax[u][e], A.ex);  // exactly 1 where unchanged
                    cmax[u][e] = nmax[u][e];
                }
        }
        // the group's terms per column, added up before they join the running sum: a sum that is not finite (an
        // infinite cost among them) is formed again with the IEEE limits of the exponential
        double part[kU][2];
        bool bad = false;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) continue;  // columns of such a group are never written out
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double t = exp_eta(v[0][u][e] - cmax[u][e], A.ex);
#pragma unroll
                for (int r = 1; r < NR; ++r) t += exp_eta(v[r][u][e] - cmax[u][e], A.ex);
                part[u][e] = t;
                bad = bad || not_finite(t);
            }
        }
        if (__ballot(bad) != 0) {
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                if (!pc.live(u)) continue;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    double t = exp_eta_any(v[0][u][e] - cmax[u][e], A.ex);
#pragma unroll
                    for (int r = 1; r < NR; ++r) t += exp_eta_any(v[r][u][e] - cmax[u][e], A.ex);
                    part[u][e] = t;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) continue;
#pragma unroll
            for (int e = 0; e < 2; ++e) csum[u][e] += part[u][e];
        }
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) group(std::integral_constant<int, kRB>{}, r_begin + q * kRB);
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves)
        group(std::integral_constant<int, 1>{}, r_begin + ngroups * kRB + t);

#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            lds_max[w][u * (2 * kLanes) + 2 * lane + e] = cmax[u][e];
            lds_sum[w][u * (2 * kLanes) + 2 * lane + e] = csum[u][e];
        }
    __syncthreads();
    for (int c = threadIdx.x; c < kPanel; c += kThreads) {
        if (!PanelCols<MODE>::owns(c, p, A.m)) continue;
        double mx = 0.0;
        bool any = false;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww)
            if (lds_sum[ww][c] > 0.0) {
                mx = any ? fmax(mx, lds_max[ww][c]) : lds_max[ww][c];
                any = true;
            }
        double sum = 0.0;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww)
            if (lds_sum[ww][c] > 0.0) sum += lds_sum[ww][c] * exp_eta(lds_max[ww][c] - mx, A.ex);
        const size_t k = ((size_t)g * A.m + col0 + c) * 2;
        A.colpart[k] = mx;
        A.colpart[k + 1] = sum;
    }
}

// The narrow last panel by strip workgroups (see plan_pass_strip): a lane carries the running (cmax, csum) of its two
// columns over the rows it sees (every fourth); the 4 x 4 partial results per column (row of the four x wave) are
// merged through LDS as the four waves' results are in col_lse_pass.
template <bool ALIGNED>
__device__ __forceinline__ void col_lse_strip(const Stage1Args &A, double (*lds_max)[kPanel], double (*lds_sum)[kPanel])
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const StripLane L(A, lane);
    __builtin_amdgcn_s_setprio(3);  // light work beside an older workgroup: go first (see plan_pass_strip)
    for (int g = (int)blockIdx.x - A.wide_blocks; g < A.g_r; g += A.strip_blocks) {
        int r_begin, r_end;
        chunk_rows(g, A.g_r, A.n, r_begin, r_end);
        double cmax[2] = {-kDblMax, -kDblMax}, csum[2] = {0.0, 0.0};
        strip_rows(r_begin, r_end, w, [&](auto nl_tag, int row0) {
            constexpr int NL = decltype(nl_tag)::value;
            double v[NL][2];
            bool live[NL];
            strip_load<ALIGNED, NL>(A, L, row0, r_end, v, live);
            double al[NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) al[i] = live[i] ? A.alpha[row0 + kStripRowsPerLoad * i + L.rsub] : 0.0;
            bool moved = false;
            double nmax[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double mx = cmax[e];
#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    v[i][e] = al[i] - v[i][e];
                    if (live[i] && L.cv[e]) mx = fmax(mx, v[i][e]);
                }
                nmax[e] = mx;
                moved = moved || (mx != cmax[e]);
            }
            if (__ballot(moved) != 0) {
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    csum[e] *= exp_eta_any(cmax[e] - nmax[e], A.ex);  // exactly 1 where unchanged
                    cmax[e] = nmax[e];
                }
            }
            double part[2];
            bool bad = false;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double t = 0.0;
#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    const bool on = live[i] && L.cv[e];
                    const double x = exp_eta(on ? v[i][e] - cmax[e] : 0.0, A.ex);
                    t += on ? x : 0.0;
                }
                part[e] = t;
                bad = bad || not_finite(t);
            }
            if (__ballot(bad) != 0) {  // an infinite cost among them: the IEEE limits of the exponential
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    double t = 0.0;
#pragma unroll
                    for (int i = 0; i < NL; ++i) {
                        const bool on = live[i] && L.cv[e];
                        const double x = exp_eta_any(on ? v[i][e] - cmax[e] : 0.0, A.ex);
                        t += on ? x : 0.0;
                    }
                    part[e] = t;
                }
            }
            csum[0] += part[0];
            csum[1] += part[1];
        });
        // entry 2 * lane + e of wave w: row-of-four lane / 16, column 2 * (lane % 16) + e
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            lds_max[w][2 * lane + e] = cmax[e];
            lds_sum[w][2 * lane + e] = csum[e];
        }
        __syncthreads();
        const int c = (int)threadIdx.x;
        if (c < L.ncol) {
            double mx = 0.0;
            bool any = false;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww)
#pragma unroll
                for (int r = 0; r < kStripRowsPerLoad; ++r) {
                    const int k = 2 * (kStripLanes * r) + c;
                    if (lds_sum[ww][k] > 0.0) {
                        mx = any ? fmax(mx, lds_max[ww][k]) : lds_max[ww][k];
                        any = true;
                    }
                }
            double sum = 0.0;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww)
#pragma unroll
                for (int r = 0; r < kStripRowsPerLoad; ++r) {
                    const int k = 2 * (kStripLanes * r) + c;
                    if (lds_sum[ww][k] > 0.0) sum += lds_sum[ww][k] * exp_eta(lds_max[ww][k] - mx, A.ex);
                }
            const size_t k = ((size_t)g * A.m + L.first + c) * 2;
            A.colpart[k] = mx;
            A.colpart[k + 1] = sum;
        }
        __syncthreads();
    }
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_COLLSE_WAVES_PER_EU) void col_lse_kernel(Stage1Args A)
{
    __shared__ double lds_max[kWaves][kPanel];
    __shared__ double lds_sum[kWaves][kPanel];
    if ((int)blockIdx.x >= A.wide_blocks) {
        col_lse_strip<ALIGNED>(A, lds_max, lds_sum);
        return;
    }
    switch (panel_mode(block_panel(blockIdx.x, A.wide_gc), A.m)) {
    case kPanelFull: col_lse_pass<ALIGNED, kPanelFull>(A, lds_max, lds_sum); break;
    case kPanelOverlap: col_lse_pass<ALIGNED, kPanelOverlap>(A, lds_max, lds_sum); break;
    case kPanelOverlapEven: col_lse_pass<ALIGNED, kPanelOverlapEven>(A, lds_max, lds_sum); break;
    default: col_lse_pass<ALIGNED, kPanelPartial>(A, lds_max, lds_sum); break;
    }
}

// Merge the partial (smax, sum) pairs of one row / column and finish the update:
// out = eta*log(marginal) - (smax + eta*log(sum)).
// Pair q of element i sits at part[(i + q*len) * 2].  A workgroup handles 64 elements; each of its
// four waves merges a quarter of the parts (coalesced over the elements), then wave 0 merges the four.
struct LseFinalizeArgs {
    int64_t len;        // n for which = 0, m for which = 1
    int parts;          // g_c for which = 0, g_r for which = 1
    const double *part;
    const double *marginal;
    double eta;
    double *out;
    ExpParams ex;
};

__global__ __launch_bounds__(kThreads) void lse_finalize_kernel(LseFinalizeArgs L)
{
    __shared__ double lds_max[kWaves][kLanes];
    __shared__ double lds_sum[kWaves][kLanes];
    const int l = threadIdx.x & (kLanes - 1), sub = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kLanes + l;
    const bool live = i < L.len;
    const int per = (L.parts + kWaves - 1) / kWaves;
    const int q0 = min(L.parts, sub * per), q1 = min(L.parts, q0 + per);
    const dbl2 *pairs = reinterpret_cast<const dbl2 *>(L.part);
    // an empty partial has sum 0; a non-empty one has sum >= 1 (its maximum contributes exp(0))
    double mx = 0.0, sum = 0.0;
    if (live) {
        bool any = false;
#pragma unroll 4
        for (int q = q0; q < q1; ++q) {
            const dbl2 pr = pairs[(size_t)q * L.len + i];
            if (pr.y > 0.0) {
                mx = any ? fmax(mx, pr.x) : pr.x;
                any = true;
            }
        }
#pragma unroll 4
        for (int q = q0; q < q1; ++q) {
            const dbl2 pr = pairs[(size_t)q * L.len + i];
            if (pr.y > 0.0) sum += pr.y * exp_eta(pr.x - mx, L.ex);
        }
    }
    lds_max[sub][l] = mx;
    lds_sum[sub][l] = sum;
    __syncthreads();
    if (sub != 0 || !live) return;
    bool any = false;
    mx = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
        if (lds_sum[w][l] > 0.0) {
            mx = any ? fmax(mx, lds_max[w][l]) : lds_max[w][l];
            any = true;
        }
    sum = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
        if (lds_sum[w][l] > 0.0) sum += lds_sum[w][l] * exp_eta(lds_max[w][l] - mx, L.ex);
    L.out[i] = L.eta * log(L.marginal[i]) - (mx + L.eta * log(sum));
}

}  // namespace regot

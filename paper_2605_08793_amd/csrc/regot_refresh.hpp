// The pattern refresh in one read of M: top-k threshold (Sec. 3.1) and the fused objective + gradient
// + CSR evaluation (Sec. 4.4) together.
//
// Called one after the other, regot_topk_threshold and regot_dual_eval_sparsify each read M once.  The
// threshold search already starts from a sample that brackets the k-th largest entry; here the fused
// pass itself runs with the lower end of that bracket as its threshold, so what it stages are
// CANDIDATES: every entry that can still be among the k largest (k plus a fraction of a percent of
// all entries).  The k-th largest is then selected among the staged values (radix passes over the
// runs, the machinery of regot_select.hpp), the candidates below it are taken out of the per-segment
// counts, and the usual second stage and scatter build the CSR from the staged records that remain.
// If the sample's bracket cannot be used or did not hold (fewer than k candidates, a pool that
// overflowed) the call says so in info[1] and the caller falls back to the two calls.
#pragma once

#include "regot_kernels.hpp"
#include "regot_select.hpp"

namespace regot {

struct CandParams {
    double t_lo;      // threshold of the candidate pass: exp of the lower end of the bracket; +inf if unusable
    u64 lo_bits;      // its bit pattern, and that of the upper end (all ones: no upper end): the bracket of
    u64 hi_bits;      // the selection among the staged values, whose bit patterns are ordered like the values
    int usable;       // the sample gave a lower end
    int pad;
};

// After the sample kernels: the bracket in the domain of the values.  One workgroup.
__global__ __launch_bounds__(kThreads) void refresh_bracket_kernel(SelectArgs A, CandParams *cp)
{
    __shared__ u64 lds_raw[kBins];
    __shared__ ResolveLds R;
    const SelState st = resolve_entry(A, kIdxBracket, R, lds_raw);
    if (threadIdx.x != 0) return;
    const bool usable = st.use_bracket && !sample_open(st) && st.side[1].need && !st.error;
    CandParams c;
    c.usable = usable ? 1 : 0;
    c.pad = 0;
    // every key of a sample bucket lies between the bucket's bounds; exp is increasing
    const double inf = __longlong_as_double(0x7ff0000000000000ll);
    c.t_lo = usable ? exp_eta_any(value_of(st.side[1].prefix), A.ex) : inf;
    c.lo_bits = (u64)__double_as_longlong(c.t_lo);
    c.hi_bits = ~0ull;
    if (usable && st.side[0].need) {
        const double t_hi = exp_eta_any(value_of(st.side[0].prefix | ~lead_mask(st.sbits)), A.ex);
        if (t_hi == t_hi && t_hi >= c.t_lo) c.hi_bits = (u64)__double_as_longlong(t_hi);
    }
    *cp = c;
}

// The runs of staged records, as the candidate pass left them.
struct RunTable {
    int n;
    const int *header;
    int fixed_runs, max_ranges;
    const PoolRange *ranges;
    const double *pool_val;
    unsigned *pool_packed;

    __device__ __forceinline__ int count() const
    {
        const long long all = (long long)fixed_runs + header[HDR_RANGE_NEXT];
        return (int)(all < max_ranges ? all : max_ranges);
    }
};

// After the candidate pass: what the bracket pass of the threshold search does over M, done over the
// staged values instead.  Counts the values above the bracket, copies the bit patterns of those
// inside it to the key pool (relative to the lower end, stretched over 64 bits) and counts them by
// their leading bits; leaves the record of kernel kIdxBracket, from which the radix steps go on.
// A workgroup takes kCollectRuns runs and keeps their values in registers: it counts, takes its place
// in the pool with ONE addition to the shared counter (thousands of additions to one address would
// queue up for longer than the whole pass takes), and copies.
constexpr int kCollectRuns = 4;                                   // runs per group of kThreads threads
constexpr int kCollectPer = (kRecCap + kThreads - 1) / kThreads;  // records per thread of one run
constexpr int kCollectThreads = 1024;                             // four such groups per workgroup: the fewer workgroups,
constexpr int kCollectWaves = kCollectThreads / kLanes;           // the fewer additions to the shared counters
constexpr int kCollectBlockRuns = kCollectRuns * (kCollectThreads / kThreads);

__global__ __launch_bounds__(kCollectThreads) void refresh_collect_kernel(SelectArgs A, const CandParams *cp, RunTable T)
{
    constexpr int kB = 1 << kBracketBits;
    __shared__ unsigned hist[kB + 1];
    __shared__ unsigned wave_in[kCollectWaves];
    __shared__ u64 block_base;
    clear_next_slot(A, kIdxBracket);
    const CandParams c = *cp;
    const bool usable = c.usable && T.header[HDR_POOL_OVERFLOW] == 0;
    SelState st = start_state(A);
    st.use_bracket = usable ? 1 : 0;
    st.error = usable ? 0 : 1;
    const u64 lo = c.lo_bits, hi = c.hi_bits;
    if (usable) {
        st.act = kActBracket;
        st.lo = lo;
        st.hi = hi;
        const int b = bracket_bits(lo, hi);
        st.width = b < kBracketBits ? b : kBracketBits;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) A.states[kIdxBracket] = st;
    const int n_runs = T.count();
    if (!usable || (int64_t)blockIdx.x * kCollectBlockRuns >= n_runs) return;
    const int group = (int)(threadIdx.x / kThreads), tid = (int)(threadIdx.x % kThreads);
    const int r0 = ((int)blockIdx.x * (kCollectThreads / kThreads) + group) * kCollectRuns;

    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lshift = 64 - bracket_bits(lo, hi);
    const int hshift = 64 - st.width;
    if (threadIdx.x <= kB) hist[threadIdx.x] = 0;
    __syncthreads();
    // all values of the workgroup's runs are requested before the first one is used
    u64 key[kCollectRuns][kCollectPer];
#pragma unroll
    for (int q = 0; q < kCollectRuns; ++q) {
        PoolRange Rg = T.ranges[min(r0 + q, n_runs - 1)];
        if (r0 + q >= n_runs) Rg.count = 0;
#pragma unroll
        for (int j = 0; j < kCollectPer; ++j) {
            const int i = j * kThreads + tid;
            // (a value is never negative: all ones, which no bracket contains, marks "no record")
            key[q][j] = i < Rg.count ? (u64)__double_as_longlong(T.pool_val[(size_t)Rg.start + i]) : ~0ull;
        }
    }
    unsigned n_above = 0, n_in = 0;  // of the wave (the same in all its lanes)
#pragma unroll
    for (int q = 0; q < kCollectRuns; ++q)
#pragma unroll
        for (int j = 0; j < kCollectPer; ++j) {
            const u64 k = key[q][j];
            const bool live = k != ~0ull;
            const bool gt = live && k > hi;
            const bool in = live && k >= lo && !gt;
            n_above += (unsigned)__builtin_popcountll(__ballot(gt));
            if (in) atomicAdd(&hist[(unsigned)(((k - lo) << lshift) >> hshift)], 1u);
            n_in += (unsigned)__builtin_popcountll(__ballot(in));
        }
    if (lane == 0) {
        wave_in[w] = n_in;
        if (n_above != 0) atomicAdd(&hist[kB], n_above);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 total = 0;
        for (int q = 0; q < kCollectWaves; ++q) total += wave_in[q];
        block_base = total != 0 ? atomicAdd(&A.cnt->bracket_fill, total) : 0ull;
        if (hist[kB] != 0) atomicAdd(&A.cnt->above, (u64)hist[kB]);
    }
    if (threadIdx.x < (1u << st.width) && hist[threadIdx.x] != 0)
        atomicAdd(&main_slot(A, kIdxBracket)[threadIdx.x], (u64)hist[threadIdx.x]);
    __syncthreads();
    // the keys inside the bracket go to the pool, each wave behind the waves before it; keys that
    // would not fit are dropped (the counter still says how many there were)
    u64 at = block_base;
    u64 block_total = 0;
    for (int q = 0; q < kCollectWaves; ++q) {
        if (q < w) at += wave_in[q];
        block_total += wave_in[q];
    }
    if (block_base + block_total > (u64)A.pool_cap) return;
#pragma unroll
    for (int q = 0; q < kCollectRuns; ++q)
#pragma unroll
        for (int j = 0; j < kCollectPer; ++j) {
            const u64 k = key[q][j];
            const bool in = k != ~0ull && k >= lo && k <= hi;
            const uint64_t mk = __ballot(in);
            if (in) A.pool[(size_t)at + lanes_below(mk)] = (k - lo) << lshift;
            at += (u64)__builtin_popcountll(mk);
        }
}

// After the selection: candidates below the threshold leave the counts of their (row, panel) segments,
// and the rank of every candidate that stays becomes its rank among those that stay (its segment's
// earlier candidates lie right before it in the run).  One workgroup per run.
__global__ __launch_bounds__(kThreads) void refresh_drop_kernel(RunTable T, const double *delta_dev, int *seg_count)
{
    __shared__ unsigned char stays[kRecCap];
    const double delta = *delta_dev;
    const int n_runs = T.count();
    for (int r = blockIdx.x; r < n_runs; r += gridDim.x) {
        const PoolRange Rg = T.ranges[r];
        const int cnt = min(Rg.count, kRecCap);
        __syncthreads();  // the flags of the previous run are done with
        for (int k = threadIdx.x; k < cnt; k += kThreads) stays[k] = T.pool_val[(size_t)Rg.start + k] >= delta ? 1 : 0;
        __syncthreads();
        for (int k = threadIdx.x; k < cnt; k += kThreads) {
            const unsigned pk = T.pool_packed[(size_t)Rg.start + k];
            if (!stays[k]) {
                const int row = min(Rg.r_begin + (int)(pk >> 18), T.n - 1);
                atomicSub(&seg_count[(size_t)Rg.panel * T.n + row], 1);
            } else {
                const int rank = (int)((pk >> 9) & 511);
                const int before = min(rank, k);  // (rank <= k always: a segment lies inside one run)
                int gone = 0;
                for (int t = 1; t <= before; ++t) gone += stays[k - t] ? 0 : 1;
                if (gone != 0) T.pool_packed[(size_t)Rg.start + k] = (pk & ~(511u << 9)) | ((unsigned)(rank - gone) << 9);
            }
        }
    }
}

}  // namespace regot

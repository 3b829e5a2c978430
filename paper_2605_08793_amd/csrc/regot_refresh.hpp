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

// What the selection among the staged values keeps between its kernels (refresh_collect_kernel,
// refresh_pick_kernel, refresh_finish_kernel); cleared by refresh_bracket_kernel, which runs before the pass.
constexpr int kPickBits = 11;             // leading bits of the bracket keys that the collect kernel histograms (a
                                          // histogram per workgroup in LDS, merged with one atomic per bin and workgroup)
constexpr int kPickBins = 1 << kPickBits;
constexpr int kPickLists = 64;            // the keys of the chosen bin are appended to one of this many lists (additions to
                                          // one counter from hundreds of workgroups would queue up), each of
constexpr int kPickCap = kSmallPool / kPickLists;  // this many places
struct RefreshSel {
    unsigned hist[kPickBins];  // keys inside the bracket by their leading bits (largest keys in the last bin)
    u64 above;                 // staged values above the bracket
    u64 fill;                  // keys inside the bracket (also those that did not fit the pool)
    unsigned small_count[kPickLists];  // keys of the chosen bin in each list (also those beyond kPickCap)
};

// After the sample kernels: the bracket in the domain of the values.  One workgroup.
__global__ __launch_bounds__(kThreads) void refresh_bracket_kernel(SelectArgs A, CandParams *cp, RefreshSel *sel, int *header)
{
    __shared__ u64 lds_raw[kBins];
    __shared__ ResolveLds R;
    for (int i = threadIdx.x; i < kPickBins; i += kThreads) sel->hist[i] = 0u;
    if (threadIdx.x < kPickLists) sel->small_count[threadIdx.x] = 0u;
    if (threadIdx.x == 0) {
        sel->above = 0ull;
        sel->fill = 0ull;
    }
    if (header != nullptr && threadIdx.x < HDR_INTS) header[threadIdx.x] = 0;  // (what init_header_kernel does for the other calls)
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

__global__ __launch_bounds__(kCollectThreads) void refresh_collect_kernel(const CandParams *cp, RunTable T, RefreshSel *sel,
                                                                         u64 *pool, unsigned pool_cap)
{
    __shared__ unsigned hist[kPickBins];
    __shared__ unsigned wave_in[kCollectWaves];
    __shared__ unsigned block_above;
    __shared__ u64 block_base;
    const CandParams c = *cp;
    const bool usable = c.usable && T.header[HDR_POOL_OVERFLOW] == 0;
    const u64 lo = c.lo_bits, hi = c.hi_bits;
    const int n_runs = T.count();
    if (!usable || (int64_t)blockIdx.x * kCollectBlockRuns >= n_runs) return;
    const int group = (int)(threadIdx.x / kThreads), tid = (int)(threadIdx.x % kThreads);
    const int r0 = ((int)blockIdx.x * (kCollectThreads / kThreads) + group) * kCollectRuns;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lshift = 64 - bracket_bits(lo, hi);
    if (threadIdx.x == 0) block_above = 0u;
    for (int i = threadIdx.x; i < kPickBins; i += kCollectThreads) hist[i] = 0u;
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
            if (in) atomicAdd(&hist[(unsigned)(((k - lo) << lshift) >> (64 - kPickBits))], 1u);
            n_in += (unsigned)__builtin_popcountll(__ballot(in));
        }
    if (lane == 0) {
        wave_in[w] = n_in;
        if (n_above != 0) atomicAdd(&block_above, n_above);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 total = 0;
        for (int q = 0; q < kCollectWaves; ++q) total += wave_in[q];
        block_base = total != 0 ? atomicAdd(&sel->fill, total) : 0ull;
        if (block_above != 0) atomicAdd(&sel->above, (u64)block_above);
    }
    for (int i = threadIdx.x; i < kPickBins; i += kCollectThreads)
        if (hist[i] != 0) atomicAdd(&sel->hist[i], hist[i]);
    __syncthreads();
    // the keys inside the bracket go to the pool, each wave behind the waves before it; keys that
    // would not fit are dropped (the counter still says how many there were)
    u64 at = block_base;
    u64 block_total = 0;
    for (int q = 0; q < kCollectWaves; ++q) {
        if (q < w) at += wave_in[q];
        block_total += wave_in[q];
    }
    if (block_base + block_total > (u64)pool_cap) return;
#pragma unroll
    for (int q = 0; q < kCollectRuns; ++q)
#pragma unroll
        for (int j = 0; j < kCollectPer; ++j) {
            const u64 k = key[q][j];
            const bool in = k != ~0ull && k >= lo && k <= hi;
            const uint64_t mk = __ballot(in);
            if (in) pool[(size_t)at + lanes_below(mk)] = (k - lo) << lshift;
            at += (u64)__builtin_popcountll(mk);
        }
}

// Which bin of the histogram holds the k-th largest staged value, and its rank inside that bin.
struct PickedBin {
    int bin;          // -1: the selection cannot be made (see refresh_finish_kernel)
    unsigned rank;    // 1 = the largest key of the bin
    u64 above_bin;    // staged values larger than every key of the bin
};

// every thread of the workgroup calls this; the first wave does the work
__device__ __forceinline__ PickedBin pick_bin(const CandParams &c, const RefreshSel *sel, long long k, unsigned pool_cap,
                                              bool overflow)
{
    __shared__ PickedBin picked;
    constexpr int kPer = kPickBins / kLanes;  // bins per lane, consecutive; lane 0 owns the largest keys
    static_assert(kPickBins % kLanes == 0, "bins per lane");
    const int tid = threadIdx.x;
    if (tid == 0) picked = PickedBin{-1, 0u, 0ull};
    __syncthreads();
    if (tid < kLanes) {
        unsigned h[kPer];
        unsigned long long mine = 0;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            h[j] = sel->hist[kPickBins - 1 - (tid * kPer + j)];
            mine += h[j];
        }
        unsigned long long incl = mine;
#pragma unroll
        for (int d = 1; d < kLanes; d <<= 1) {
            const unsigned long long up = __shfl_up(incl, d, kLanes);
            if (tid >= d) incl += up;
        }
        const u64 above = sel->above, fill = sel->fill;
        const bool ok = c.usable && !overflow && (long long)above < k && (u64)k <= above + fill && fill <= (u64)pool_cap;
        const u64 want = ok ? (u64)k - above : 0ull;  // rank among the keys inside the bracket, 1 = largest
        u64 before = incl - mine;
        if (ok && before < want && want <= incl) {
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                if (want > before && want <= before + h[j])
                    picked = PickedBin{kPickBins - 1 - (tid * kPer + j), (unsigned)(want - before), above + before};
                before += h[j];
            }
        }
    }
    __syncthreads();
    return picked;
}

// After the collect kernel: the keys of the bin that holds the k-th largest value are copied out of the pool.
__global__ __launch_bounds__(kThreads) void refresh_pick_kernel(const CandParams *cp, RunTable T, RefreshSel *sel, const u64 *pool,
                                                                 unsigned pool_cap, long long k, u64 *small)
{
    const PickedBin pk = pick_bin(*cp, sel, k, pool_cap, T.header[HDR_POOL_OVERFLOW] != 0);
    if (pk.bin < 0) return;
    const u64 fill = sel->fill;
    for (u64 i = (u64)blockIdx.x * kThreads + threadIdx.x; i < fill; i += (u64)gridDim.x * kThreads) {
        const u64 key = pool[i];
        if ((int)(key >> (64 - kPickBits)) == pk.bin) {
            const unsigned list = blockIdx.x % kPickLists;
            const unsigned at = atomicAdd(&sel->small_count[list], 1u);
            if (at < (unsigned)kPickCap) small[(size_t)list * kPickCap + at] = key;
        }
    }
}

// One workgroup: the k-th largest staged value from the keys of the chosen bin, by a radix selection over
// them (eight bits per round, histogram in LDS; a few hundred keys in the usual case, any number of equal ones).
//   delta[0] = that value; info[0] = staged values above it, info[1] = equal to it;
//   delta[0] = NaN, info = -1, -1 if the selection cannot be made this way: no usable bracket, a pool that
//   overflowed, a bracket that does not hold the k-th value, or more than kFinishCap keys in the chosen bin
//   (or more than kPickCap of them from the workgroups that share one list).
constexpr int kFinishBits = 8;
constexpr int kFinishCap = 16384;  // keys of the chosen bin the kernel holds in LDS (128 KB)
__global__ __launch_bounds__(kThreads) void refresh_finish_kernel(const CandParams *cp, RunTable T, const RefreshSel *sel,
                                                                  unsigned pool_cap, long long k, const u64 *small,
                                                                  double *delta, int64_t *info)
{
    __shared__ unsigned hist[1 << kFinishBits];
    __shared__ unsigned wave_tot[kWaves];
    __shared__ u64 sh_prefix;
    __shared__ unsigned sh_rank;
    __shared__ u64 sh_greater;
    static_assert((1 << kFinishBits) == kThreads && kThreads % kPickLists == 0, "one thread per bin, some threads per list");
    const int tid = threadIdx.x;
    const CandParams c = *cp;
    const PickedBin pk = pick_bin(c, sel, k, pool_cap, T.header[HDR_POOL_OVERFLOW] != 0);
    // the lists' fills; n = keys of the chosen bin; a list that ran over makes the selection fail
    __shared__ unsigned list_fill[kPickLists], list_at[kPickLists];
    __shared__ u64 keys[kFinishCap];
    __shared__ unsigned sh_n, sh_over;
    if (tid == 0) sh_n = sh_over = 0u;
    __syncthreads();
    if (tid < kPickLists) {
        const unsigned f = sel->small_count[tid];
        list_fill[tid] = f < (unsigned)kPickCap ? f : (unsigned)kPickCap;
        atomicAdd(&sh_n, f);
        if (f > (unsigned)kPickCap) sh_over = 1u;
    }
    __syncthreads();
    const unsigned n = sh_n;
    if (pk.bin < 0 || sh_over != 0u || pk.rank > n || n > (unsigned)kFinishCap) {
        if (tid == 0) {
            delta[0] = __longlong_as_double(0x7ff8000000000000ll);
            info[0] = info[1] = -1;
        }
        return;
    }
    if (tid == 0) {
        sh_prefix = (u64)pk.bin << (64 - kPickBits);
        sh_rank = pk.rank;
        sh_greater = 0ull;
        unsigned run = 0;
        for (int l = 0; l < kPickLists; ++l) {
            list_at[l] = run;
            run += list_fill[l];
        }
    }
    __syncthreads();
    {   // all keys into LDS, four threads per list
        const int list = tid / (kThreads / kPickLists), sub = tid % (kThreads / kPickLists);
        for (unsigned i = sub; i < list_fill[list]; i += kThreads / kPickLists)
            keys[list_at[list] + i] = small[(size_t)list * kPickCap + i];
    }
    unsigned in_bin = n;
    for (int fixed = kPickBits; fixed < 64;) {
        const int w = 64 - fixed < kFinishBits ? 64 - fixed : kFinishBits;
        const int shift = 64 - fixed - w;
        hist[tid] = 0u;
        __syncthreads();
        const u64 prefix = sh_prefix;
        const unsigned rank = sh_rank;
        for (unsigned i = tid; i < n; i += kThreads) {
            const u64 key = keys[i];
            if ((key >> (64 - fixed)) == (prefix >> (64 - fixed))) atomicAdd(&hist[(unsigned)(key >> shift) & ((1u << w) - 1u)], 1u);
        }
        __syncthreads();
        // the bin that holds the rank-th largest: thread t looks at bin t; `larger` = keys in the bins above it
        // (suffix sums: inside the wave by shuffles, across the four waves through LDS)
        const unsigned mine = tid < (1 << w) ? hist[tid] : 0u;
        const int lane = tid & (kLanes - 1), wv = tid >> 6;
        unsigned suffix = mine;
#pragma unroll
        for (int d = 1; d < kLanes; d <<= 1) {
            const unsigned down = __shfl_down(suffix, d, kLanes);
            if (lane + d < kLanes) suffix += down;
        }
        if (lane == 0) wave_tot[wv] = suffix;
        __syncthreads();
        unsigned larger = suffix - mine;
        for (int q = wv + 1; q < kWaves; ++q) larger += wave_tot[q];
        if (tid < (1 << w) && larger < rank && rank <= larger + mine) {
            sh_prefix = prefix | ((u64)tid << shift);
            sh_rank = rank - larger;
            sh_greater += larger;
            hist[0] = mine;  // (read back below as the number of keys that share the bits fixed so far)
        }
        __syncthreads();
        in_bin = hist[0];
        __syncthreads();
        fixed += w;
        if (in_bin == 1 && fixed < 64) {
            // a single key is left with these leading bits (the usual case after two rounds): it is the one
            const u64 pre = sh_prefix;
            __syncthreads();
            for (unsigned i = tid; i < n; i += kThreads)
                if ((keys[i] >> (64 - fixed)) == (pre >> (64 - fixed))) sh_prefix = keys[i];
            __syncthreads();
            break;
        }
    }
    if (tid == 0) {
        const int lshift = 64 - bracket_bits(c.lo_bits, c.hi_bits);
        delta[0] = __longlong_as_double((long long)(c.lo_bits + (sh_prefix >> lshift)));
        info[0] = (int64_t)(pk.above_bin + sh_greater);
        info[1] = (int64_t)in_bin;
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

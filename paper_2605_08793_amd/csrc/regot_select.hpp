// Threshold of the top-k rule (Sec. 3.1): the k-th largest plan entry, found without forming T.
//
// T_ij = exp(s_ij / eta) is increasing in s_ij = (alpha_i + beta_j) - M_ij, so the k-th largest
// T is exp of the k-th largest s and no exponential is needed while searching.  The search is an
// exact most-significant-digit radix selection on an order-preserving 64-bit integer image of s
// (the "key"): a pass over M builds the histogram of one 13-bit digit of all keys that share the
// digits found so far, a one-workgroup step kernel walks the histogram from the top and fixes
// the digit that holds rank k.  As soon as the surviving bucket fits the pool in the workspace,
// the same pass also copies its keys there, and the remaining digits are resolved on the pool
// (a few MB) instead of on M.  Every kernel of the worst case is enqueued up front and decides
// from a small state record in device memory whether it has work, so the host never waits.
#pragma once

#include "regot_kernels.hpp"

namespace regot {

#ifndef REGOT_SELECT_WAVES_PER_EU
#define REGOT_SELECT_WAVES_PER_EU 2
#endif

typedef unsigned long long u64;

constexpr int kDigits = 5;                  // 13 + 13 + 13 + 13 + 12 bits
constexpr int kDigitBits = 13;
constexpr int kBins = 1 << kDigitBits;      // histogram bins (the last digit uses half of them)
constexpr int kKeyBuf = 1024;               // keys a wave stages in LDS before it writes them to the pool
constexpr int kPoolGrid = 256;              // workgroups of a pass over the pool
static_assert(kKeyBuf >= 2 * kPanel, "a wave appends up to one panel row between two checks");

__host__ __device__ constexpr int digit_shift(int d) { return d < kDigits - 1 ? 64 - kDigitBits * (d + 1) : 0; }
__host__ __device__ constexpr int digit_bins(int d) { return d < kDigits - 1 ? kBins : 1 << (64 - kDigitBits * (kDigits - 1)); }
// mask of the digits before digit d
__host__ __device__ constexpr u64 digits_before(int d) { return d == 0 ? 0ull : ~0ull << (64 - kDigitBits * d); }

// Order-preserving map double -> u64: a < b  <=>  key(a) < key(b) for all non-NaN a, b except
// that -0 sorts just below +0 (callers add +0.0 first, which turns -0 into +0).
__device__ __forceinline__ u64 key_of(double s)
{
    const long long b = __double_as_longlong(s);
    return (u64)b ^ ((u64)(b >> 63) | 0x8000000000000000ull);
}
__device__ __forceinline__ double value_of(u64 key)
{
    const u64 b = (key & 0x8000000000000000ull) ? key ^ 0x8000000000000000ull : ~key;
    return __longlong_as_double((long long)b);
}

// The search state.  Only the step kernels write it (one workgroup, between two passes), except
// pool_fill, which the collecting pass advances atomically, and error.
struct SelState {
    u64 prefix;          // digits fixed so far, in place; lower bits zero
    long long k_rem;     // rank of the target among the keys of the current bucket (1 = largest)
    long long above;     // keys larger than every key of the current bucket
    long long bucket;    // keys in the current bucket (= keys sharing the fixed digits)
    int digit;           // next digit to fix; kDigits when the key is complete
    int collected;       // 1 once the pool holds the current bucket
    int error;           // 1 if a count did not add up (cannot happen with finite inputs)
    unsigned pool_fill;  // keys appended to the pool so far
};

struct SelectArgs {
    int n, m;
    int64_t ldM;
    const double *M;
    const double *alpha;
    const double *beta;
    int g_c, g_r;
    long long k;
    SelState *state;
    u64 *ghist;          // [kBins] histogram of the digit being fixed
    u64 *pool;           // [pool_cap] keys of the collected bucket
    unsigned pool_cap;
    // results
    double *delta;       // [1] exp(s_k / eta)
    double *s_k;         // [1] optional
    int64_t *info;       // [2] keys above the k-th, keys equal to it
    ExpParams ex;
};

__global__ void select_init_kernel(SelectArgs A)
{
    for (int i = threadIdx.x; i < kBins; i += blockDim.x) A.ghist[i] = 0;
    if (threadIdx.x == 0) {
        SelState st;
        st.prefix = 0;
        st.k_rem = A.k;
        st.above = 0;
        st.bucket = (long long)A.n * A.m;
        st.digit = 0;
        st.collected = 0;
        st.error = 0;
        st.pool_fill = 0;
        *A.state = st;
    }
}

// add a workgroup's LDS histogram to the global one; most bins are empty
__device__ __forceinline__ void merge_histogram(const unsigned *hist, u64 *ghist, int nbins)
{
    for (int i = threadIdx.x; i < nbins; i += kThreads) {
        const unsigned c = hist[i];
        if (c != 0) atomicAdd(&ghist[i], (u64)c);
    }
}

// One pass over M for digit st.digit: histogram of that digit over the keys that carry the fixed
// digits; if the bucket fits the pool, the same keys are also appended to the pool.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void select_pass(const SelectArgs &A, const SelState &st, unsigned *hist, u64 *stage_all)
{
    constexpr bool FULL = MODE == kPanelFull;
    constexpr bool VEC16 = ALIGNED && (FULL || MODE == kPanelOverlapEven);
    constexpr bool GUARDED = MODE == kPanelPartial;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int g, p;
    block_task(blockIdx.x, A.g_c, g, p);
    int r_begin, r_end;
    chunk_rows(g, A.g_r, A.n, r_begin, r_end);

    const int d = st.digit;
    const bool collect = st.bucket <= (long long)A.pool_cap;
    const u64 prefix = st.prefix;
    const u64 fmask = digits_before(d);
    const int shift = digit_shift(d);
    const unsigned bmask = (unsigned)digit_bins(d) - 1u;

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

    u64 *stage = stage_all + w * kKeyBuf;
    int fill = 0;  // keys waiting in `stage` (wave-uniform)
    auto flush = [&]() {
        if (fill == 0) return;
        unsigned base = 0;
        if (lane == 0) base = atomicAdd(&A.state->pool_fill, (unsigned)fill);
        base = __builtin_amdgcn_readfirstlane(base);
        if ((u64)base + (u64)fill <= (u64)A.pool_cap) {
            for (int i = lane; i < fill; i += kLanes) A.pool[(size_t)base + i] = stage[i];
        } else if (lane == 0) {
            A.state->error = 1;
        }
        fill = 0;
    };

    auto one_row = [&](double al, const double (&v)[kU][2]) {
        if (collect && fill > kKeyBuf - kPanel) flush();
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) continue;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                // the same association as the plan entry; + 0.0 folds -0 into +0
                const double s = ((al + bet[u][e]) - v[u][e]) + 0.0;
                const u64 key = key_of(s);
                bool hit = ((key ^ prefix) & fmask) == 0;
                if constexpr (!FULL) hit = hit && cv[u][e];
                if (hit) atomicAdd(&hist[(unsigned)(key >> shift) & bmask], 1u);
                if (collect) {
                    const uint64_t mk = __ballot(hit);
                    if (mk != 0) {
                        if (hit) stage[fill + lanes_below(mk)] = key;
                        fill += __builtin_popcountll(mk);
                    }
                }
            }
        }
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) {
        const int row0 = r_begin + q * kRB;
        double v[kRB][kU][2];
        load_rows<VEC16, GUARDED, kRB>(Mlane, A.ldM, row0, cv, pc.u_lo, pc.u_hi, v);
        double al[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) al[r] = A.alpha[row0 + r];
#pragma unroll
        for (int r = 0; r < kRB; ++r) one_row(al[r], v[r]);
    }
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        const int row = r_begin + ngroups * kRB + t;
        double v[1][kU][2];
        load_rows<VEC16, GUARDED, 1>(Mlane, A.ldM, row, cv, pc.u_lo, pc.u_hi, v);
        one_row(A.alpha[row], v[0]);
    }
    flush();
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_SELECT_WAVES_PER_EU) void select_pass_kernel(SelectArgs A)
{
    __shared__ unsigned hist[kBins];
    __shared__ u64 stage[kWaves * kKeyBuf];
    static_assert((sizeof(unsigned) * kBins + sizeof(u64) * kWaves * kKeyBuf) * REGOT_SELECT_WAVES_PER_EU <= 160 * 1024,
                  "LDS per CU");
    const SelState st = *A.state;
    // idle once the bucket lives in the pool (later passes read the pool) or the key is complete
    if (st.collected || st.digit >= kDigits) return;
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    __syncthreads();
    switch (panel_mode(block_panel(blockIdx.x, A.g_c), A.m)) {
    case kPanelFull: select_pass<ALIGNED, kPanelFull>(A, st, hist, stage); break;
    case kPanelOverlap: select_pass<ALIGNED, kPanelOverlap>(A, st, hist, stage); break;
    case kPanelOverlapEven: select_pass<ALIGNED, kPanelOverlapEven>(A, st, hist, stage); break;
    default: select_pass<ALIGNED, kPanelPartial>(A, st, hist, stage); break;
    }
    __syncthreads();
    merge_histogram(hist, A.ghist, digit_bins(st.digit));
}

// One pass over the pool for digit st.digit.
__global__ __launch_bounds__(kThreads) void select_pool_kernel(SelectArgs A)
{
    __shared__ unsigned hist[kBins];
    const SelState st = *A.state;
    if (!st.collected || st.digit >= kDigits) return;
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    __syncthreads();
    const unsigned count = st.pool_fill < A.pool_cap ? st.pool_fill : A.pool_cap;
    const u64 prefix = st.prefix;
    const u64 fmask = digits_before(st.digit);
    const int shift = digit_shift(st.digit);
    const unsigned bmask = (unsigned)digit_bins(st.digit) - 1u;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += (size_t)gridDim.x * kThreads) {
        const u64 key = A.pool[i];
        if (((key ^ prefix) & fmask) == 0) atomicAdd(&hist[(unsigned)(key >> shift) & bmask], 1u);
    }
    __syncthreads();
    merge_histogram(hist, A.ghist, digit_bins(st.digit));
}

// Fix one digit: walk the histogram from the top bin down to the bin that holds rank k_rem.
// after_pool tells which kind of pass ran just before (0: over M, 1: over the pool); a step whose
// pass was idle is idle too.  One workgroup of kThreads threads; thread t owns the kPer bins
// below nbins - t*kPer.
__global__ __launch_bounds__(kThreads) void select_step_kernel(SelectArgs A, int after_pool)
{
    constexpr int kPer = kBins / kThreads;
    __shared__ u64 tsum[kThreads];
    __shared__ int found_thread;
    const SelState st = *A.state;
    if (st.digit >= kDigits || (after_pool ? !st.collected : st.collected)) return;
    const int tid = threadIdx.x;
    const int nbins = digit_bins(st.digit);
    // bins in descending order: position q = t*kPer + j  <->  bin nbins-1-q
    u64 c[kPer];
    u64 mine = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int bin = nbins - 1 - (tid * kPer + j);
        c[j] = bin >= 0 ? A.ghist[bin] : 0;
        mine += c[j];
    }
    tsum[tid] = mine;
    if (tid == 0) found_thread = -1;
    __syncthreads();
    // inclusive scan over threads (Hillis-Steele)
    for (int off = 1; off < kThreads; off <<= 1) {
        const u64 add = tid >= off ? tsum[tid - off] : 0;
        __syncthreads();
        tsum[tid] += add;
        __syncthreads();
    }
    const u64 incl = tsum[tid], excl = incl - mine;
    const u64 k_rem = (u64)st.k_rem;
    if (excl < k_rem && k_rem <= incl) found_thread = tid;  // exactly one thread, if the counts add up
    __syncthreads();
    if (tid == found_thread) {
        // first bin (from the top) whose cumulative count reaches k_rem
        u64 run = excl, csel = 0;
        int jsel = kPer - 1;
        bool done = false;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            if (!done) {
                if (run + c[j] >= k_rem) {
                    jsel = j;
                    csel = c[j];
                    done = true;
                } else {
                    run += c[j];
                }
            }
        }
        const int bin = nbins - 1 - (tid * kPer + jsel);
        SelState nx = st;
        nx.prefix = st.prefix | ((u64)bin << digit_shift(st.digit));
        nx.k_rem = (long long)(k_rem - run);
        nx.above = st.above + (long long)run;
        nx.bucket = (long long)csel;
        nx.digit = st.digit + 1;
        // a pass over M whose bucket fitted the pool has filled it
        if (!after_pool && st.bucket <= (long long)A.pool_cap) {
            nx.collected = 1;
            if ((long long)A.state->pool_fill != st.bucket) nx.error = 1;
        }
        nx.error |= A.state->error;
        nx.pool_fill = A.state->pool_fill;
        if (bin < 0 || csel == 0) nx.error = 1;
        *A.state = nx;
    }
    if (found_thread < 0 && tid == 0) {  // the histogram holds fewer than k_rem keys
        A.state->error = 1;
        A.state->digit = kDigits;
    }
    __syncthreads();
    for (int i = tid; i < kBins; i += kThreads) A.ghist[i] = 0;
}

__global__ void select_finish_kernel(SelectArgs A)
{
    if (threadIdx.x != 0) return;
    const SelState st = *A.state;
    const bool ok = st.digit == kDigits && !st.error;
    const double s = ok ? value_of(st.prefix) : __longlong_as_double(0x7ff8000000000000ll);
    A.delta[0] = ok ? exp_eta(s, A.ex) : s;
    if (A.s_k) A.s_k[0] = s;
    A.info[0] = ok ? st.above : -1;
    A.info[1] = ok ? st.bucket : -1;
}

}  // namespace regot

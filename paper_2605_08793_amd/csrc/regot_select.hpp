// Threshold of the top-k rule (Sec. 3.1): the k-th largest plan entry, found without forming T.
//
// T_ij = exp(s_ij / eta) is increasing in s_ij = (alpha_i + beta_j) - M_ij, so the k-th largest
// T is exp of the k-th largest s and no exponential is needed while searching.  s is mapped to an
// order-preserving 64-bit integer (the "key") and the k-th largest key is found exactly:
//
//   sample    One workgroup takes a stratified sample of 65536 entries (gathered by the kernel
//             before it), locates two of its order statistics and so brackets the k-th key: lo <= key_k <= hi with overwhelming
//             probability, with only a fraction of a percent of all keys inside [lo, hi].
//   bracket   One pass over M counts the keys above hi and copies the keys inside [lo, hi] to a
//             pool in the workspace.  If the counts show that the k-th key is in the pool
//             (above < k <= above + pool size, checked exactly), the search continues on the pool.
//   radix     Otherwise (a bracket that missed, ties that overflow the pool, a tiny problem) the
//             search falls back to a most-significant-digit radix selection over M: a pass
//             builds the histogram of one 13-bit digit of all keys that share the digits found
//             so far; once the surviving bucket fits the pool the pass also copies it there.
//   pool      The remaining digits are fixed by histogram passes over the pool (a few MB).
//
// The result never depends on the sample, only the number of passes does.  All kernels of the
// worst case are enqueued up front (15 launches).  Each one starts by working out, from the
// record its predecessor left and from that predecessor's histogram or counters, what state the
// search is in and whether it has anything to do, so the host never waits and no kernel is
// launched just to take a decision.
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
constexpr int kPoolGrid = 512;              // workgroups of a pass over the pool
constexpr int kSmallPool = 1 << 16;         // keys of the second, small pool
constexpr int kHistSlots = 3;               // kernel i fills slot i % 3, reads slot (i-1) % 3, clears slot (i+1) % 3
constexpr int kSampleThreads = 1024;
#ifndef REGOT_SAMPLE_LOG2
#define REGOT_SAMPLE_LOG2 16
#endif
constexpr int kSampleLog2 = REGOT_SAMPLE_LOG2;
constexpr int kSample = 1 << kSampleLog2;   // sampled entries
constexpr int kSampleFew = 4;               // a sample bucket this small is not refined further
constexpr double kBracketZ = 5.0;           // half-width of the bracket in standard deviations of the sample rank
static_assert(kKeyBuf >= 2 * kPanel, "a wave appends up to one panel row between two checks");
static_assert(kSample % kSampleThreads == 0, "sample size");

// position of each launch in the sequence of one call
enum { kIdxGather = 0, kIdxSample = 1, kIdxBracket = 2, kIdxFirstM = 3, kIdxFirstPool = kIdxFirstM + kDigits,
       kIdxFinish = kIdxFirstPool + kDigits, kSelKernels = kIdxFinish + 1 };

__host__ __device__ constexpr int digit_shift(int d) { return d < kDigits - 1 ? 64 - kDigitBits * (d + 1) : 0; }
__host__ __device__ constexpr int digit_bins(int d) { return d < kDigits - 1 ? kBins : 1 << (64 - kDigitBits * (kDigits - 1)); }
// mask of the first nd digits
__host__ __device__ constexpr u64 prefix_mask(int nd)
{
    return nd <= 0 ? 0ull : nd >= kDigits ? ~0ull : ~0ull << (64 - kDigitBits * nd);
}

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
// the key of entry (i, j): the same association as the plan entry; + 0.0 folds -0 into +0
__device__ __forceinline__ u64 entry_key(double al, double be, double mij) { return key_of(((al + be) - mij) + 0.0); }

// Keys inside a bracket [lo, hi] are stored relative to lo and shifted left so that the bracket
// covers the whole 64-bit range: their leading digit then spreads them over all bins, and only
// the digits that can differ need fixing.
__host__ __device__ __forceinline__ int bracket_bits(u64 lo, u64 hi)
{
    const u64 range = hi - lo;
    int b = 1;
    while (b < 64 && (range >> b) != 0) ++b;
    return b;  // range < 2^b
}
__host__ __device__ constexpr int digits_for_bits(int b) { return (b + kDigitBits - 1) / kDigitBits < kDigits ? (b + kDigitBits - 1) / kDigitBits : kDigits; }

enum SelAct { kActIdle = 0, kActSample, kActBracket, kActHistM, kActHistPool };

// State of the search at the entry of one kernel, and what that kernel does about it.
struct SelState {
    u64 prefix;          // digits fixed so far, in place; lower bits zero
    u64 lo, hi;          // the bracket (kernel kIdxBracket)
    long long k_rem;     // rank of the target among the keys of the current bucket (1 = largest)
    long long above;     // keys larger than every key of the current bucket
    long long bucket;    // keys in the current bucket (= keys sharing the fixed digits)
    unsigned pool_count; // keys in the pool the passes read, once collected
    int small_pool;      // the passes read the small pool (a bucket copied out of the large one)
    int digit;           // next digit to fix; digit_end when the key is complete
    int digit_end;       // number of digits to fix (kDigits, fewer for keys taken relative to a bracket)
    int lshift;          // >= 0: pool keys are (key - lo) << lshift, the image of the bracket [lo, hi]
                         // stretched over the 64 bits; -1: plain keys
    int collected;       // the pool holds the current bucket
    int collecting;      // this kernel also copies its bucket to the pool (kActHistM) / the small pool (kActHistPool)
    int use_bracket;     // the sample produced a usable bracket
    int act;             // SelAct of the kernel that owns this record
    int error;           // a count did not add up (cannot happen with finite inputs)
};

struct SelCounters {     // cleared by the sample kernel
    u64 above;               // bracket pass: keys > hi
    unsigned bracket_fill;   // bracket pass: keys inside the bracket (also those that did not fit the pool)
    unsigned radix_fill;     // collecting histogram pass over M: keys appended
    unsigned small_fill;     // collecting histogram pass over the pool: keys appended to the small pool
    unsigned pad;
};

struct SelectArgs {
    int n, m;
    int64_t ldM;
    const double *M;
    const double *alpha;
    const double *beta;
    int g_c, g_r;
    long long k;
    SelState *states;    // [kSelKernels]
    SelCounters *cnt;
    u64 *ghist;          // [kHistSlots][kBins]
    u64 *pool;           // [pool_cap] keys of the bracket / of the collected bucket
    u64 *small_pool;     // [kSmallPool]
    u64 *sample;         // [kSample]
    unsigned pool_cap;
    // results
    double *delta;       // [1] exp(s_k / eta)
    double *s_k;         // [1] optional
    int64_t *info;       // [2] keys above the k-th, keys equal to it
    ExpParams ex;
};

// ---------------------------------------------------------------------------------------------
// block-wide helpers
// ---------------------------------------------------------------------------------------------

// inclusive prefix sum over the threads of a workgroup (NT threads, a multiple of 64)
template <typename T, int NT>
__device__ __forceinline__ T block_inclusive_scan(T v, T *wave_tot /* LDS [NT / 64] */)
{
    const int lane = threadIdx.x & (kLanes - 1), w = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const T up = __shfl_up(v, off, kLanes);
        if (lane >= off) v += up;
    }
    __syncthreads();  // wave_tot may still be read by a previous call
    if (lane == kLanes - 1) wave_tot[w] = v;
    __syncthreads();
    T base = 0;
    for (int q = 0; q < w; ++q) base += wave_tot[q];
    return v + base;
}

struct ResolveLds {
    u64 wave_tot[kThreads / kLanes];
    SelState next;
};

// Fix one digit from a complete histogram: the first bin from the top whose cumulative count
// reaches st.k_rem.  Thread t owns the kPer bins below nbins - t*kPer.  Returns the new state
// to every thread of the workgroup.
__device__ __forceinline__ SelState fix_digit(const SelState &st, const u64 *hist, ResolveLds &L)
{
    constexpr int kPer = kBins / kThreads;
    const int tid = threadIdx.x;
    const int nbins = digit_bins(st.digit);
    u64 c[kPer];
    u64 mine = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int bin = nbins - 1 - (tid * kPer + j);
        c[j] = bin >= 0 ? hist[bin] : 0;
        mine += c[j];
    }
    if (tid == 0) {
        // in case no thread finds the rank: the histogram holds fewer than k_rem keys
        L.next = st;
        L.next.error = 1;
        L.next.digit = st.digit_end;
    }
    const u64 incl = block_inclusive_scan<u64, kThreads>(mine, L.wave_tot);
    const u64 excl = incl - mine;
    const u64 k_rem = (u64)st.k_rem;
    if (excl < k_rem && k_rem <= incl) {  // exactly one thread
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
        if (bin < 0 || csel == 0) nx.error = 1;
        L.next = nx;
    }
    __syncthreads();
    const SelState out = L.next;
    __syncthreads();
    return out;
}

// State at the entry of kernel idx (>= 1), from the record of kernel idx - 1 and what that kernel
// produced.  Every workgroup computes it for itself; all get the same answer.
__device__ __forceinline__ SelState resolve_entry(const SelectArgs &A, int idx, ResolveLds &L)
{
    const SelState prev = A.states[idx - 1];
    SelState cur = prev;
    if (prev.act == kActBracket) {
        const u64 above = A.cnt->above;
        const unsigned fill = A.cnt->bracket_fill;
        if (fill <= A.pool_cap && above < (u64)A.k && (u64)A.k <= above + fill) {
            // the k-th key is in the pool, stored relative to lo
            const int b = bracket_bits(prev.lo, prev.hi);
            cur.prefix = 0;
            cur.digit = 0;
            cur.digit_end = digits_for_bits(b);
            cur.lshift = 64 - b;
            cur.collected = 1;
            cur.pool_count = fill;
            cur.k_rem = A.k - (long long)above;
            cur.above = (long long)above;
            cur.bucket = (long long)fill;
        }
        // otherwise cur is still the untouched start state: the radix passes take over
    } else if (prev.act == kActHistM || prev.act == kActHistPool) {
        cur = fix_digit(prev, A.ghist + (size_t)((idx - 1) % kHistSlots) * kBins, L);
        if (prev.collecting) {
            const unsigned fill = prev.act == kActHistM ? A.cnt->radix_fill : A.cnt->small_fill;
            cur.collected = 1;
            cur.small_pool = prev.act == kActHistPool;
            cur.pool_count = fill;
            if ((long long)fill != prev.bucket) cur.error = 1;
        }
    }
    cur.collecting = 0;
    cur.act = kActIdle;
    return cur;
}

// every kernel clears the histogram slot of its successor
__device__ __forceinline__ void clear_next_slot(const SelectArgs &A, int idx)
{
    u64 *slot = A.ghist + (size_t)((idx + 1) % kHistSlots) * kBins;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kBins; i += gridDim.x * blockDim.x) slot[i] = 0;
}

// add a workgroup's LDS histogram to the global one; most bins are empty
__device__ __forceinline__ void merge_histogram(const unsigned *hist, u64 *ghist, int nbins)
{
    for (int i = threadIdx.x; i < nbins; i += kThreads) {
        const unsigned c = hist[i];
        if (c != 0) atomicAdd(&ghist[i], (u64)c);
    }
}

// ---------------------------------------------------------------------------------------------
// sample: a gather kernel (one entry per thread) and a one-workgroup kernel that brackets the k-th key
// ---------------------------------------------------------------------------------------------

// integer hash of the sample index (multiply / xor-shift rounds): where in its stratum a sample falls
__device__ __forceinline__ unsigned mix32(unsigned x)
{
    x *= 0x9e3779b1u;
    x ^= x >> 15;
    x *= 0x85ebca77u;
    x ^= x >> 13;
    x *= 0xc2b2ae3du;
    return x ^ (x >> 16);
}

// Ranks (1 = largest) of the two sample keys that bracket the k-th of all keys, and whether the
// bracket is worth trying.  The sample rank of the k-th key is close to ks = k * kSample / nm, with
// standard deviation at most sqrt(ks (1 - ks / kSample)).
struct BracketPlan {
    long long r_hi;  // < 1: no upper bound
    long long r_lo;  // > kSample: no lower bound
    bool use;
};
__device__ __forceinline__ BracketPlan bracket_plan(const SelectArgs &A)
{
    const u64 nm = (u64)A.n * (u64)A.m;
    const double ks = (double)A.k * (double)kSample / (double)nm;
    const double sg = sqrt(fmax(ks * (1.0 - ks / (double)kSample), 1.0));
    BracketPlan P;
    P.r_hi = (long long)floor(ks - kBracketZ * sg) - 1;
    P.r_lo = (long long)ceil(ks + kBracketZ * sg) + 1;
    const long long hi_c = P.r_hi < 0 ? 0 : P.r_hi, lo_c = P.r_lo > kSample ? kSample : P.r_lo;
    const double expect = (double)(lo_c - hi_c) / (double)kSample * (double)nm;
    // worth it only when strata are long enough to sample from and the bracket should fit the pool
    P.use = nm >= (u64)16 * kSample && 1.25 * expect <= (double)A.pool_cap;
    return P;
}

__device__ __forceinline__ SelState start_state(const SelectArgs &A)
{
    SelState st;
    st.prefix = 0;
    st.lo = 0;
    st.hi = ~0ull;
    st.k_rem = A.k;
    st.above = 0;
    st.bucket = (long long)A.n * (long long)A.m;
    st.pool_count = 0;
    st.small_pool = 0;
    st.digit = 0;
    st.digit_end = kDigits;
    st.lshift = -1;
    st.collected = 0;
    st.collecting = 0;
    st.use_bracket = 0;
    st.act = kActIdle;
    st.error = 0;
    return st;
}

// First kernel of a call: clears counters and histogram slots, and gathers the sample.  Stratum t =
// entries [t*q, (t+1)*q) in row-major order, q = nm / kSample (the last nm % kSample entries are
// never sampled, which only matters to the quality of the bracket); thread t takes one entry of it.
__global__ __launch_bounds__(kSampleThreads) void select_gather_kernel(SelectArgs A)
{
    const unsigned t = blockIdx.x * kSampleThreads + threadIdx.x;
    for (int i = (int)t; i < kHistSlots * kBins; i += kSample) A.ghist[i] = 0;
    if (t == 0) {
        SelCounters c;
        c.above = 0;
        c.bracket_fill = 0;
        c.radix_fill = 0;
        c.small_fill = 0;
        c.pad = 0;
        *A.cnt = c;
        SelState st = start_state(A);
        st.act = kActSample;
        A.states[kIdxGather] = st;
    }
    if (!bracket_plan(A).use) return;
    const u64 nm = (u64)A.n * (u64)A.m;
    const u64 q = nm >> kSampleLog2;
    // offset inside the stratum: floor(hash * q / 2^32) < q
    const unsigned h = mix32(t);
    const u64 off = (u64)h * (q >> 32) + (((u64)h * (q & 0xffffffffu)) >> 32);
    const u64 pos = (u64)t * q + off;
    // row = pos / m through a double: pos < 2^31 * m, so the estimate is off by at most one
    int i = (int)((double)pos * (1.0 / (double)A.m));
    long long jj = (long long)pos - (long long)i * A.m;
    if (jj < 0) {
        jj += A.m;
        --i;
    } else if (jj >= A.m) {
        jj -= A.m;
        ++i;
    }
    A.sample[t] = entry_key(A.alpha[i], A.beta[jj], A.M[(int64_t)i * A.ldM + jj]);
}

struct SampleLds {
    unsigned hist[2][kBins];
    unsigned wave_tot[kSampleThreads / kLanes];
    int bin[2];
    unsigned run[2], cnt[2];
};

// the bin of L.hist[which] that holds rank k_rem from the top -> L.bin / L.run / L.cnt [which]
__device__ __forceinline__ void sample_fix_digit(SampleLds &L, int which, int nbins, unsigned k_rem)
{
    constexpr int kPer = kBins / kSampleThreads;
    const int tid = threadIdx.x;
    unsigned c[kPer];
    unsigned mine = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int bin = nbins - 1 - (tid * kPer + j);
        c[j] = bin >= 0 ? L.hist[which][bin] : 0u;
        mine += c[j];
    }
    const unsigned incl = block_inclusive_scan<unsigned, kSampleThreads>(mine, L.wave_tot);
    const unsigned excl = incl - mine;
    if (excl < k_rem && k_rem <= incl) {  // exactly one thread
        unsigned run = excl, csel = 0;
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
        L.bin[which] = nbins - 1 - (tid * kPer + jsel);
        L.run[which] = run;
        L.cnt[which] = csel;
    }
    __syncthreads();
}

// Second kernel: one workgroup.  Digit by digit it narrows down the sample keys of ranks r_hi and
// r_lo, until the bucket of each holds only a few sample keys; the bounds of those buckets are the
// bracket.  (Stopping early only widens the bracket by those few sample ranks.)
__global__ __launch_bounds__(kSampleThreads) void select_sample_kernel(SelectArgs A)
{
    __shared__ SampleLds L;
    const int tid = threadIdx.x;
    SelState st = start_state(A);
    st.act = kActSample;
    const BracketPlan P = bracket_plan(A);
    if (P.use) {
        // side 0: the upper end (rank r_hi), side 1: the lower end (rank r_lo)
        const bool need[2] = {P.r_hi >= 1, P.r_lo <= kSample};
        u64 prefix[2] = {0, 0};
        unsigned k_rem[2] = {(unsigned)(need[0] ? P.r_hi : 1), (unsigned)(need[1] ? P.r_lo : 1)};
        unsigned bucket[2] = {kSample, kSample};
        int d = 0;
        for (; d < kDigits; ++d) {
            const bool go0 = need[0] && bucket[0] > kSampleFew, go1 = need[1] && bucket[1] > kSampleFew;
            if (!go0 && !go1) break;
            const int nbins = digit_bins(d);
            const int shift = digit_shift(d);
            const u64 fmask = prefix_mask(d);
            for (int i = tid; i < 2 * kBins; i += kSampleThreads) (&L.hist[0][0])[i] = 0;
            if (tid < 2) {
                L.bin[tid] = 0;
                L.run[tid] = 0;
                L.cnt[tid] = 0;
            }
            __syncthreads();
            // sixteen loads in flight per thread: the sample sits in L2 and the loop is latency-bound
            constexpr int kBatch = 16;
            static_assert(kSample % (kSampleThreads * kBatch) == 0, "sample batches");
            for (int i0 = tid; i0 < kSample; i0 += kSampleThreads * kBatch) {
                u64 key[kBatch];
#pragma unroll
                for (int j = 0; j < kBatch; ++j) key[j] = A.sample[i0 + j * kSampleThreads];
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const unsigned bin = (unsigned)(key[j] >> shift) & (unsigned)(nbins - 1);
                    if (need[0] && ((key[j] ^ prefix[0]) & fmask) == 0) atomicAdd(&L.hist[0][bin], 1u);
                    if (need[1] && ((key[j] ^ prefix[1]) & fmask) == 0) atomicAdd(&L.hist[1][bin], 1u);
                }
            }
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                if (!need[e]) continue;
                sample_fix_digit(L, e, nbins, k_rem[e]);
                prefix[e] |= (u64)(unsigned)L.bin[e] << shift;
                k_rem[e] -= L.run[e];
                bucket[e] = L.cnt[e];
            }
            __syncthreads();
        }
        // d digits are fixed: every key of the bucket lies between these two
        if (need[0]) st.hi = prefix[0] | ~prefix_mask(d);
        if (need[1]) st.lo = prefix[1];
        st.use_bracket = 1;
    }
    if (tid == 0) A.states[kIdxSample] = st;
}

// ---------------------------------------------------------------------------------------------
// passes over M
// ---------------------------------------------------------------------------------------------

// Keys a wave wants to keep go to its LDS buffer first and to the pool in large runs.
struct KeyStage {
    u64 *stage;          // [kKeyBuf] of this wave
    u64 *pool;
    unsigned *fill_ctr;  // global count of keys appended
    unsigned pool_cap;
    int fill;            // keys waiting (wave-uniform)
    int lane;
    __device__ __forceinline__ void flush()
    {
        if (fill == 0) return;
        unsigned base = 0;
        if (lane == 0) base = atomicAdd(fill_ctr, (unsigned)fill);
        base = __builtin_amdgcn_readfirstlane(base);
        // keys beyond the capacity are dropped; the counter still says how many there were
        if ((u64)base + (u64)fill <= (u64)pool_cap)
            for (int i = lane; i < fill; i += kLanes) pool[(size_t)base + i] = stage[i];
        fill = 0;
    }
    // make room for up to `most` more keys
    __device__ __forceinline__ void reserve(int most)
    {
        if (fill > kKeyBuf - most) flush();
    }
    __device__ __forceinline__ void push(bool keep, u64 key)
    {
        const uint64_t mk = __ballot(keep);
        if (mk != 0) {
            if (keep) stage[fill + lanes_below(mk)] = key;
            fill += __builtin_popcountll(mk);
        }
    }
};

// Stream the rows of the workgroup's task and hand every row to `one_row(al, v)`.
template <bool ALIGNED, int MODE, typename RowFn>
__device__ __forceinline__ void stream_task(const SelectArgs &A, const PanelCols<MODE> &pc, int lane, int w,
                                            RowFn &&one_row)
{
    constexpr bool FULL = MODE == kPanelFull;
    constexpr bool VEC16 = ALIGNED && (FULL || MODE == kPanelOverlapEven);
    constexpr bool GUARDED = MODE == kPanelPartial;
    int g, p;
    block_task(blockIdx.x, A.g_c, g, p);
    int r_begin, r_end;
    chunk_rows(g, A.g_r, A.n, r_begin, r_end);
    const double *Mlane = A.M + pc.col0 + 2 * lane;
    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) {
        const int row0 = r_begin + q * kRB;
        double v[kRB][kU][2];
        load_rows<VEC16, GUARDED, kRB>(Mlane, A.ldM, row0, pc.cv, pc.u_lo, pc.u_hi, v);
        double al[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) al[r] = A.alpha[row0 + r];
#pragma unroll
        for (int r = 0; r < kRB; ++r) one_row(al[r], v[r]);
    }
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        const int row = r_begin + ngroups * kRB + t;
        double v[1][kU][2];
        load_rows<VEC16, GUARDED, 1>(Mlane, A.ldM, row, pc.cv, pc.u_lo, pc.u_hi, v);
        one_row(A.alpha[row], v[0]);
    }
}

template <int MODE>
__device__ __forceinline__ void load_beta(const SelectArgs &A, const PanelCols<MODE> &pc, int lane, double (&bet)[kU][2])
{
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = u * (2 * kLanes) + 2 * lane + e;
            bet[u][e] = pc.cv[u][e] ? A.beta[pc.col0 + c] : 0.0;
        }
}

// Histogram of digit st.digit over the keys that carry the fixed digits; with st.collecting the
// same keys are also appended to the pool.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void hist_pass(const SelectArgs &A, const SelState &st, unsigned *hist, u64 *stage_all)
{
    constexpr bool FULL = MODE == kPanelFull;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool collect = st.collecting != 0;
    const u64 prefix = st.prefix;
    const u64 fmask = prefix_mask(st.digit);
    const int shift = digit_shift(st.digit);
    const unsigned bmask = (unsigned)digit_bins(st.digit) - 1u;
    const PanelCols<MODE> pc(block_panel(blockIdx.x, A.g_c), A.m, lane);
    double bet[kU][2];
    load_beta(A, pc, lane, bet);
    KeyStage ks{stage_all + w * kKeyBuf, A.pool, &A.cnt->radix_fill, A.pool_cap, 0, lane};

    stream_task<ALIGNED, MODE>(A, pc, lane, w, [&](double al, const double (&v)[kU][2]) {
        if (collect) ks.reserve(kPanel);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) continue;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const u64 key = entry_key(al, bet[u][e], v[u][e]);
                bool hit = ((key ^ prefix) & fmask) == 0;
                if constexpr (!FULL) hit = hit && pc.cv[u][e];
                if (hit) atomicAdd(&hist[(unsigned)(key >> shift) & bmask], 1u);
                if (collect) ks.push(hit, key);
            }
        }
    });
    ks.flush();
}

// Count the keys above st.hi and copy the keys inside [st.lo, st.hi] to the pool.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void bracket_pass(const SelectArgs &A, const SelState &st, unsigned *block_above,
                                             u64 *stage_all)
{
    constexpr bool FULL = MODE == kPanelFull;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const u64 lo = st.lo, hi = st.hi;
    const int lshift = 64 - bracket_bits(lo, hi);
    const PanelCols<MODE> pc(block_panel(blockIdx.x, A.g_c), A.m, lane);
    double bet[kU][2];
    load_beta(A, pc, lane, bet);
    KeyStage ks{stage_all + w * kKeyBuf, A.pool, &A.cnt->bracket_fill, A.pool_cap, 0, lane};
    unsigned n_above = 0;  // this lane's count; a lane sees at most kMaxChunkRows * 8 entries

    stream_task<ALIGNED, MODE>(A, pc, lane, w, [&](double al, const double (&v)[kU][2]) {
        ks.reserve(kPanel);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (!pc.live(u)) continue;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const u64 key = entry_key(al, bet[u][e], v[u][e]);
                bool gt = key > hi;
                bool in = key >= lo && !gt;
                if constexpr (!FULL) {
                    gt = gt && pc.cv[u][e];
                    in = in && pc.cv[u][e];
                }
                n_above += gt ? 1u : 0u;
                ks.push(in, (key - lo) << lshift);
            }
        }
    });
    ks.flush();
    if (n_above != 0) atomicAdd(block_above, n_above);
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_SELECT_WAVES_PER_EU) void select_pass_kernel(SelectArgs A, int idx)
{
    __shared__ unsigned hist[kBins];
    __shared__ u64 stage[kWaves * kKeyBuf];
    __shared__ ResolveLds R;
    static_assert((sizeof(unsigned) * kBins + sizeof(u64) * kWaves * kKeyBuf + sizeof(ResolveLds)) *
                          REGOT_SELECT_WAVES_PER_EU <= 160 * 1024, "LDS per CU");
    clear_next_slot(A, idx);
    SelState st = resolve_entry(A, idx, R);
    if (!st.error && !st.collected && st.digit < st.digit_end) {
        if (idx == kIdxBracket && st.use_bracket) {
            st.act = kActBracket;
        } else {
            st.act = kActHistM;
            st.collecting = st.bucket <= (long long)A.pool_cap;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) A.states[idx] = st;
    if (st.act == kActIdle) return;

    const int mode = panel_mode(block_panel(blockIdx.x, A.g_c), A.m);
    if (st.act == kActBracket) {
        if (threadIdx.x == 0) hist[0] = 0;  // the workgroup's count of keys above the bracket
        __syncthreads();
        switch (mode) {
        case kPanelFull: bracket_pass<ALIGNED, kPanelFull>(A, st, hist, stage); break;
        case kPanelOverlap: bracket_pass<ALIGNED, kPanelOverlap>(A, st, hist, stage); break;
        case kPanelOverlapEven: bracket_pass<ALIGNED, kPanelOverlapEven>(A, st, hist, stage); break;
        default: bracket_pass<ALIGNED, kPanelPartial>(A, st, hist, stage); break;
        }
        __syncthreads();
        if (threadIdx.x == 0 && hist[0] != 0) atomicAdd(&A.cnt->above, (u64)hist[0]);
        return;
    }
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    __syncthreads();
    switch (mode) {
    case kPanelFull: hist_pass<ALIGNED, kPanelFull>(A, st, hist, stage); break;
    case kPanelOverlap: hist_pass<ALIGNED, kPanelOverlap>(A, st, hist, stage); break;
    case kPanelOverlapEven: hist_pass<ALIGNED, kPanelOverlapEven>(A, st, hist, stage); break;
    default: hist_pass<ALIGNED, kPanelPartial>(A, st, hist, stage); break;
    }
    __syncthreads();
    merge_histogram(hist, A.ghist + (size_t)(idx % kHistSlots) * kBins, digit_bins(st.digit));
}

// One pass over the pool for digit st.digit.  A thread takes two neighbouring keys per step.  When
// the bucket has become small while the pool is large, the pass also copies the bucket to the small
// pool, which the later passes read instead.
__global__ __launch_bounds__(kThreads) void select_pool_kernel(SelectArgs A, int idx)
{
    __shared__ unsigned hist[kBins];
    __shared__ u64 stage[kWaves * kKeyBuf];
    __shared__ ResolveLds R;
    clear_next_slot(A, idx);
    const SelState prev = A.states[idx - 1];
    // the pool never grows: a workgroup whose first key lies beyond it has nothing to do, now or later
    constexpr size_t kStep = 2 * kThreads;
    const size_t first = (size_t)blockIdx.x * kStep;
    if (blockIdx.x > 0 && prev.collected && first >= prev.pool_count) return;
    SelState st = resolve_entry(A, idx, R);
    if (!st.error && st.collected && st.digit < st.digit_end) {
        st.act = kActHistPool;
        st.collecting = !st.small_pool && st.pool_count > (unsigned)kSmallPool && st.bucket <= (long long)kSmallPool;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) A.states[idx] = st;
    if (st.act == kActIdle) return;
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    __syncthreads();
    const size_t cap = st.small_pool ? (size_t)kSmallPool : (size_t)A.pool_cap;
    const size_t count = st.pool_count < cap ? st.pool_count : cap;
    const u64 *src = st.small_pool ? A.small_pool : A.pool;
    const u64 prefix = st.prefix;
    const u64 fmask = prefix_mask(st.digit);
    const int shift = digit_shift(st.digit);
    const unsigned bmask = (unsigned)digit_bins(st.digit) - 1u;
    const bool collect = st.collecting != 0;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    KeyStage ks{stage + w * kKeyBuf, A.small_pool, &A.cnt->small_fill, (unsigned)kSmallPool, 0, lane};
    // two steps (four keys per thread) in flight; the trip count is the same for all threads of the workgroup
    const size_t stride = (size_t)gridDim.x * kStep;
    for (size_t base = first; base < count; base += 2 * stride) {
        u64 key[4] = {0, 0, 0, 0};
        bool hit[4] = {false, false, false, false};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const size_t i = base + h * stride + 2 * threadIdx.x;
            if (i + 1 < count) {
                const ulonglong2 kk = *reinterpret_cast<const ulonglong2 *>(src + i);
                key[2 * h] = kk.x;
                key[2 * h + 1] = kk.y;
                hit[2 * h] = hit[2 * h + 1] = true;
            } else if (i < count) {
                key[2 * h] = src[i];
                hit[2 * h] = true;
            }
        }
        if (collect) ks.reserve(4 * kLanes);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            hit[e] = hit[e] && ((key[e] ^ prefix) & fmask) == 0;
            if (hit[e]) atomicAdd(&hist[(unsigned)(key[e] >> shift) & bmask], 1u);
            if (collect) ks.push(hit[e], key[e]);
        }
    }
    ks.flush();
    __syncthreads();
    merge_histogram(hist, A.ghist + (size_t)(idx % kHistSlots) * kBins, digit_bins(st.digit));
}

__global__ __launch_bounds__(kThreads) void select_finish_kernel(SelectArgs A, int idx)
{
    __shared__ ResolveLds R;
    const SelState st = resolve_entry(A, idx, R);
    if (threadIdx.x != 0) return;
    A.states[idx] = st;
    const bool ok = st.digit == st.digit_end && !st.error;
    const u64 key = st.lshift >= 0 ? st.lo + (st.prefix >> st.lshift) : st.prefix;
    const double s = ok ? value_of(key) : __longlong_as_double(0x7ff8000000000000ll);
    A.delta[0] = ok ? exp_eta(s, A.ex) : s;
    if (A.s_k) A.s_k[0] = s;
    A.info[0] = ok ? st.above : -1;
    A.info[1] = ok ? st.bucket : -1;
}

}  // namespace regot

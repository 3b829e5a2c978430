// Threshold of the top-k rule (Sec. 3.1): the k-th largest plan entry, found without forming T.
//
// T_ij = exp(s_ij / eta) is increasing in s_ij = (alpha_i + beta_j) - M_ij, so the k-th largest
// T is exp of the k-th largest s and no exponential is needed while searching.  s is mapped to an
// order-preserving 64-bit integer (the "key") and the k-th largest key is found exactly:
//
//   sample    A stratified sample of 65536 entries is gathered; two histogram kernels locate two
//             of its order statistics to 26 bits and so bracket the k-th key: lo <= key_k <= hi
//             with overwhelming probability, with a fraction of a percent of all keys in [lo, hi].
//   bracket   One pass over M counts the keys above hi and copies the keys inside [lo, hi] to a
//             pool in the workspace.  If the counts show that the k-th key is in the pool
//             (above < k <= above + pool size, checked exactly), the search continues on the pool.
//   radix     Otherwise (a bracket that missed, ties that overflow the pool, a tiny problem) the
//             search falls back to a most-significant-digit radix selection over M: a pass
//             builds the histogram of the next 13 bits of all keys that share the bits found so
//             far; once the surviving bucket fits the pool the pass also copies it there.
//   pool      The remaining bits are fixed by histogram passes over the pool (a few MB), which
//             move on to a second, small pool as soon as the bucket fits it.
//
// The result never depends on the sample, only the number of passes does.  All kernels of the
// worst case are enqueued up front (10 launches).  Each one starts by working out, from the
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

constexpr int kDigitBits = 13;              // bits fixed per histogram pass
constexpr int kBins = 1 << kDigitBits;
constexpr int kBracketBits = 7;             // leading bits of the bracket keys the bracket pass itself histograms
constexpr int kRadixPasses = (64 + kDigitBits - 1) / kDigitBits;  // radix passes (over M, then over the pool) in the worst case
constexpr int kKeyBuf = 1024;               // keys a wave stages in LDS before it writes them to a pool
constexpr int kSmallPool = 1 << 16;         // keys of the second, small pool
constexpr int kHistSlots = 3;               // kernel i fills slot i % 3, reads slot (i-1) % 3, clears slot (i+1) % 3
constexpr int kSampleSlots = 2;             // two more slots: second sample histogram of either end of the bracket
constexpr int kSampleLog2 = 16;
constexpr int kSample = 1 << kSampleLog2;   // sampled entries
constexpr int kSamplePasses = 2;            // histogram kernels over the sample: its keys are located to 26 bits
constexpr int kSampleFew = 4;               // a sample bucket this small is not refined further
constexpr double kBracketZ = 5.0;           // half-width of the bracket in standard deviations of the sample rank
static_assert((1 << kBracketBits) < kThreads, "one thread per bin of the bracket histogram");
static_assert(kKeyBuf >= 2 * kPanel, "a wave appends up to one panel row between two checks");
static_assert(kSample % (kThreads * 16) == 0, "sample size");
static_assert(kBracketBits + kRadixPasses * kDigitBits >= 64, "the passes after a bracket pass fix all bits");

// position of each launch in the sequence of one call
// (kernel kIdxBracket is the bracket pass or, without a usable sample, the first radix pass; the
// kRadixPasses step kernels after it are radix passes over M or over the pool, whatever the state asks for)
enum { kIdxGather = 0, kIdxFirstSample = 1, kIdxBracket = kIdxFirstSample + kSamplePasses,
       kIdxFinish = kIdxBracket + 1 + kRadixPasses, kSelKernels = kIdxFinish + 1 };

// mask of the leading `bits` bits
__host__ __device__ constexpr u64 lead_mask(int bits) { return bits <= 0 ? 0ull : bits >= 64 ? ~0ull : ~0ull << (64 - bits); }

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
// covers the whole 64-bit range: their leading bits then spread them over all bins, and only
// the bits that can differ need fixing.  Returns b with hi - lo < 2^b.
__host__ __device__ __forceinline__ int bracket_bits(u64 lo, u64 hi)
{
    const u64 range = hi - lo;
    int b = 1;
    while (b < 64 && (range >> b) != 0) ++b;
    return b;
}

enum SelAct { kActIdle = 0, kActGather, kActSampleHist, kActBracket, kActHistM, kActHistPool };

// the search for one of the two sample keys that become the bracket
struct SampleSide {
    u64 prefix;       // leading bits found so far
    unsigned k_rem;   // rank among the sample keys that share them (1 = largest)
    unsigned bucket;  // number of those keys
    int need;         // 0: this end of the bracket is open
    int pad;
};

// State of the search at the entry of one kernel, and what that kernel does about it.
struct SelState {
    u64 prefix;          // leading bits fixed so far, in place; lower bits zero
    u64 lo, hi;          // the bracket (set by kernel kIdxBracket)
    long long k_rem;     // rank of the target among the keys of the current bucket (1 = largest)
    long long above;     // keys larger than every key of the current bucket
    long long bucket;    // keys in the current bucket (= keys sharing the fixed bits)
    SampleSide side[2];  // 0: upper end of the bracket, 1: lower end
    unsigned pool_count; // keys in the pool the passes read, once collected
    int small_pool;      // the passes read the small pool (a bucket copied out of the large one)
    int bits;            // leading bits fixed so far; bits_end when the key is complete
    int bits_end;        // bits to fix in all (64, fewer for keys taken relative to a bracket)
    int width;           // bits the kernel that owns this record fixes: its histogram has 1 << width bins
    int lshift;          // >= 0: pool keys are (key - lo) << lshift, the image of the bracket [lo, hi]
                         // stretched over the 64 bits; -1: plain keys
    int collected;       // the pool holds the current bucket
    int collecting;      // this kernel also copies its bucket to the pool (kActHistM) / the small pool (kActHistPool)
    int use_bracket;     // the bracket is being tried
    int sbits;           // leading bits of the two sample keys fixed so far
    int act;             // SelAct of the kernel that owns this record
    int error;           // a count did not add up (cannot happen with finite inputs)
};

struct SelCounters {     // cleared by the gather kernel
    u64 above;               // bracket pass: keys > hi
    // 64-bit: with more than 2^32 entries and heavy ties a 32-bit count of the keys inside a bracket could wrap
    u64 bracket_fill;        // bracket pass: keys inside the bracket (also those that did not fit the pool)
    u64 radix_fill;          // collecting histogram pass over M: keys appended
    u64 small_fill;          // collecting histogram pass over the pool: keys appended to the small pool
};

struct SelectArgs {
    int n, m;
    int64_t ldM;
    const double *M;
    const double *alpha;
    const double *beta;
    int g_c, g_r;
    int pair_stride;     // > 0: the passes over M keep pace between the workgroups of a compute unit (PaceKeeper)
    int *progress;       // [grid][kWaves]
    long long k;
    SelState *states;    // [kSelKernels]
    SelCounters *cnt;
    u64 *ghist;          // [kHistSlots + kSampleSlots][kBins]
    u64 *pool;           // [pool_cap] keys of the bracket / of the collected bucket
    u64 *small_pool;     // [kSmallPool]
    u64 *sample;         // [kSample]
    unsigned pool_cap;
    int value_domain;    // the keys are bit patterns of values T >= 0 themselves (regot_refresh.hpp): the result is
                         // the key's value, not exp of it, and there is no matrix to fall back to
    // results
    double *delta;       // [1] exp(s_k / eta)
    double *s_k;         // [1] optional
    int64_t *info;       // [2] keys above the k-th, keys equal to it
    ExpParams ex;
};

__device__ __forceinline__ u64 *main_slot(const SelectArgs &A, int idx) { return A.ghist + (size_t)(idx % kHistSlots) * kBins; }
__device__ __forceinline__ u64 *sample_slot(const SelectArgs &A, int e) { return A.ghist + (size_t)(kHistSlots + e) * kBins; }

// ---------------------------------------------------------------------------------------------
// workgroup-wide helpers (kThreads threads)
// ---------------------------------------------------------------------------------------------

// inclusive prefix sum over the threads of the workgroup
__device__ __forceinline__ u64 block_inclusive_scan(u64 v, u64 *wave_tot /* LDS [kWaves] */)
{
    const int lane = threadIdx.x & (kLanes - 1), w = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const u64 up = __shfl_up(v, off, kLanes);
        if (lane >= off) v += up;
    }
    __syncthreads();  // wave_tot may still be read by a previous call
    if (lane == kLanes - 1) wave_tot[w] = v;
    __syncthreads();
    u64 base = 0;
    for (int q = 0; q < w; ++q) base += wave_tot[q];
    return v + base;
}

constexpr int kChunk = 32;                  // bins per chunk in the two-level search of a histogram
constexpr int kChunks = kBins / kChunk;
static_assert(kChunks == kThreads, "one chunk per thread");

struct ResolveLds {
    u64 wave_tot[kWaves];
    u64 wave_fill[kWaves + 1];
    u64 run, cnt;
    int sel, bin;
};

// The bin of a complete histogram that holds rank k_rem counted from the top bin down: `run` keys
// lie in the bins above it, `cnt` in the bin itself.  bin = -1 if the histogram holds fewer than
// k_rem keys.  Every thread gets the result.  The histogram is copied to LDS (coalesced), then two
// levels: sums of chunks of 32 bins, a scan over the chunks from the top, and the bins of the one
// chunk that holds the rank.
struct RankHit {
    int bin;
    u64 run, cnt;
};
__device__ __forceinline__ RankHit find_rank(const u64 *hist, int nbins, u64 k_rem, ResolveLds &L,
                                             u64 *copy /* LDS [kBins] */)
{
    const int tid = threadIdx.x;
    const int lane = tid & (kLanes - 1);
    {
        // all loads of a thread are issued before the first one is used (nbins is a multiple of 2)
        constexpr int kLoads = kBins / (2 * kThreads);
        ulonglong2 v[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int i = 2 * (j * kThreads + tid);
            v[j] = i < nbins ? *reinterpret_cast<const ulonglong2 *>(hist + i) : ulonglong2{0, 0};
        }
#pragma unroll
        for (int j = 0; j < kLoads; ++j) *reinterpret_cast<ulonglong2 *>(copy + 2 * (j * kThreads + tid)) = v[j];
    }
    if (tid == 0) {
        L.sel = -1;
        L.bin = -1;
        L.run = 0;
        L.cnt = 0;
    }
    __syncthreads();
    // thread t sums chunk kChunks-1-t (in a rotated order that keeps the lanes on different banks):
    // a scan over the threads then runs over the chunks from the top
    const u64 *mine_bins = copy + (size_t)(kChunks - 1 - tid) * kChunk;
    u64 mine = 0;
#pragma unroll
    for (int j = 0; j < kChunk; ++j) mine += mine_bins[(j + tid) & (kChunk - 1)];
    const u64 incl = block_inclusive_scan(mine, L.wave_tot);
    const u64 excl = incl - mine;
    if (excl < k_rem && k_rem <= incl) {  // at most one thread
        L.sel = kChunks - 1 - tid;
        L.run = excl;
    }
    __syncthreads();
    const int sel = L.sel;
    if (sel >= 0 && tid < kLanes) {
        // lane l < 32 takes bin 32*sel + 31 - l
        const int bin = sel * kChunk + (kChunk - 1 - (lane & (kChunk - 1)));
        const u64 c = lane < kChunk ? copy[bin] : 0;
        u64 inc = c;
#pragma unroll
        for (int off = 1; off < kChunk; off <<= 1) {
            const u64 up = __shfl_up(inc, off, kLanes);
            if (lane >= off) inc += up;
        }
        const u64 before = L.run + inc - c;
        if (lane < kChunk && before < k_rem && k_rem <= before + c) {  // exactly one lane
            L.bin = bin;
            L.cnt = c;
            L.run = before;
        }
    }
    __syncthreads();
    const RankHit hit{L.bin, L.run, L.cnt};
    __syncthreads();
    return hit;
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
    const BracketPlan P = bracket_plan(A);
    SelState st;
    st.prefix = 0;
    st.lo = 0;
    st.hi = ~0ull;
    st.k_rem = A.k;
    st.above = 0;
    st.bucket = (long long)A.n * (long long)A.m;
    st.side[0] = SampleSide{0, (unsigned)(P.r_hi >= 1 ? P.r_hi : 1), (unsigned)kSample, P.r_hi >= 1 ? 1 : 0, 0};
    st.side[1] = SampleSide{0, (unsigned)(P.r_lo <= kSample ? P.r_lo : 1), (unsigned)kSample, P.r_lo <= kSample ? 1 : 0, 0};
    st.pool_count = 0;
    st.small_pool = 0;
    st.bits = 0;
    st.bits_end = 64;
    st.width = 0;
    st.lshift = -1;
    st.collected = 0;
    st.collecting = 0;
    st.use_bracket = P.use ? 1 : 0;
    st.sbits = 0;
    st.act = kActIdle;
    st.error = 0;
    return st;
}

// does the sample search still have something to narrow down
__device__ __forceinline__ bool sample_open(const SelState &st)
{
    return st.use_bracket && ((st.side[0].need && st.side[0].bucket > (unsigned)kSampleFew) ||
                              (st.side[1].need && st.side[1].bucket > (unsigned)kSampleFew));
}

// State at the entry of kernel idx (>= 1), from the record of kernel idx - 1 and what that kernel
// produced.  Every workgroup computes it for itself; all get the same answer.
__device__ __forceinline__ SelState resolve_entry(const SelectArgs &A, int idx, ResolveLds &L,
                                                  u64 *scratch /* LDS [kBins], free until the kernel's own work starts */)
{
    const SelState prev = A.states[idx - 1];
    SelState cur = prev;
    if (prev.act == kActSampleHist) {
        // the first sample histogram serves both ends, the second has one slot per end
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            if (!prev.side[e].need) continue;
            const u64 *hist = prev.sbits == 0 ? main_slot(A, idx - 1) : sample_slot(A, e);
            const RankHit hit = find_rank(hist, kBins, prev.side[e].k_rem, L, scratch);
            if (hit.bin < 0) {
                cur.use_bracket = 0;  // cannot happen; the radix passes do not need the sample
            } else {
                cur.side[e].prefix = prev.side[e].prefix | ((u64)hit.bin << (64 - prev.sbits - kDigitBits));
                cur.side[e].k_rem = prev.side[e].k_rem - (unsigned)hit.run;
                cur.side[e].bucket = (unsigned)hit.cnt;
            }
        }
        cur.sbits = prev.sbits + kDigitBits;
    } else if (prev.act == kActBracket) {
        const u64 above = A.cnt->above;
        const u64 fill = A.cnt->bracket_fill;
        if (fill <= A.pool_cap && above < (u64)A.k && (u64)A.k <= above + fill) {
            // the k-th key is in the pool, stored relative to lo; the pass has also counted the pool
            // keys by their leading bits
            const int b = bracket_bits(prev.lo, prev.hi);
            const RankHit hit = find_rank(main_slot(A, idx - 1), 1 << prev.width, (u64)A.k - above, L, scratch);
            cur.bits_end = b;
            cur.lshift = 64 - b;
            cur.collected = 1;
            cur.pool_count = (unsigned)fill;
            if (hit.bin < 0 || hit.cnt == 0) {
                cur.error = 1;
            } else {
                cur.prefix = (u64)hit.bin << (64 - prev.width);
                cur.bits = prev.width;
                cur.k_rem = A.k - (long long)above - (long long)hit.run;
                cur.above = (long long)above + (long long)hit.run;
                cur.bucket = (long long)hit.cnt;
            }
        } else if (A.value_domain) {
            cur.error = 1;  // the keys came from staged values: there is no matrix for radix passes to take over
        }
        // otherwise cur is still the untouched start state: the radix passes over M take over
    } else if (prev.act == kActHistM || prev.act == kActHistPool) {
        const RankHit hit = find_rank(main_slot(A, idx - 1), 1 << prev.width, (u64)prev.k_rem, L, scratch);
        if (hit.bin < 0 || hit.cnt == 0) {
            cur.error = 1;
        } else {
            cur.prefix = prev.prefix | ((u64)hit.bin << (64 - prev.bits - prev.width));
            cur.k_rem = prev.k_rem - (long long)hit.run;
            cur.above = prev.above + (long long)hit.run;
            cur.bucket = (long long)hit.cnt;
            cur.bits = prev.bits + prev.width;
        }
        if (prev.collecting) {
            const u64 fill = prev.act == kActHistM ? A.cnt->radix_fill : A.cnt->small_fill;
            cur.collected = 1;
            cur.small_pool = prev.act == kActHistPool;
            cur.pool_count = (unsigned)fill;
            if ((long long)fill != prev.bucket) cur.error = 1;
        }
    }
    cur.collecting = 0;
    cur.width = 0;
    cur.act = kActIdle;
    return cur;
}

// every kernel clears the histogram slot of its successor
__device__ __forceinline__ void clear_next_slot(const SelectArgs &A, int idx)
{
    u64 *slot = main_slot(A, idx + 1);
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
// sample: a gather kernel and histogram kernels, one sampled entry per thread
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

// First kernel of a call: clears counters and histogram slots, and gathers the sample.  Stratum t =
// entries [t*q, (t+1)*q) in row-major order, q = nm / kSample (the last nm % kSample entries are
// never sampled, which only matters to the quality of the bracket); thread t takes one entry of it.
__global__ __launch_bounds__(kThreads) void select_gather_kernel(SelectArgs A)
{
    const unsigned t = blockIdx.x * kThreads + threadIdx.x;
    for (int i = (int)t; i < (kHistSlots + kSampleSlots) * kBins; i += kSample) A.ghist[i] = 0;
    const SelState st0 = start_state(A);
    if (t == 0) {
        SelCounters c;
        c.above = 0;
        c.bracket_fill = 0;
        c.radix_fill = 0;
        c.small_fill = 0;
        *A.cnt = c;
        SelState st = st0;
        st.act = kActGather;
        A.states[kIdxGather] = st;
    }
    if (!st0.use_bracket) return;
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

// Histogram of the next 13 bits of the sample keys that share what is known of either end's key.
// A workgroup takes kSamplePer keys per thread, so that few workgroups add to the global slots.
constexpr int kSamplePer = 16;
constexpr int kSampleGrid = kSample / (kThreads * kSamplePer);
__global__ __launch_bounds__(kThreads) void select_sample_kernel(SelectArgs A, int idx)
{
    __shared__ u64 lds_raw[kBins];  // two histograms of 32-bit counts; before that, scratch of the entry
    __shared__ ResolveLds R;
    unsigned(*hist)[kBins] = reinterpret_cast<unsigned(*)[kBins]>(lds_raw);
    clear_next_slot(A, idx);
    SelState st = resolve_entry(A, idx, R, lds_raw);
    if (sample_open(st)) st.act = kActSampleHist;
    if (blockIdx.x == 0 && threadIdx.x == 0) A.states[idx] = st;
    if (st.act == kActIdle) return;
    const bool first = st.sbits == 0;  // no bits known yet: one histogram serves both ends
    for (int i = threadIdx.x; i < (first ? 1 : 2) * kBins; i += kThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
    u64 key[kSamplePer];
#pragma unroll
    for (int j = 0; j < kSamplePer; ++j) key[j] = A.sample[(blockIdx.x * kSamplePer + j) * kThreads + threadIdx.x];
    const int shift = 64 - st.sbits - kDigitBits;
    const u64 fmask = lead_mask(st.sbits);
#pragma unroll
    for (int j = 0; j < kSamplePer; ++j) {
        const unsigned bin = (unsigned)(key[j] >> shift) & (unsigned)(kBins - 1);
        if (first) {
            atomicAdd(&hist[0][bin], 1u);
        } else {
#pragma unroll
            for (int e = 0; e < 2; ++e)
                if (st.side[e].need && ((key[j] ^ st.side[e].prefix) & fmask) == 0) atomicAdd(&hist[e][bin], 1u);
        }
    }
    __syncthreads();
    if (first) {
        merge_histogram(hist[0], main_slot(A, idx), kBins);
    } else {
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (st.side[e].need) merge_histogram(hist[e], sample_slot(A, e), kBins);
    }
}

// ---------------------------------------------------------------------------------------------
// passes over M
// ---------------------------------------------------------------------------------------------

// Keys a wave wants to keep go to its LDS buffer first and to the pool in large runs.
struct KeyStage {
    u64 *stage;          // [kKeyBuf] of this wave
    u64 *pool;
    u64 *fill_ctr;       // global count of keys appended
    unsigned pool_cap;
    int fill;            // keys waiting (wave-uniform)
    int lane;
    __device__ __forceinline__ void flush()
    {
        if (fill == 0) return;
        u64 base = 0;
        if (lane == 0) base = atomicAdd(fill_ctr, (u64)fill);
        base = ((u64)(unsigned)__builtin_amdgcn_readfirstlane((int)(base >> 32)) << 32) |
               (u64)(unsigned)__builtin_amdgcn_readfirstlane((int)(base & 0xffffffffull));
        // keys beyond the capacity are dropped; the counter still says how many there were
        if ((u64)base + (u64)fill <= (u64)pool_cap)
            for (int i = lane; i < fill; i += kLanes) pool[(size_t)base + i] = stage[i];
        fill = 0;
    }
    // The last flush of every wave of a workgroup as one allocation (a workgroup-wide call): thousands
    // of waves each adding a few keys to one counter would queue up on it.
    __device__ __forceinline__ void flush_workgroup(u64 *wave_fill /* LDS [kWaves + 1] */, int w)
    {
        if (lane == 0) wave_fill[w] = (u64)fill;
        __syncthreads();
        if (threadIdx.x == 0) {
            u64 total = 0;
            for (int q = 0; q < kWaves; ++q) total += wave_fill[q];
            wave_fill[kWaves] = total != 0 ? atomicAdd(fill_ctr, total) : 0ull;
        }
        __syncthreads();
        u64 base = wave_fill[kWaves];
        for (int q = 0; q < w; ++q) base += wave_fill[q];
        if ((u64)base + (u64)fill <= (u64)pool_cap)
            for (int i = lane; i < fill; i += kLanes) pool[(size_t)base + i] = stage[i];
        fill = 0;
        __syncthreads();
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
    PaceKeeper<REGOT_SELECT_WAVES_PER_EU> pace(A.progress, A.pair_stride, w, (int)gridDim.x);
    int it = 0;
    for (int q = w; q < ngroups; q += kWaves, ++it) {
        const int row0 = r_begin + q * kRB;
        pace.tick(it, lane);
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

// Histogram of the next st.width bits over the keys that carry the fixed bits; with st.collecting
// the same keys are also appended to the pool.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void hist_pass(const SelectArgs &A, const SelState &st, unsigned *hist, u64 *stage_all)
{
    constexpr bool FULL = MODE == kPanelFull;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool collect = st.collecting != 0;
    const u64 prefix = st.prefix;
    const u64 fmask = lead_mask(st.bits);
    const int shift = 64 - st.bits - st.width;
    const unsigned bmask = (1u << st.width) - 1u;
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

// Count the keys above st.hi and copy the keys inside [st.lo, st.hi] to the pool, relative to the
// bracket; the copied keys are also counted by their st.width leading bits.
template <bool ALIGNED, int MODE>
__device__ __forceinline__ void bracket_pass(const SelectArgs &A, const SelState &st, unsigned *hist,
                                             unsigned *block_above, u64 *stage_all)
{
    constexpr bool FULL = MODE == kPanelFull;
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const u64 lo = st.lo, hi = st.hi;
    const int lshift = 64 - bracket_bits(lo, hi);
    const int hshift = 64 - st.width;
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
                const u64 rel = (key - lo) << lshift;
                if (in) atomicAdd(&hist[(unsigned)(rel >> hshift)], 1u);
                ks.push(in, rel);
            }
        }
    });
    ks.flush();
    if (n_above != 0) atomicAdd(block_above, n_above);
}

// One pass over the pool for the next st.width bits.  A thread takes two neighbouring keys per step.  When
// the bucket has become small while the pool is large, the pass also copies the bucket to the small
// pool, which the later passes read instead.
__device__ __forceinline__ void pool_pass(const SelectArgs &A, const SelState &st, unsigned *hist, u64 *stage,
                                          ResolveLds &R, int idx)
{
    constexpr size_t kStep = 2 * kThreads;
    const size_t first = (size_t)blockIdx.x * kStep;
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    __syncthreads();
    const size_t cap = st.small_pool ? (size_t)kSmallPool : (size_t)A.pool_cap;
    const size_t count = st.pool_count < cap ? st.pool_count : cap;
    const u64 *src = st.small_pool ? A.small_pool : A.pool;
    const u64 prefix = st.prefix;
    const u64 fmask = lead_mask(st.bits);
    const int shift = 64 - st.bits - st.width;
    const unsigned bmask = (1u << st.width) - 1u;
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
    if (collect) ks.flush_workgroup(R.wave_fill, w);
    __syncthreads();
    merge_histogram(hist, main_slot(A, idx), 1 << st.width);
}

// Kernel kIdxBracket and the radix steps after it.  What a launch does follows from the state it
// finds: the bracket pass (kernel kIdxBracket only), a radix pass over M, a radix pass over the pool
// once the keys that matter have been collected there, or nothing.
template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) REGOT_WAVES_ATTR(REGOT_SELECT_WAVES_PER_EU) void select_step_kernel(SelectArgs A, int idx)
{
    __shared__ u64 lds_raw[kBins];  // histogram of 32-bit counts + key staging; before that, scratch of the entry
    __shared__ ResolveLds R;
    static_assert(sizeof(unsigned) * kBins + sizeof(u64) * kWaves * kKeyBuf <= sizeof(u64) * kBins, "LDS carving");
    static_assert((sizeof(u64) * kBins + sizeof(ResolveLds)) * REGOT_SELECT_WAVES_PER_EU <= 160 * 1024, "LDS per CU");
    unsigned *hist = reinterpret_cast<unsigned *>(lds_raw);
    u64 *stage = lds_raw + kBins / 2;
    clear_next_slot(A, idx);
    {
        // the pool never grows: a workgroup whose first key lies beyond it has nothing to do, now or later
        const SelState prev = A.states[idx - 1];
        if (blockIdx.x > 0 && prev.collected && (size_t)blockIdx.x * (2 * kThreads) >= prev.pool_count) return;
    }
    SelState st = resolve_entry(A, idx, R, lds_raw);
    if (idx == kIdxBracket && sample_open(st)) st.use_bracket = 0;  // 26 bits did not separate the sample keys
    if (!st.error && st.bits < st.bits_end) {
        if (st.collected) {
            st.act = kActHistPool;
            const bool large = !st.small_pool && st.pool_count > (unsigned)kSmallPool;
            st.width = st.bits_end - st.bits < kDigitBits ? st.bits_end - st.bits : kDigitBits;
            st.collecting = large && st.bucket <= (long long)kSmallPool;
        } else if (idx == kIdxBracket && st.use_bracket) {
            // every key of a sample bucket lies between the bucket's bounds
            st.act = kActBracket;
            st.hi = st.side[0].need ? st.side[0].prefix | ~lead_mask(st.sbits) : ~0ull;
            st.lo = st.side[1].need ? st.side[1].prefix : 0ull;
            if (st.lo > st.hi) st.lo = st.hi;  // cannot happen (rank r_lo is below rank r_hi)
            const int b = bracket_bits(st.lo, st.hi);
            st.width = b < kBracketBits ? b : kBracketBits;
        } else {
            st.act = kActHistM;
            st.width = st.bits_end - st.bits < kDigitBits ? st.bits_end - st.bits : kDigitBits;
            st.collecting = st.bucket <= (long long)A.pool_cap;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) A.states[idx] = st;
    if (st.act == kActIdle) return;
    if (st.act == kActHistPool) {
        pool_pass(A, st, hist, stage, R, idx);
        return;
    }

    const int mode = panel_mode(block_panel(blockIdx.x, A.g_c), A.m);
    if (st.act == kActBracket) {
        constexpr int kB = 1 << kBracketBits;  // hist[kB] is the workgroup's count of keys above the bracket
        if (threadIdx.x <= kB) hist[threadIdx.x] = 0;
        __syncthreads();
        switch (mode) {
        case kPanelFull: bracket_pass<ALIGNED, kPanelFull>(A, st, hist, hist + kB, stage); break;
        case kPanelOverlap: bracket_pass<ALIGNED, kPanelOverlap>(A, st, hist, hist + kB, stage); break;
        case kPanelOverlapEven: bracket_pass<ALIGNED, kPanelOverlapEven>(A, st, hist, hist + kB, stage); break;
        default: bracket_pass<ALIGNED, kPanelPartial>(A, st, hist, hist + kB, stage); break;
        }
        __syncthreads();
        if (threadIdx.x == 0 && hist[kB] != 0) atomicAdd(&A.cnt->above, (u64)hist[kB]);
        if (threadIdx.x < (1u << st.width) && hist[threadIdx.x] != 0)
            atomicAdd(&main_slot(A, idx)[threadIdx.x], (u64)hist[threadIdx.x]);
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
    merge_histogram(hist, main_slot(A, idx), 1 << st.width);
}

__global__ __launch_bounds__(kThreads) void select_finish_kernel(SelectArgs A, int idx)
{
    __shared__ u64 lds_raw[kBins];
    __shared__ ResolveLds R;
    const SelState st = resolve_entry(A, idx, R, lds_raw);
    if (threadIdx.x != 0) return;
    A.states[idx] = st;
    const bool ok = st.bits == st.bits_end && !st.error;
    const u64 key = st.lshift >= 0 ? st.lo + (st.prefix >> st.lshift) : st.prefix;
    const double nan = __longlong_as_double(0x7ff8000000000000ll);
    const double s = !ok ? nan : A.value_domain ? __longlong_as_double((long long)key) : value_of(key);
    A.delta[0] = ok && !A.value_domain ? exp_eta_any(s, A.ex) : s;
    if (A.s_k) A.s_k[0] = s;
    A.info[0] = ok ? st.above : -1;
    A.info[1] = ok ? st.bucket : -1;
}

}  // namespace regot

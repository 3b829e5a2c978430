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
    double t_lo;     // threshold of the candidate pass: exp of the lower end of the bracket; +inf if unusable
    int usable;      // the sample gave a lower end
    int pad;
};

// After the sample kernels: the lower end of the bracket as a threshold for the plan pass.  One workgroup.
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
    // every key of the sample bucket at the lower end is >= the bucket's first key
    c.t_lo = usable ? exp_eta(value_of(st.side[1].prefix), A.ex) : __longlong_as_double(0x7ff0000000000000ll);
    *cp = c;
}

// After the candidate pass: the state from which the radix steps select the k-th largest staged value.
// Takes the place of kernel kIdxBracket in the sequence (it also clears the histogram slot of its successor).
__global__ __launch_bounds__(kThreads) void refresh_adopt_kernel(SelectArgs A, const CandParams *cp, int pool_slots)
{
    clear_next_slot(A, kIdxBracket);
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    SelState st = start_state(A);
    const long long used = A.run_header[HDR_SLOT_NEXT];
    const long long records = (used < pool_slots ? used : pool_slots) * (long long)kSlot;  // an upper bound of the candidates
    st.use_bracket = 0;
    st.collected = 1;
    st.small_pool = 0;
    st.pool_count = (unsigned)(records > 0xffffffffll ? 0xffffffffll : records);
    st.bucket = records;
    st.lshift = -1;
    st.act = kActIdle;
    st.error = (!cp->usable || A.run_header[HDR_POOL_OVERFLOW] != 0 || records < A.k) ? 1 : 0;
    A.states[kIdxBracket] = st;
}

// After the selection: candidates below the threshold leave the counts of their (row, panel) segments.
struct DropArgs {
    int n;
    const int *header;
    int fixed_runs, max_ranges;
    const PoolRange *ranges;
    const double *pool_val;
    const unsigned *pool_packed;
    const double *delta_dev;
    int *seg_count;   // [g_c][n]
};

__global__ __launch_bounds__(kThreads) void refresh_drop_kernel(DropArgs D)
{
    const double delta = *D.delta_dev;
    const long long n_runs_all = (long long)D.fixed_runs + D.header[HDR_RANGE_NEXT];
    const int n_runs = (int)(n_runs_all < D.max_ranges ? n_runs_all : D.max_ranges);
    for (int r = blockIdx.x; r < n_runs; r += gridDim.x) {
        const PoolRange R = D.ranges[r];
        for (int k = threadIdx.x; k < R.count; k += kThreads) {
            if (D.pool_val[(size_t)R.start + k] < delta) {
                const int row = min(R.r_begin + (int)(D.pool_packed[(size_t)R.start + k] >> 18), D.n - 1);
                atomicSub(&D.seg_count[(size_t)R.panel * D.n + row], 1);
            }
        }
    }
}

}  // namespace regot

// C ABI of libregot.so: argument checks, workspace layout and kernel launches.
// The interface is documented in include/regot.h.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "regot.h"
#include "exp_poly_coeffs.h"
#include "regot_kernels.hpp"
#include "regot_select.hpp"
#include "regot_refresh.hpp"
#include "regot_sparse.hpp"
#include "regot_pcg.hpp"

using namespace regot;

static_assert(REGOT_EXP_DEGREE == kExpDegree, "regenerate exp_poly_coeffs.h for this degree");

namespace {

constexpr int64_t kMaxDim = 2147483647LL;
constexpr int kNumCU = 256;  // MI355X
constexpr size_t kAlign = 256;

constexpr int cmax(int a, int b) { return a > b ? a : b; }
// A workgroup is one wave per SIMD, so resident workgroups per CU = resident waves per SIMD.
// The plan pass of a sparsify call may run up to kMaxRounds rounds of resident workgroups.
#ifndef REGOT_MAX_ROUNDS
#define REGOT_MAX_ROUNDS 4
#endif
constexpr int kMaxRounds = REGOT_MAX_ROUNDS;
#ifdef REGOT_NO_LSE_STRIP
constexpr bool kLseStrip = false;
#else
constexpr bool kLseStrip = true;   // the half-step passes and the read probe use strip workgroups too
#endif
constexpr int kMaxWavesPerEu =
    cmax(kMaxRounds * REGOT_PLAN_WAVES_PER_EU, cmax(REGOT_ROWLSE_WAVES_PER_EU, REGOT_COLLSE_WAVES_PER_EU));

// How the matrix is cut into (row chunk, column panel) tasks.  Depends on (n, m), on the kernel's
// compiled occupancy and (sparsify calls) on the capacity the caller passes, never on the device the
// call runs on.
struct Geometry {
    int g_c = 0;  // column panels
    int g_r = 0;  // row chunks
    int nblk_rows = 0, nblk_cols = 0;  // finalize workgroups over rows / columns
    int strip_blocks = 0;  // plan pass: > 0 if the narrow last panel is run as a strip by this many workgroups
};

// Row chunks for `panels` panels per chunk on a chip that holds `target` workgroups at once.
int64_t chunks_for(int64_t n, int64_t panels, int64_t target)
{
    int64_t g_r = target / panels;
    const int64_t most = (n + kRB * kWaves - 1) / (kRB * kWaves);
    if (g_r > most) g_r = most;
    // a staged CSR record holds its row relative to the chunk in 14 bits: very tall matrices get more
    // (non-resident) chunks instead.  Chunk boundaries are rounded down to multiples of kRB and the
    // last chunk ends at n, so a chunk can be up to ceil(n / g_r) + kRB - 1 rows tall.
    const int64_t least = (n + (kMaxChunkRows - kRB) - 1) / (kMaxChunkRows - kRB);
    if (g_r < least) g_r = least;
    if (g_r < 1) g_r = 1;
    return g_r;
}

// allow_strip: the plan pass may run a last panel of at most kStripCols columns as a strip beside the
// tasks of the full panels (plan_pass_strip), if that fills the chip better.
Geometry make_geometry(int64_t n, int64_t m, int waves_per_eu, bool allow_strip = false)
{
    Geometry G;
    G.nblk_rows = (int)((n + kFinRows - 1) / kFinRows);
    G.nblk_cols = (int)((m + kLanes - 1) / kLanes);
    if (n == 0 || m == 0) return G;
    G.g_c = (int)((m + kPanel - 1) / kPanel);
    // exactly as many workgroups as the chip holds at once (or fewer): one balanced round
    const int64_t target = (int64_t)kNumCU * waves_per_eu;
    const int64_t ragged = m - (int64_t)(G.g_c - 1) * kPanel;  // columns of the last panel
#ifdef REGOT_NO_STRIP
    allow_strip = false;
#endif
    if (allow_strip && G.g_c >= 2 && ragged <= kStripCols) {
        // Tasks of the full panels fill the chip; the places left over go to strip workgroups.  A task of the
        // narrow panel costs a strip workgroup about a quarter of what a full panel's task costs its
        // workgroup, so each may take up to three.
        const int64_t wide = G.g_c - 1;
        int64_t g_r = chunks_for(n, wide, target);
        if (target - wide * g_r < 1 && g_r > chunks_for(n, wide, 0)) --g_r;  // make room, unless the height bound forbids
        int64_t spare = target - wide * g_r;
        if (spare > g_r) spare = g_r;
        if (spare >= 1 && g_r <= 3 * spare) {
            G.g_r = (int)g_r;
            G.strip_blocks = (int)spare;
            return G;
        }
    }
    G.g_r = (int)chunks_for(n, G.g_c, target);
    return G;
}


// Rounds of resident workgroups the plan pass of a sparsify call runs when it is expected to stage
// `staged` records: one, unless the waves of one round could not keep them on chip (kRecCap each).
int plan_rounds(int64_t staged)
{
    const int64_t per_round = (int64_t)kRecCap * kNumCU * REGOT_PLAN_WAVES_PER_EU * kWaves;
    const int64_t want = (staged + per_round - 1) / per_round;
    return (int)(want < 1 ? 1 : want > kMaxRounds ? kMaxRounds : want);
}

struct Layout {
    size_t header, progress, cu_table, rowpart, colpart, objpart, metric_part;
    size_t seg_count, row_excl, blk_nnz, ranges, pool_val, pool_packed;
    int pool_slots, max_ranges;
    size_t total;
};

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// The layout is the same for every entry point (sized for the kernel with the most row chunks).
Layout make_layout(int64_t n, int64_t m, int64_t capacity)
{
    Geometry G = make_geometry(n, m, kMaxWavesPerEu);
    const Geometry Gs = make_geometry(n, m, kMaxWavesPerEu, true);
    if (Gs.g_r > G.g_r) G.g_r = Gs.g_r;  // a plan pass with a strip cuts the rows into more chunks
    Layout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L.header = take(HDR_INTS * sizeof(int));
    L.progress = take((size_t)kNumCU * kMaxWavesPerEu * kWaves * sizeof(int));
    L.cu_table = take((size_t)kCuKeys * sizeof(CuSlot));
    L.rowpart = take((size_t)2 * G.g_c * (size_t)n * sizeof(double));
    L.colpart = take((size_t)2 * G.g_r * (size_t)m * sizeof(double));
    L.objpart = take((size_t)(G.nblk_rows + G.nblk_cols + 1) * 3 * sizeof(double));
    L.metric_part = take((size_t)kMetricParts * kMetricSums * sizeof(double));
    L.pool_slots = L.max_ranges = 0;
    if (capacity >= 0) {
        // One run per wave when its rows are done, plus one whenever a wave's LDS buffer fills up, which
        // takes more than kRecCap - kPanel records; every run wastes less than one slot.
        const int64_t runs = (int64_t)G.g_r * G.g_c * kWaves + capacity / (kRecCap - kPanel) + 2;
        const int64_t slots = capacity / kSlot + runs + 1;
        L.max_ranges = (int)(runs > kMaxDim ? kMaxDim : runs);
        L.pool_slots = (int)(slots > kMaxDim / kSlot ? kMaxDim / kSlot : slots);
        L.seg_count = take((size_t)G.g_c * (size_t)n * sizeof(int));
        L.row_excl = take((size_t)n * sizeof(int64_t));
        L.blk_nnz = take((size_t)(G.nblk_rows + 1) * sizeof(int64_t));
        L.ranges = take((size_t)L.max_ranges * sizeof(PoolRange));
        L.pool_val = take((size_t)L.pool_slots * kSlot * sizeof(double));
        L.pool_packed = take((size_t)L.pool_slots * kSlot * sizeof(unsigned));
    }
    L.total = off;
    return L;
}

ExpParams make_exp_params(double eta)
{
    ExpParams P;
    const long double e = (long double)eta;
    const long double inv = 1.0L / e;
    P.c1 = (double)(1.442695040888963407359924681001892137L * inv);
    P.l = (double)(e * 0.693147180559945309417232121458176568L);
    long double pw = 1.0L;
    for (int i = 0; i <= kExpDegree; ++i) {
        P.q[i] = (double)(REGOT_EXP_COEF[i] * pw);
        pw *= inv;
    }
    return P;
}

bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

int check_matrix(int64_t n, int64_t m, const double *M, int64_t ldM, double eta, bool allow_empty)
{
    if (n < 0 || m < 0 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!allow_empty && (n == 0 || m == 0)) return REGOT_ERR_DIM;
    if (!(eta > 0.0) || !isfinite(eta)) return REGOT_ERR_ETA;
    if (ldM < m) return REGOT_ERR_LD;
    if (n > 0 && m > 0 && !M) return REGOT_ERR_NULL;
    if (misaligned(M, 8)) return REGOT_ERR_ALIGN;
    return REGOT_OK;
}

int check_workspace(const void *ws, size_t have, size_t need)
{
    if (!ws) return REGOT_ERR_NULL;
    if (misaligned(ws, kAlign)) return REGOT_ERR_ALIGN;
    if (have < need) return REGOT_ERR_WORKSPACE;
    return REGOT_OK;
}

bool aligned16(const double *M, int64_t ldM) { return !misaligned(M, 16) && (ldM % 2 == 0); }

int hip_status()
{
    return hipGetLastError() == hipSuccess ? REGOT_OK : REGOT_ERR_HIP;
}

// one-shot profiling hook (regot_profile_stage1): events recorded around the next streaming kernel
thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

void prof_begin(hipStream_t s)
{
    if (g_prof_start) (void)hipEventRecord(g_prof_start, s);
}

void prof_end(hipStream_t s)
{
    if (g_prof_stop) (void)hipEventRecord(g_prof_stop, s);
    g_prof_start = g_prof_stop = nullptr;
}

template <typename T>
T *at(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }

// Workspace of regot_dual_eval_noalloc: device memory that belongs to the loaded code object, one
// copy per GPU, there from the moment the library is loaded until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress, never an address to pass on: each device's
// address is looked up once (with that device current) and kept in g_scratch_ptr.
constexpr size_t kScratchBytes = (size_t)REGOT_NOALLOC_MAX_WORKSPACE;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// address of the current device's copy of `scratch` (nullptr + status on failure)
int scratch_of_current_device(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return REGOT_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return REGOT_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return REGOT_OK;
}

// What regot_dual_eval_sparsify_topk adds to the fused pass: the pass stages candidates (threshold read
// from the device), the k-th largest staged value is selected, and the scatter keeps what is not below it.
struct RefreshCtx {
    int64_t cand_capacity;     // records the pool is laid out for
    int64_t cand_expected;     // records the candidate pass is expected to stage
    const CandParams *cp;      // device: threshold of the candidate pass
    SelectArgs sel;            // the selection's arguments (its run fields are filled in here)
    unsigned sel_blocks;
    bool sel_aligned;
    int64_t *sel_info;         // device [2]
    RefreshSel *rsel;          // histogram and counters of the selection among the staged values
};

// Argument checks of the plan-pass entry points (everything but the workspace), before any HIP call.
template <bool REDUCE, bool SPARSIFY>
int check_plan_args(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a, const double *b,
                    const double *alpha, const double *beta, double eta, const double *obj, const double *grad_alpha,
                    const double *grad_beta, const double *row_sum, const double *col_sum, double delta,
                    const int64_t *row_ptr, const int32_t *col_idx, const double *val, int64_t capacity,
                    const int64_t *info)
{
    const int st = check_matrix(n, m, M, ldM, eta, true);
    if (st != REGOT_OK) return st;
    if ((n > 0 && !alpha) || (m > 0 && !beta)) return REGOT_ERR_NULL;
    if (misaligned(alpha, 8) || misaligned(beta, 8)) return REGOT_ERR_ALIGN;
    if (REDUCE) {
        if (!obj || (n > 0 && (!a || !grad_alpha)) || (m > 0 && (!b || !grad_beta))) return REGOT_ERR_NULL;
        if (misaligned(a, 8) || misaligned(b, 8) || misaligned(obj, 8) || misaligned(grad_alpha, 8) ||
            misaligned(grad_beta, 8) || misaligned(row_sum, 8) || misaligned(col_sum, 8))
            return REGOT_ERR_ALIGN;
    }
    if (SPARSIFY) {
        if (capacity < 0 || delta != delta) return REGOT_ERR_ARG;
        if (!row_ptr || !info || (capacity > 0 && (!col_idx || !val))) return REGOT_ERR_NULL;
        if (misaligned(row_ptr, 8) || misaligned(info, 8) || misaligned(col_idx, 4) || misaligned(val, 8))
            return REGOT_ERR_ALIGN;
    }
    return REGOT_OK;
}

// Shared implementation of dual_eval / sparsify_csr / dual_eval_sparsify (and, with rc, of the variant
// that finds the threshold itself).
template <bool REDUCE, bool SPARSIFY>
int run_plan_pass(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a, const double *b,
                  const double *alpha, const double *beta, double eta, double *obj, double *grad_alpha,
                  double *grad_beta, double *row_sum, double *col_sum, double delta, int64_t *row_ptr,
                  int32_t *col_idx, double *val, int64_t capacity, int64_t *info, void *workspace,
                  size_t workspace_bytes, regot_stream_t stream, const RefreshCtx *rc = nullptr)
{
    int st = check_plan_args<REDUCE, SPARSIFY>(n, m, M, ldM, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum,
                                               col_sum, delta, row_ptr, col_idx, val, capacity, info);
    if (st != REGOT_OK) return st;
    // One round of resident workgroups, unless the caller expects more entries than the waves of one
    // round can keep on chip (kRecCap each): then as many rounds of lower chunks as it takes (at most
    // kMaxRounds), which keeps most waves from writing their records to HBM in the middle of the pass.
    const int64_t staged = rc ? rc->cand_capacity : capacity;  // records the pass is expected to stage
    int rounds = SPARSIFY ? plan_rounds(staged) : 1;
    // (The pool of a pattern refresh is laid out with a margin of a quarter.  Where that margin alone asks for a second
    // round while the candidates the sample lets one expect exceed what the waves of one round hold by less than a
    // fifth, one round it is: the few waves that fill up write once in mid-stream, which costs less than giving up the
    // resident grid.  20000 x 20000, 0.5 %: 0.68 -> 0.65 ms.  With more rounds the count makes little difference.)
    if (rc && rounds == 2 && plan_rounds(rc->cand_expected - rc->cand_expected / 6) == 1) rounds = 1;
    const Geometry G = make_geometry(n, m, REGOT_PLAN_WAVES_PER_EU * rounds, true);
    const Layout L = make_layout(n, m, SPARSIFY ? staged : -1);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;
    const int64_t tasks = (int64_t)G.g_r * G.g_c;  // (row chunk, panel) pairs; the runs of records are numbered by them
    if (tasks > kMaxDim / kWaves) return REGOT_ERR_DIM;
    const int wide_gc = G.strip_blocks > 0 ? G.g_c - 1 : G.g_c;
    const int64_t nblocks = (int64_t)G.g_r * wide_gc + G.strip_blocks;

    hipStream_t s = static_cast<hipStream_t>(stream);
    int *header = at<int>(workspace, L.header);
    if (SPARSIFY && !rc) hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(HDR_INTS), 0, s, header);  // (rc: refresh_bracket_kernel did it)

    Stage1Args A{};
    A.n = (int)n;
    A.m = (int)m;
    A.ldM = ldM;
    A.M = M;
    A.alpha = alpha;
    A.beta = beta;
    A.g_c = G.g_c;
    A.g_r = G.g_r;
    A.wide_gc = wide_gc;
    A.wide_blocks = G.g_r * wide_gc;
    A.strip_blocks = G.strip_blocks;
#ifndef REGOT_NO_PACE
    // a few workgroups per compute unit, all resident: b, b + kNumCU, ... are neighbours and keep pace
    if (rounds == 1 && nblocks > kNumCU && nblocks <= (int64_t)kNumCU * REGOT_PLAN_WAVES_PER_EU)
        A.pair_stride = kNumCU;
#endif
    A.progress = at<int>(workspace, L.progress);
    A.cu_table = at<int>(workspace, L.cu_table);
    // a grid of several rounds: the workgroups find their neighbours themselves, by hardware id (PaceKeeperHw)
    bool hw_pace = false;
#ifndef REGOT_NO_PACE
    hw_pace = rounds > 1 && nblocks > kNumCU;
#endif
    A.rowpart = at<double>(workspace, L.rowpart);
    A.colpart = at<double>(workspace, L.colpart);
    A.delta = delta;
    A.delta_dev = rc ? &rc->cp->t_lo : nullptr;
    A.header = header;
    if (SPARSIFY) {
        A.seg_count = at<int>(workspace, L.seg_count);
        A.pool_slots = L.pool_slots;
        A.max_ranges = L.max_ranges;
        A.fixed_runs = (int)(tasks * kWaves);
        A.ranges = at<PoolRange>(workspace, L.ranges);
        A.pool_val = at<double>(workspace, L.pool_val);
        A.pool_packed = at<unsigned>(workspace, L.pool_packed);
    }
    A.ex = make_exp_params(eta);
    prof_begin(s);
    if (nblocks > 0) {
        const bool al16 = aligned16(M, ldM);
        auto launch = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3((unsigned)nblocks), dim3(kThreads), 0, s, A); };
        bool done = false;
        if constexpr (REDUCE && SPARSIFY) {
            if (rc) {
                if (hw_pace) al16 ? launch(plan_pass_candidates_kernel<true, true>) : launch(plan_pass_candidates_kernel<false, true>);
                else al16 ? launch(plan_pass_candidates_kernel<true, false>) : launch(plan_pass_candidates_kernel<false, false>);
                done = true;
            }
        }
        if (!done) {
            if (hw_pace) al16 ? launch(plan_pass_kernel<REDUCE, SPARSIFY, true, true>) : launch(plan_pass_kernel<REDUCE, SPARSIFY, false, true>);
            else al16 ? launch(plan_pass_kernel<REDUCE, SPARSIFY, true, false>) : launch(plan_pass_kernel<REDUCE, SPARSIFY, false, false>);
        }
    }
    prof_end(s);

    FinalizeArgs F{};
    F.n = (int)n;
    F.m = (int)m;
    F.g_c = G.g_c;
    F.g_r = G.g_r;
    F.rowpart = A.rowpart;
    F.colpart = A.colpart;
    F.a = a;
    F.b = b;
    F.alpha = alpha;
    F.beta = beta;
    F.eta = eta;
    F.obj = obj;
    F.grad_alpha = grad_alpha;
    F.grad_beta = grad_beta;
    F.row_sum = row_sum;
    F.col_sum = col_sum;
    F.objpart = at<double>(workspace, L.objpart);
    F.nblk_rows = G.nblk_rows;
    F.header = header;
    F.seg_count = A.seg_count;
    F.row_excl = SPARSIFY ? at<int64_t>(workspace, L.row_excl) : nullptr;
    F.blk_nnz = SPARSIFY ? at<int64_t>(workspace, L.blk_nnz) : nullptr;
    F.capacity = capacity;
    F.info = info;
    F.cu_table = hw_pace ? A.cu_table : nullptr;
    int fin_blocks = G.nblk_rows + (REDUCE ? G.nblk_cols : 0);
    if (fin_blocks < 1) fin_blocks = 1;
    if constexpr (REDUCE && SPARSIFY) {
        if (rc) {
            // the k-th largest staged value, then the candidates below it leave the counts
            const SelectArgs &Q = rc->sel;
            RunTable T{};
            T.n = (int)n;
            T.header = header;
            T.fixed_runs = A.fixed_runs;
            T.max_ranges = L.max_ranges;
            T.ranges = A.ranges;
            T.pool_val = A.pool_val;
            T.pool_packed = A.pool_packed;
            int64_t run_blocks = (int64_t)A.fixed_runs + (L.max_ranges - A.fixed_runs < 256 ? L.max_ranges - A.fixed_runs : 256);
            if (run_blocks > 2048) run_blocks = 2048;
            if (run_blocks < 1) run_blocks = 1;
            // (kCollectRuns runs per workgroup: one addition to the pool's counter per workgroup)
            const int64_t collect_blocks = ((int64_t)L.max_ranges + kCollectBlockRuns - 1) / kCollectBlockRuns;
            hipLaunchKernelGGL(refresh_collect_kernel, dim3((unsigned)collect_blocks), dim3(kCollectThreads), 0, s, rc->cp, T, rc->rsel,
                               Q.pool, Q.pool_cap);
            hipLaunchKernelGGL(refresh_pick_kernel, dim3(2 * kNumCU), dim3(kThreads), 0, s, rc->cp, T, rc->rsel, Q.pool, Q.pool_cap,
                               Q.k, Q.small_pool);
            hipLaunchKernelGGL(refresh_finish_kernel, dim3(1), dim3(kThreads), 0, s, rc->cp, T, rc->rsel, Q.pool_cap, Q.k, Q.small_pool,
                               Q.delta, Q.info);
            hipLaunchKernelGGL(refresh_drop_kernel, dim3((unsigned)run_blocks), dim3(kThreads), 0, s, T, Q.delta, A.seg_count);
        }
    }
    hipLaunchKernelGGL((finalize_kernel<REDUCE, SPARSIFY>), dim3(fin_blocks), dim3(kFinThreads), 0, s, F);
    // With few row workgroups the scatter kernel also does the one-workgroup work (scan of the
    // per-workgroup counts, scalars of the call): one launch less on the critical path.
    const bool fold = SPARSIFY && G.nblk_rows <= kFoldBlocks;
    if (!fold) hipLaunchKernelGGL((epilogue_kernel<REDUCE, SPARSIFY>), dim3(1), dim3(kThreads), 0, s, F, fin_blocks);

    if (SPARSIFY) {
        ScatterArgs S{};
        S.n = (int)n;
        S.m = (int)m;
        S.g_c = G.g_c;
        S.g_r = G.g_r;
        S.header = header;
        S.max_ranges = L.max_ranges;
        S.fixed_runs = A.fixed_runs;
        S.ranges = A.ranges;
        S.pool_val = A.pool_val;
        S.pool_packed = A.pool_packed;
        S.seg_rel = A.seg_count;
        S.row_excl = F.row_excl;
        S.capacity = capacity;
        S.blk_off = F.blk_nnz;
        S.nblk = G.nblk_rows;
        S.row_ptr = row_ptr;
        S.info = info;
        S.col_idx = col_idx;
        S.val = val;
        // Workgroups that place records (a multiple of kXcds, at most 4096): one per run with a fixed
        // id, plus room for a quarter as many runs of earlier flushes (the kernel loops if there are more).
        const int64_t fixed_items = scatter_fixed_items(G.g_r, G.g_c);
        int64_t spare = L.max_ranges - A.fixed_runs;
        if (spare > fixed_items / 4 + kXcds) spare = fixed_items / 4 + kXcds;
        int64_t items = (fixed_items + spare + kXcds - 1) / kXcds * kXcds;
        const int grid = (int)(items < 4096 ? items : 4096);
        if (rc) {
            if constexpr (REDUCE) {   // (rc comes with the fused call only)
                S.delta_dev = rc->sel.delta;
                S.select_info = rc->sel_info;
                if (fold)
                    hipLaunchKernelGGL((scatter_kernel<true, true, true>), dim3(grid + 1), dim3(kThreads), 0, s, S, F, fin_blocks);
                else
                    hipLaunchKernelGGL((scatter_kernel<false, false, true>), dim3(grid), dim3(kThreads), 0, s, S, F, fin_blocks);
            }
        } else if (fold)
            hipLaunchKernelGGL((scatter_kernel<true, REDUCE>), dim3(grid + 1), dim3(kThreads), 0, s, S, F, fin_blocks);
        else
            hipLaunchKernelGGL((scatter_kernel<false, false>), dim3(grid), dim3(kThreads), 0, s, S, F, fin_blocks);
    }
    return hip_status();
}

// Workspace of regot_topk_threshold: state records | counters | digit histograms | key pool.
struct SelectLayout {
    size_t states, counters, ghist, sample, small_pool, pool, extra, refresh_sel, progress;
    unsigned pool_cap;
    size_t total;
};

// The pool holds the keys the search narrows down to before it leaves M: the bracket around the
// k-th key (a fraction of k, or a few 1/10000 of all keys when k is small: hence at least n*m/1024), or the bucket that
// survives the first digits.  4k covers both; it never needs more than all n*m keys and is capped
// at 1/16 of the matrix and at 2^28 keys.
SelectLayout make_select_layout(int64_t n, int64_t m, int64_t k)
{
    SelectLayout L{};
    const int64_t nm = n * m;
    int64_t cap = k > (1LL << 26) ? (1LL << 28) : 4 * k;
    if (cap > nm / 16) cap = nm / 16;
    if (cap < nm / 1024) cap = nm / 1024;
    if (cap < 65536) cap = 65536;
    if (cap > nm) cap = nm;
    if (cap > (1LL << 28)) cap = 1LL << 28;
    if (cap < 1) cap = 1;
    L.pool_cap = (unsigned)cap;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L.states = take(sizeof(SelState) * kSelKernels);
    L.counters = take(sizeof(SelCounters));
    L.ghist = take((size_t)(kHistSlots + kSampleSlots) * kBins * sizeof(u64));
    L.sample = take((size_t)kSample * sizeof(u64));
    L.small_pool = take((size_t)kSmallPool * sizeof(u64));
    L.pool = take((size_t)L.pool_cap * sizeof(u64));
    L.extra = take(256);  // regot_dual_eval_sparsify_topk: CandParams | counts of its selection
    L.refresh_sel = take(sizeof(RefreshSel));
    L.progress = take((size_t)kNumCU * REGOT_SELECT_WAVES_PER_EU * kWaves * sizeof(int));
    L.total = off;
    return L;
}

int check_topk_dims(int64_t n, int64_t m, int64_t k)
{
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (k < 1 || k > n * m) return REGOT_ERR_ARG;
    return REGOT_OK;
}

// Workspace of regot_pcg_solve: r | z | p | Ap | partial sums | scalars.
struct PcgLayout {
    size_t x, r, z, p, Ap, part, sc;
    size_t total;
};

// Entries the candidate pass of regot_dual_eval_sparsify_topk is expected to stage, with a margin: all
// entries from the largest down to the lower end of the sample's bracket, whose sample rank is
// ks + 5 sigma + 1 of kSample (ks = k kSample / (n m), sigma^2 = ks (1 - ks / kSample)); the bucket of
// that sample key adds at most a few sample ranks.
int64_t refresh_candidate_capacity(int64_t n, int64_t m, int64_t k)
{
    const double nm = (double)n * (double)m;
    const double ks = (double)k * (double)kSample / nm;
    const double sg = sqrt(fmax(ks * (1.0 - ks / (double)kSample), 1.0));
    double r_lo = ceil(ks + kBracketZ * sg) + 1.0 + 2.0 * kSampleFew;
    if (r_lo > (double)kSample) r_lo = (double)kSample;
    double cap = 1.25 * r_lo / (double)kSample * nm + 65536.0;
    if (cap > nm) cap = nm;
    return (int64_t)cap;
}

// the same without the margin: the number of candidates to expect (at most; the bracket is 5 sigma wide)
int64_t refresh_candidate_expected(int64_t n, int64_t m, int64_t k)
{
    const double nm = (double)n * (double)m;
    const double ks = (double)k * (double)kSample / nm;
    const double sg = sqrt(fmax(ks * (1.0 - ks / (double)kSample), 1.0));
    double r_lo = ceil(ks + kBracketZ * sg) + 1.0;
    if (r_lo > (double)kSample) r_lo = (double)kSample;
    return (int64_t)(r_lo / (double)kSample * nm);
}

// sized for kPcgMaxRhs systems side by side, so one workspace serves regot_pcg_solve and regot_pcg_solve2
PcgLayout make_pcg_layout(int64_t n, int64_t m)
{
    PcgLayout L{};
    const size_t N = (size_t)(n + m - 1);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L.x = take(N * kPcgMaxRhs * sizeof(double));
    L.r = take(N * kPcgMaxRhs * sizeof(double));
    L.z = take(N * kPcgMaxRhs * sizeof(double));
    L.p = take(N * kPcgMaxRhs * sizeof(double));
    L.Ap = take(N * kPcgMaxRhs * sizeof(double));
    // (the partial sums of the combination use the same region)
    L.part = take((size_t)(kCombineDots > kPcgPartRows ? kCombineDots : kPcgPartRows) * kPcgParts * sizeof(double));
    L.sc = take(2 * sizeof(PcgScalars<kPcgMaxRhs>));
    L.total = off;
    return L;
}

// regot_pcg_solve (R = 1) and regot_pcg_solve2 (R = 2)
template <int R>
int run_pcg(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr, const int32_t *col_idx,
            const double *val, const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
            int64_t capacity, const double *row_sum, const double *col_sum, const double *const (&rhs)[R],
            double *const (&x)[R], double rtol, int iterations, int restart, double *info, void *workspace,
            size_t workspace_bytes, regot_stream_t stream)
{
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!(eta > 0.0) || !isfinite(eta)) return REGOT_ERR_ETA;
    if (capacity < 0 || tau != tau || !(rtol >= 0.0) || iterations < 0 || iterations > 100000 ||
        (restart != 0 && restart != 1))
        return REGOT_ERR_ARG;
    if (!row_ptr || !col_ptr || !row_sum || !col_sum || !info) return REGOT_ERR_NULL;
    for (int k = 0; k < R; ++k) {
        if (!rhs[k] || !x[k]) return REGOT_ERR_NULL;
        if (misaligned(rhs[k], 8) || misaligned(x[k], 8)) return REGOT_ERR_ALIGN;
    }
    if (capacity > 0 && (!col_idx || !val || !row_idx || !val_csc)) return REGOT_ERR_NULL;
    if (misaligned(row_ptr, 8) || misaligned(col_ptr, 8) || misaligned(val, 8) || misaligned(val_csc, 8) ||
        misaligned(row_sum, 8) || misaligned(col_sum, 8) || misaligned(info, 8) || misaligned(col_idx, 4) ||
        misaligned(row_idx, 4))
        return REGOT_ERR_ALIGN;
    const PcgLayout L = make_pcg_layout(n, m);
    int st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;

    PcgArgs A{};
    A.mv.n = (int)n;
    A.mv.m = (int)m;
    A.mv.eta = eta;
    A.mv.tau = tau;
    A.mv.row_ptr = row_ptr;
    A.mv.col_idx = col_idx;
    A.mv.val = val;
    A.mv.col_ptr = col_ptr;
    A.mv.row_idx = row_idx;
    A.mv.val_csc = val_csc;
    A.mv.capacity = capacity;
    A.mv.row_sum = row_sum;
    A.mv.col_sum = col_sum;
    A.N = n + m - 1;
    for (int k = 0; k < R; ++k) {
        A.rhs[k] = rhs[k];
        A.x_out[k] = x[k];
    }
    A.x = R == 1 ? x[0] : at<double>(workspace, L.x);  // one system: the caller's array is the iterate
    A.r = at<double>(workspace, L.r);
    A.z = at<double>(workspace, L.z);
    A.p = at<double>(workspace, L.p);
    A.Ap = at<double>(workspace, L.Ap);
    A.mv.x = A.p;
    A.mv.y = A.Ap;
    A.part = at<double>(workspace, L.part);
    A.sc = at<char>(workspace, L.sc);
    A.rtol = rtol;
    A.info = info;
    // product: workgroups for rows and for columns, together at most kPcgParts
    int64_t rb = (n + kWaves - 1) / kWaves, cb = (m - 1 + kWaves - 1) / kWaves;
    // (counted in groups of kWaves waves, whose sums for p^T A p are the partial sums; the product's workgroups
    // hold kMatvecLdsGroup such groups each)
    constexpr int kGroup = kMatvecLdsGroup;
    rb = (rb + kGroup - 1) / kGroup * kGroup;
    cb = (cb + kGroup - 1) / kGroup * kGroup;
    if (rb > kPcgParts / 2) rb = kPcgParts / 2;
    if (cb > kPcgParts / 2) cb = kPcgParts / 2;
    static_assert((kPcgParts / 2) % (kMatvecLdsWaves / kWaves) == 0, "the cap keeps the multiple");
    A.mv.row_waves = rb * kWaves;
    A.mv_blocks = (int)(rb + cb);
    int64_t vb = (A.N + kThreads - 1) / kThreads;
    if (vb > kPcgParts) vb = kPcgParts;
    A.vec_blocks = (int)vb;

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (restart) {
        hipLaunchKernelGGL((pcg_start_kernel<R>), dim3((unsigned)vb), dim3(kThreads), 0, s, A);
        hipLaunchKernelGGL((pcg_start_scalars_kernel<R>), dim3(1), dim3(kThreads), 0, s, A, 0);
    }
    for (int it = 0; it < iterations; ++it) {
        const int *skip = reinterpret_cast<const int *>(at<char>(workspace, L.sc) + (it & 1) * sizeof(PcgScalars<R>) +
                                                        offsetof(PcgScalars<R>, all_done));
        if (n * R <= kMatvecLdsCap && (m - 1) * R <= kMatvecLdsCap)  // both halves of the vector(s) fit the LDS
            hipLaunchKernelGGL((hessian_matvec_lds_kernel<true, R, true>), dim3((unsigned)(A.mv_blocks / kGroup)),
                               dim3(kMatvecLdsThreads), 0, s, A.mv, A.part, (int)kPcgParts, skip, (int)(rb / kGroup));
        else
            hipLaunchKernelGGL((hessian_matvec_lds_kernel<true, R, false>), dim3((unsigned)(A.mv_blocks / kGroup)),
                               dim3(kMatvecLdsThreads), 0, s, A.mv, A.part, (int)kPcgParts, skip, (int)(rb / kGroup));
        hipLaunchKernelGGL((pcg_update_kernel<R>), dim3((unsigned)vb), dim3(kThreads), 0, s, A, it);
        hipLaunchKernelGGL((pcg_direction_kernel<R>), dim3((unsigned)vb), dim3(kThreads), 0, s, A, it);
    }
    hipLaunchKernelGGL((pcg_finish_kernel<R>), dim3(R == 1 ? 1u : (unsigned)vb), dim3(kThreads), 0, s, A, iterations);
    return hip_status();
}

// regot_pcg_solve_reduced (R = 1) and regot_pcg_solve2_reduced (R = 2): conjugate gradients on the Schur
// complement of the first block
template <int R>
int run_pcg_reduced(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr, const int32_t *col_idx,
                    const double *val, const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                    int64_t capacity, const double *row_sum, const double *col_sum, const double *const (&rhs)[R],
                    double *const (&x)[R], double rtol, int iterations, int restart, double *info, void *workspace,
                    size_t workspace_bytes, regot_stream_t stream)
{
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!(eta > 0.0) || !isfinite(eta)) return REGOT_ERR_ETA;
    if (capacity < 0 || tau != tau || !(rtol >= 0.0) || iterations < 0 || iterations > 100000 ||
        (restart != 0 && restart != 1))
        return REGOT_ERR_ARG;
    if (!row_ptr || !col_ptr || !row_sum || !col_sum || !info) return REGOT_ERR_NULL;
    for (int k = 0; k < R; ++k) {
        if (!rhs[k] || !x[k]) return REGOT_ERR_NULL;
        if (misaligned(rhs[k], 8) || misaligned(x[k], 8)) return REGOT_ERR_ALIGN;
    }
    if (capacity > 0 && (!col_idx || !val || !row_idx || !val_csc)) return REGOT_ERR_NULL;
    if (misaligned(row_ptr, 8) || misaligned(col_ptr, 8) || misaligned(val, 8) || misaligned(val_csc, 8) ||
        misaligned(row_sum, 8) || misaligned(col_sum, 8) || misaligned(info, 8) || misaligned(col_idx, 4) ||
        misaligned(row_idx, 4))
        return REGOT_ERR_ALIGN;
    const PcgLayout L = make_pcg_layout(n, m);
    const int st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;

    const int64_t mb = m - 1, N = n + mb;
    SchurArgs<R> S{};
    S.mv.n = (int)n;
    S.mv.m = (int)m;
    S.mv.eta = eta;
    S.mv.tau = tau;
    S.mv.row_ptr = row_ptr;
    S.mv.col_idx = col_idx;
    S.mv.val = val;
    S.mv.col_ptr = col_ptr;
    S.mv.row_idx = row_idx;
    S.mv.val_csc = val_csc;
    S.mv.capacity = capacity;
    S.mv.row_sum = row_sum;
    S.mv.col_sum = col_sum;
    // the vector kernels see the second block alone: systems of m - 1 unknowns whose diagonal is D2
    // (their diagonal is "row sums of the first mv.n entries, column sums after them": mv.n = 0)
    PcgArgs V{};
    V.mv = S.mv;
    V.mv.n = 0;
    V.N = mb;
    // the regions of the workspace hold R = 2 vectors of n + m - 1 entries each: the iterate of a pair (m - 1 entries
    // per system) and u (n per system) share the first; the right-hand sides of the reduced systems (plain arrays)
    // use the region of S p, which is not written before the first iteration
    double *u = at<double>(workspace, L.x) + (R == 1 ? 0 : (size_t)kPcgMaxRhs * mb);
    for (int k = 0; k < R; ++k) {
        V.rhs[k] = at<double>(workspace, L.Ap) + (size_t)k * mb;
        V.x_out[k] = x[k] + n;
    }
    V.x = R == 1 ? x[0] + n : at<double>(workspace, L.x);  // one system: the second block of the caller's array
    V.r = at<double>(workspace, L.r);
    V.z = at<double>(workspace, L.z);
    V.p = at<double>(workspace, L.p);
    V.Ap = at<double>(workspace, L.Ap);
    V.part = at<double>(workspace, L.part);
    V.sc = at<char>(workspace, L.sc);
    V.rtol = rtol;
    V.info = info;
    auto blocks_for = [](int64_t items) {
        int64_t b = (items + kMatvecLdsWaves - 1) / kMatvecLdsWaves;
        if (b < 1) b = 1;
        return (unsigned)(b < kNumCU ? b : kNumCU);
    };
    const unsigned row_wg = blocks_for(n), col_wg = blocks_for(mb);
    static_assert(kNumCU * kMatvecLdsGroup <= kPcgParts, "one partial sum per group of waves");
    V.mv_blocks = (int)col_wg * kMatvecLdsGroup;
    int64_t vb = (mb + kThreads - 1) / kThreads;
    if (vb < 1) vb = 1;
    if (vb > kPcgParts) vb = kPcgParts;
    V.vec_blocks = (int)vb;
    int64_t nb = (N + kThreads - 1) / kThreads;
    if (nb > kPcgParts) nb = kPcgParts;
    const bool all = n * R <= kMatvecLdsCap && mb * R <= kMatvecLdsCap;  // either half fits the LDS

    hipStream_t s = static_cast<hipStream_t>(stream);
    // packed vectors go in own[0] / out[0]
    auto half = [&](int mode, const double *in, const double *const (&own)[R], double *const (&out)[R], const int *skip) {
        SchurArgs<R> H = S;
        H.in = in;
        for (int k = 0; k < R; ++k) {
            H.own[k] = own[k];
            H.out[k] = out[k];
        }
        H.dot_part = V.part;
        H.skip = skip;
        const dim3 grid(mode == kSchurRows || mode == kSchurRowsFinal ? row_wg : col_wg), block(kMatvecLdsThreads);
#define REGOT_SCHUR_LAUNCH(MODE)                                                                  \
    if (all) hipLaunchKernelGGL((schur_half_kernel<MODE, R, true>), grid, block, 0, s, H);       \
    else hipLaunchKernelGGL((schur_half_kernel<MODE, R, false>), grid, block, 0, s, H)
        switch (mode) {
        case kSchurRows: REGOT_SCHUR_LAUNCH(kSchurRows); break;
        case kSchurRowsFinal: REGOT_SCHUR_LAUNCH(kSchurRowsFinal); break;
        case kSchurCols: REGOT_SCHUR_LAUNCH(kSchurCols); break;
        default: REGOT_SCHUR_LAUNCH(kSchurColsRhs); break;
        }
#undef REGOT_SCHUR_LAUNCH
    };
    const double *none[R] = {};
    const double *g1[R], *g2[R], *p_packed[R] = {};
    double *rs[R], *x1[R], *u_packed[R] = {}, *Ap_packed[R] = {};
    for (int k = 0; k < R; ++k) {
        g1[k] = rhs[k];
        g2[k] = rhs[k] + n;
        rs[k] = const_cast<double *>(V.rhs[k]);
        x1[k] = x[k];
    }
    p_packed[0] = V.p;
    u_packed[0] = u;
    Ap_packed[0] = V.Ap;
    if (restart) {
        SchurPrepareArgs<R> P{};
        P.n = n;
        P.N = N;
        for (int k = 0; k < R; ++k) P.rhs[k] = rhs[k];
        P.row_sum = row_sum;
        P.eta = eta;
        P.tau = tau;
        P.u = u;
        P.part = V.part;
        hipLaunchKernelGGL((schur_prepare_kernel<R>), dim3((unsigned)nb), dim3(kThreads), 0, s, P);
        half(kSchurColsRhs, u, g2, rs, nullptr);
        hipLaunchKernelGGL((pcg_start_kernel<R>), dim3((unsigned)vb), dim3(kThreads), 0, s, V);
        hipLaunchKernelGGL((pcg_start_scalars_kernel<R>), dim3(1), dim3(kThreads), 0, s, V, (int)nb);
    }
    for (int it = 0; it < iterations; ++it) {
        const int *skip = reinterpret_cast<const int *>(at<char>(workspace, L.sc) + (it & 1) * sizeof(PcgScalars<R>) +
                                                        offsetof(PcgScalars<R>, all_done));
        half(kSchurRows, V.p, none, u_packed, skip);
        half(kSchurCols, u, p_packed, Ap_packed, skip);
        hipLaunchKernelGGL((pcg_update_kernel<R>), dim3((unsigned)vb), dim3(kThreads), 0, s, V, it);
        hipLaunchKernelGGL((pcg_direction_kernel<R>), dim3((unsigned)vb), dim3(kThreads), 0, s, V, it);
    }
    // the first blocks of the solutions for the second blocks as they stand, and the record of the iteration
    half(kSchurRowsFinal, V.x, g1, x1, nullptr);
    hipLaunchKernelGGL((pcg_finish_kernel<R>), dim3(R == 1 ? 1u : (unsigned)vb), dim3(kThreads), 0, s, V, iterations);
    return hip_status();
}

}  // namespace

extern "C" {

const char *regot_status_string(int status)
{
    switch (status) {
    case REGOT_OK: return "REGOT_OK";
    case REGOT_ERR_NULL: return "REGOT_ERR_NULL: a required pointer is NULL";
    case REGOT_ERR_DIM: return "REGOT_ERR_DIM: invalid n or m";
    case REGOT_ERR_ETA: return "REGOT_ERR_ETA: eta must be finite and > 0";
    case REGOT_ERR_LD: return "REGOT_ERR_LD: ldM < m";
    case REGOT_ERR_ALIGN: return "REGOT_ERR_ALIGN: misaligned pointer";
    case REGOT_ERR_WORKSPACE: return "REGOT_ERR_WORKSPACE: workspace too small";
    case REGOT_ERR_ARG: return "REGOT_ERR_ARG: invalid argument";
    case REGOT_ERR_HIP: return "REGOT_ERR_HIP: a HIP call failed";
    case REGOT_ERR_SCRATCH: return "REGOT_ERR_SCRATCH: the problem needs more workspace than the library's static buffer holds";
    default: return "REGOT: unknown status";
    }
}

int regot_profile_stage1(void *start_event, void *stop_event)
{
    g_prof_start = static_cast<hipEvent_t>(start_event);
    g_prof_stop = static_cast<hipEvent_t>(stop_event);
    return REGOT_OK;
}

int regot_plan_geometry(int64_t n, int64_t m, int64_t csr_capacity, int64_t *geometry)
{
    if (!geometry) return REGOT_ERR_NULL;
    if (n < 0 || m < 0 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (csr_capacity < -1) return REGOT_ERR_ARG;
    const int rounds = csr_capacity >= 0 ? plan_rounds(csr_capacity) : 1;
    const Geometry G = make_geometry(n, m, REGOT_PLAN_WAVES_PER_EU * rounds, true);
    int64_t tallest = 0;
    for (int g = 0; g < G.g_r; ++g) {
        int begin, end;
        chunk_rows(g, G.g_r, (int)n, begin, end);
        if (end - begin > tallest) tallest = end - begin;
    }
    geometry[0] = G.g_r;
    geometry[1] = G.g_c;
    geometry[2] = rounds;
    geometry[3] = tallest;
    geometry[4] = G.strip_blocks;
    return REGOT_OK;
}

int regot_placement_probe(int grid, uint32_t *ids, regot_stream_t stream)
{
    if (!ids) return REGOT_ERR_NULL;
    if (grid < 1 || grid > 65536) return REGOT_ERR_ARG;
    if (misaligned(ids, 4)) return REGOT_ERR_ALIGN;
    hipLaunchKernelGGL(placement_probe_kernel, dim3((unsigned)grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), ids);
    return hip_status();
}

int regot_stream_read_probe(int64_t n, int64_t m, const double *M, int64_t ldM, double *sum, void *workspace,
                            size_t workspace_bytes, regot_stream_t stream)
{
    int st = check_matrix(n, m, M, ldM, 1.0, true);
    if (st != REGOT_OK) return st;
    if (!sum) return REGOT_ERR_NULL;
    if (misaligned(sum, 8)) return REGOT_ERR_ALIGN;
    const Geometry G = make_geometry(n, m, REGOT_PLAN_WAVES_PER_EU, kLseStrip);  // the cut of the dense calls, strip included
    const Layout L = make_layout(n, m, -1);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;
    const int wide_gc = G.strip_blocks > 0 ? G.g_c - 1 : G.g_c;
    const int64_t nblocks = (int64_t)G.g_r * wide_gc + G.strip_blocks;
    if (nblocks > kMaxDim) return REGOT_ERR_DIM;
    Stage1Args A{};
    A.n = (int)n;
    A.m = (int)m;
    A.ldM = ldM;
    A.M = M;
    A.g_c = G.g_c;
    A.g_r = G.g_r;
    A.wide_gc = wide_gc;
    A.wide_blocks = G.g_r * wide_gc;
    A.strip_blocks = G.strip_blocks;
    A.colpart = at<double>(workspace, L.colpart);
    hipStream_t s = static_cast<hipStream_t>(stream);
    prof_begin(s);
    if (nblocks > 0) {
        if (aligned16(M, ldM))
            hipLaunchKernelGGL((read_probe_kernel<true>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A);
        else
            hipLaunchKernelGGL((read_probe_kernel<false>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A);
    }
    prof_end(s);
    hipLaunchKernelGGL(read_probe_sum_kernel, dim3(1), dim3(kThreads), 0, s, A.colpart, (int)nblocks, sum);
    return hip_status();
}

int regot_workspace_bytes(int64_t n, int64_t m, int64_t csr_capacity, size_t *bytes)
{
    if (!bytes) return REGOT_ERR_NULL;
    if (n < 0 || m < 0 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (csr_capacity < -1) return REGOT_ERR_ARG;
    *bytes = make_layout(n, m, csr_capacity).total;
    return REGOT_OK;
}

int regot_dual_eval(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a, const double *b,
                    const double *alpha, const double *beta, double eta, double *obj, double *grad_alpha,
                    double *grad_beta, double *row_sum, double *col_sum, void *workspace,
                    size_t workspace_bytes, regot_stream_t stream)
{
    return run_plan_pass<true, false>(n, m, M, ldM, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum,
                                      col_sum, 0.0, nullptr, nullptr, nullptr, -1, nullptr, workspace,
                                      workspace_bytes, stream);
}

int regot_dual_eval_noalloc(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a, const double *b,
                            const double *alpha, const double *beta, double eta, double *obj, double *grad_alpha,
                            double *grad_beta, double *row_sum, double *col_sum, regot_stream_t stream)
{
    int st = check_plan_args<true, false>(n, m, M, ldM, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum,
                                          col_sum, 0.0, nullptr, nullptr, nullptr, -1, nullptr);
    if (st != REGOT_OK) return st;
    if (make_layout(n, m, -1).total > kScratchBytes) return REGOT_ERR_SCRATCH;
    void *ws = nullptr;
    st = scratch_of_current_device(&ws);
    if (st != REGOT_OK) return st;
    // Nothing in the workspace of this call has to start at zero: every partial sum the second kernel reads
    // has been written by the first, whatever an earlier (larger) call left behind.
    return run_plan_pass<true, false>(n, m, M, ldM, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum,
                                      col_sum, 0.0, nullptr, nullptr, nullptr, -1, nullptr, ws, kScratchBytes, stream);
}

int regot_sparsify_csr(int64_t n, int64_t m, const double *M, int64_t ldM, const double *alpha,
                       const double *beta, double eta, double delta, int64_t *row_ptr, int32_t *col_idx,
                       double *val, int64_t capacity, int64_t *info, void *workspace, size_t workspace_bytes,
                       regot_stream_t stream)
{
    return run_plan_pass<false, true>(n, m, M, ldM, nullptr, nullptr, alpha, beta, eta, nullptr, nullptr, nullptr,
                                      nullptr, nullptr, delta, row_ptr, col_idx, val, capacity, info, workspace,
                                      workspace_bytes, stream);
}

int regot_dual_eval_sparsify(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a,
                             const double *b, const double *alpha, const double *beta, double eta, double *obj,
                             double *grad_alpha, double *grad_beta, double *row_sum, double *col_sum,
                             double delta, int64_t *row_ptr, int32_t *col_idx, double *val, int64_t capacity,
                             int64_t *info, void *workspace, size_t workspace_bytes, regot_stream_t stream)
{
    return run_plan_pass<true, true>(n, m, M, ldM, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum,
                                     col_sum, delta, row_ptr, col_idx, val, capacity, info, workspace,
                                     workspace_bytes, stream);
}

int regot_refresh_candidate_capacity(int64_t n, int64_t m, int64_t k, int64_t *capacity)
{
    if (!capacity) return REGOT_ERR_NULL;
    const int st = check_topk_dims(n, m, k);
    if (st != REGOT_OK) return st;
    *capacity = refresh_candidate_capacity(n, m, k);
    return REGOT_OK;
}

int regot_dual_eval_sparsify_topk(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a, const double *b,
                                  const double *alpha, const double *beta, double eta, int64_t k, double *obj,
                                  double *grad_alpha, double *grad_beta, double *row_sum, double *col_sum,
                                  double *delta, int64_t *row_ptr, int32_t *col_idx, double *val, int64_t capacity,
                                  int64_t *info, void *workspace, size_t workspace_bytes, void *topk_workspace,
                                  size_t topk_workspace_bytes, regot_stream_t stream)
{
    int st = check_topk_dims(n, m, k);
    if (st != REGOT_OK) return st;
    st = check_matrix(n, m, M, ldM, eta, false);
    if (st != REGOT_OK) return st;
    if (!a || !b || !alpha || !beta || !obj || !grad_alpha || !grad_beta || !delta || !row_ptr || !info)
        return REGOT_ERR_NULL;
    if (capacity < 0) return REGOT_ERR_ARG;
    if (capacity > 0 && (!col_idx || !val)) return REGOT_ERR_NULL;
    if (misaligned(a, 8) || misaligned(b, 8) || misaligned(alpha, 8) || misaligned(beta, 8) || misaligned(obj, 8) ||
        misaligned(grad_alpha, 8) || misaligned(grad_beta, 8) || misaligned(row_sum, 8) || misaligned(col_sum, 8) ||
        misaligned(delta, 8) || misaligned(row_ptr, 8) || misaligned(info, 8) || misaligned(col_idx, 4) ||
        misaligned(val, 8))
        return REGOT_ERR_ALIGN;
    RefreshCtx rc{};
    rc.cand_capacity = refresh_candidate_capacity(n, m, k);
    rc.cand_expected = refresh_candidate_expected(n, m, k);
    st = check_workspace(workspace, workspace_bytes, make_layout(n, m, rc.cand_capacity).total);
    if (st != REGOT_OK) return st;
    const SelectLayout SL = make_select_layout(n, m, k);
    st = check_workspace(topk_workspace, topk_workspace_bytes, SL.total);
    if (st != REGOT_OK) return st;
    const Geometry G = make_geometry(n, m, REGOT_SELECT_WAVES_PER_EU);
    const int64_t sel_blocks = (int64_t)G.g_r * G.g_c;
    if (sel_blocks > kMaxDim) return REGOT_ERR_DIM;

    SelectArgs Q{};
    Q.n = (int)n;
    Q.m = (int)m;
    Q.ldM = ldM;
    Q.M = M;
    Q.alpha = alpha;
    Q.beta = beta;
    Q.g_c = G.g_c;
    Q.g_r = G.g_r;
    Q.k = k;
    Q.states = at<SelState>(topk_workspace, SL.states);
    Q.cnt = at<SelCounters>(topk_workspace, SL.counters);
    Q.ghist = at<u64>(topk_workspace, SL.ghist);
    Q.pool = at<u64>(topk_workspace, SL.pool);
    Q.small_pool = at<u64>(topk_workspace, SL.small_pool);
    Q.sample = at<u64>(topk_workspace, SL.sample);
    Q.pool_cap = SL.pool_cap;
    Q.value_domain = 1;
    Q.delta = delta;
    Q.s_k = nullptr;
    CandParams *cp = at<CandParams>(topk_workspace, SL.extra);
    Q.info = reinterpret_cast<int64_t *>(at<char>(topk_workspace, SL.extra) + 64);
    Q.ex = make_exp_params(eta);
    rc.cp = cp;
    rc.sel = Q;
    rc.sel_blocks = (unsigned)sel_blocks;
    rc.sel_aligned = aligned16(M, ldM);
    rc.sel_info = Q.info;
    rc.rsel = at<RefreshSel>(topk_workspace, SL.refresh_sel);

    // the sample and the lower end of its bracket; then the fused pass with that end as its threshold
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(select_gather_kernel, dim3(kSample / kThreads), dim3(kThreads), 0, s, Q);
    for (int idx = kIdxFirstSample; idx < kIdxBracket; ++idx)
        hipLaunchKernelGGL(select_sample_kernel, dim3(kSampleGrid), dim3(kThreads), 0, s, Q, idx);
    // (also clears the header of the dense calls' workspace: same layout whatever the capacity, see make_layout)
    hipLaunchKernelGGL(refresh_bracket_kernel, dim3(1), dim3(kThreads), 0, s, Q, cp, rc.rsel,
                       at<int>(workspace, make_layout(n, m, rc.cand_capacity).header));
    return run_plan_pass<true, true>(n, m, M, ldM, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum, col_sum,
                                     0.0, row_ptr, col_idx, val, capacity, info, workspace, workspace_bytes, stream, &rc);
}

int regot_sinkhorn_half_step(int64_t n, int64_t m, const double *M, int64_t ldM, const double *marginal,
                             const double *alpha, const double *beta, double eta, int which, double *out,
                             void *workspace, size_t workspace_bytes, regot_stream_t stream)
{
    int st = check_matrix(n, m, M, ldM, eta, false);
    if (st != REGOT_OK) return st;
    if (which != 0 && which != 1) return REGOT_ERR_ARG;
    const double *other = which == 0 ? beta : alpha;
    if (!marginal || !other || !out) return REGOT_ERR_NULL;
    if (misaligned(marginal, 8) || misaligned(other, 8) || misaligned(out, 8)) return REGOT_ERR_ALIGN;
    // (a narrow last panel is shared by a few strip workgroups beside the tasks of the full panels, as in the plan pass)
    const Geometry G = make_geometry(n, m, which == 0 ? REGOT_ROWLSE_WAVES_PER_EU : REGOT_COLLSE_WAVES_PER_EU, kLseStrip);
    const Layout L = make_layout(n, m, -1);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;

    hipStream_t s = static_cast<hipStream_t>(stream);
    Stage1Args A{};
    A.n = (int)n;
    A.m = (int)m;
    A.ldM = ldM;
    A.M = M;
    A.alpha = alpha;
    A.beta = beta;
    A.g_c = G.g_c;
    A.g_r = G.g_r;
    A.rowpart = at<double>(workspace, L.rowpart);
    A.colpart = at<double>(workspace, L.colpart);
    A.ex = make_exp_params(eta);
    A.wide_gc = G.strip_blocks > 0 ? G.g_c - 1 : G.g_c;
    A.wide_blocks = G.g_r * A.wide_gc;
    A.strip_blocks = G.strip_blocks;
    const int64_t nblocks = (int64_t)A.wide_blocks + G.strip_blocks;
    if (nblocks > kMaxDim) return REGOT_ERR_DIM;
    const bool al16 = aligned16(M, ldM);
    LseFinalizeArgs F{};
    F.marginal = marginal;
    F.eta = eta;
    F.out = out;
    F.ex = A.ex;
    prof_begin(s);
    if (which == 0) {
        if (al16)
            hipLaunchKernelGGL((row_lse_kernel<true>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A);
        else
            hipLaunchKernelGGL((row_lse_kernel<false>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A);
        F.len = n;
        F.parts = G.g_c;
        F.part = A.rowpart;
    } else {
        if (al16)
            hipLaunchKernelGGL((col_lse_kernel<true>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A);
        else
            hipLaunchKernelGGL((col_lse_kernel<false>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A);
        F.len = m;
        F.parts = G.g_r;
        F.part = A.colpart;
    }
    prof_end(s);
    const unsigned fin = (unsigned)((F.len + kLanes - 1) / kLanes);
    hipLaunchKernelGGL(lse_finalize_kernel, dim3(fin), dim3(kThreads), 0, s, F);
    return hip_status();
}

int regot_topk_workspace_bytes(int64_t n, int64_t m, int64_t k, size_t *bytes)
{
    if (!bytes) return REGOT_ERR_NULL;
    const int st = check_topk_dims(n, m, k);
    if (st != REGOT_OK) return st;
    *bytes = make_select_layout(n, m, k).total;
    return REGOT_OK;
}

int regot_topk_threshold(int64_t n, int64_t m, const double *M, int64_t ldM, const double *alpha,
                         const double *beta, double eta, int64_t k, double *delta, double *s_k, int64_t *info,
                         void *workspace, size_t workspace_bytes, regot_stream_t stream)
{
    int st = check_matrix(n, m, M, ldM, eta, false);
    if (st != REGOT_OK) return st;
    st = check_topk_dims(n, m, k);
    if (st != REGOT_OK) return st;
    if (!alpha || !beta || !delta || !info) return REGOT_ERR_NULL;
    if (misaligned(alpha, 8) || misaligned(beta, 8) || misaligned(delta, 8) || misaligned(s_k, 8) ||
        misaligned(info, 8))
        return REGOT_ERR_ALIGN;
    const Geometry G = make_geometry(n, m, REGOT_SELECT_WAVES_PER_EU);
    const SelectLayout L = make_select_layout(n, m, k);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;
    const int64_t nblocks = (int64_t)G.g_r * G.g_c;
    if (nblocks > kMaxDim) return REGOT_ERR_DIM;

    hipStream_t s = static_cast<hipStream_t>(stream);
    SelectArgs A{};
    A.n = (int)n;
    A.m = (int)m;
    A.ldM = ldM;
    A.M = M;
    A.alpha = alpha;
    A.beta = beta;
    A.g_c = G.g_c;
    A.g_r = G.g_r;
    A.k = k;
    A.states = at<SelState>(workspace, L.states);
    A.cnt = at<SelCounters>(workspace, L.counters);
    A.ghist = at<u64>(workspace, L.ghist);
    A.pool = at<u64>(workspace, L.pool);
    A.small_pool = at<u64>(workspace, L.small_pool);
    A.sample = at<u64>(workspace, L.sample);
    A.pool_cap = L.pool_cap;
    // (pace keeping between the two workgroups of a compute unit is built into the passes over M, SelectArgs::pair_stride,
    // but left off: measured -3 % at 50000^2, +1 % at 20000^2, nothing at 40000 x 10000: these passes wait for memory)
    A.progress = at<int>(workspace, L.progress);
    A.delta = delta;
    A.s_k = s_k;
    A.info = info;
    A.ex = make_exp_params(eta);
    const bool al16 = aligned16(M, ldM);

    // The whole worst case is enqueued; every kernel works out from its predecessor's record whether
    // it has anything to do.  Order: sample (gather, two histograms), bracket pass, radix steps (over the
    // pool the bracket pass has filled; over M, then the pool, if the bracket was not usable), result.
    hipLaunchKernelGGL(select_gather_kernel, dim3(kSample / kThreads), dim3(kThreads), 0, s, A);
    for (int idx = kIdxFirstSample; idx < kIdxBracket; ++idx)
        hipLaunchKernelGGL(select_sample_kernel, dim3(kSampleGrid), dim3(kThreads), 0, s, A, idx);
    for (int idx = kIdxBracket; idx < kIdxFinish; ++idx) {
        if (idx == kIdxBracket) prof_begin(s);
        if (al16)
            hipLaunchKernelGGL((select_step_kernel<true>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A, idx);
        else
            hipLaunchKernelGGL((select_step_kernel<false>), dim3((unsigned)nblocks), dim3(kThreads), 0, s, A, idx);
        if (idx == kIdxBracket) prof_end(s);
    }
    hipLaunchKernelGGL(select_finish_kernel, dim3(1), dim3(kThreads), 0, s, A, (int)kIdxFinish);
    return hip_status();
}

int regot_sinkhorn_sweeps(int64_t n, int64_t m, const double *M, int64_t ldM, const double *a, const double *b,
                          double *alpha, double *beta, double eta, int sweeps, void *workspace, size_t workspace_bytes,
                          regot_stream_t stream)
{
    if (sweeps < 0 || sweeps > 1000000) return REGOT_ERR_ARG;
    if (!alpha || !beta) return REGOT_ERR_NULL;
    if (sweeps == 0) {
        // nothing to enqueue, but the arguments are checked as they would be
        const int st = check_matrix(n, m, M, ldM, eta, false);
        if (st != REGOT_OK) return st;
        return (!a || !b) ? REGOT_ERR_NULL : REGOT_OK;
    }
    for (int s = 0; s < sweeps; ++s) {
        int st = regot_sinkhorn_half_step(n, m, M, ldM, a, alpha, beta, eta, 0, alpha, workspace, workspace_bytes, stream);
        if (st != REGOT_OK) return st;
        st = regot_sinkhorn_half_step(n, m, M, ldM, b, alpha, beta, eta, 1, beta, workspace, workspace_bytes, stream);
        if (st != REGOT_OK) return st;
    }
    return REGOT_OK;
}

int regot_pattern_values(int64_t n, int64_t m, const double *M, int64_t ldM, const double *alpha,
                         const double *beta, double eta, const int64_t *row_ptr, const int32_t *col_idx,
                         const int64_t *csc_pos, int64_t capacity, double *val, double *val_csc,
                         regot_stream_t stream)
{
    int st = check_matrix(n, m, M, ldM, eta, true);
    if (st != REGOT_OK) return st;
    if (capacity < 0) return REGOT_ERR_ARG;
    if (!row_ptr || (n > 0 && !alpha) || (m > 0 && !beta)) return REGOT_ERR_NULL;
    if (capacity > 0 && (!col_idx || !val)) return REGOT_ERR_NULL;
    if (val_csc && !csc_pos) return REGOT_ERR_NULL;
    if (misaligned(alpha, 8) || misaligned(beta, 8) || misaligned(row_ptr, 8) || misaligned(csc_pos, 8) ||
        misaligned(val, 8) || misaligned(val_csc, 8) || misaligned(col_idx, 4))
        return REGOT_ERR_ALIGN;
    if (n == 0 || m == 0 || capacity == 0) return REGOT_OK;
    PatternArgs A{};
    A.n = (int)n;
    A.m = (int)m;
    A.ldM = ldM;
    A.M = M;
    A.alpha = alpha;
    A.beta = beta;
    A.row_ptr = row_ptr;
    A.col_idx = col_idx;
    A.csc_pos = csc_pos;
    A.capacity = capacity;
    A.val = val;
    A.val_csc = val_csc;
    A.ex = make_exp_params(eta);
    const int64_t want = (n + kWaves - 1) / kWaves;
    const unsigned grid = (unsigned)(want < 16 * kNumCU ? want : 16 * kNumCU);
    hipLaunchKernelGGL(pattern_values_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), A);
    return hip_status();
}

int regot_hessian_matvec(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr,
                         const int32_t *col_idx, const double *val, const int64_t *col_ptr,
                         const int32_t *row_idx, const double *val_csc, int64_t capacity, const double *row_sum,
                         const double *col_sum, const double *x, double *y, regot_stream_t stream)
{
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!(eta > 0.0) || !isfinite(eta)) return REGOT_ERR_ETA;
    if (capacity < 0 || tau != tau) return REGOT_ERR_ARG;
    if (!row_ptr || !col_ptr || !row_sum || !col_sum || !x || !y) return REGOT_ERR_NULL;
    if (capacity > 0 && (!col_idx || !val || !row_idx || !val_csc)) return REGOT_ERR_NULL;
    if (misaligned(row_ptr, 8) || misaligned(col_ptr, 8) || misaligned(val, 8) || misaligned(val_csc, 8) ||
        misaligned(row_sum, 8) || misaligned(col_sum, 8) || misaligned(x, 8) || misaligned(y, 8) ||
        misaligned(col_idx, 4) || misaligned(row_idx, 4))
        return REGOT_ERR_ALIGN;
    MatvecArgs A{};
    A.n = (int)n;
    A.m = (int)m;
    A.eta = eta;
    A.tau = tau;
    A.row_ptr = row_ptr;
    A.col_idx = col_idx;
    A.val = val;
    A.col_ptr = col_ptr;
    A.row_idx = row_idx;
    A.val_csc = val_csc;
    A.capacity = capacity;
    A.row_sum = row_sum;
    A.col_sum = col_sum;
    A.x = x;
    A.y = y;
    if (n <= kMatvecLdsCap && m - 1 <= kMatvecLdsCap) {
        // both halves of x fit the LDS: the kernel of the conjugate-gradient iteration (without its inner product), one
        // workgroup per compute unit, half of them on the rows; the same sums by the same lanes in the same order
        int64_t rw = (n + kMatvecLdsWaves - 1) / kMatvecLdsWaves, cw = (m - 1 + kMatvecLdsWaves - 1) / kMatvecLdsWaves;
        if (rw > kNumCU / 2) rw = kNumCU / 2;
        if (cw > kNumCU / 2) cw = kNumCU / 2;
        if (cw < 1) cw = 1;
        hipLaunchKernelGGL((hessian_matvec_lds_kernel<false, 1, true>), dim3((unsigned)(rw + cw)), dim3(kMatvecLdsThreads), 0,
                           static_cast<hipStream_t>(stream), A, (double *)nullptr, 0, (const int *)nullptr, (int)rw);
        return hip_status();
    }
    // workgroups (4 waves each) for the rows and for the m - 1 columns, at most 16 per CU each
    const int64_t cap_blocks = 16 * kNumCU;
    int64_t rb = (n + kWaves - 1) / kWaves, cb = (m - 1 + kWaves - 1) / kWaves;
    if (rb > cap_blocks) rb = cap_blocks;
    if (cb > cap_blocks) cb = cap_blocks;
    A.row_waves = rb * kWaves;
    hipLaunchKernelGGL(hessian_matvec_kernel, dim3((unsigned)(rb + cb)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), A);
    return hip_status();
}

int regot_hessian_workspace_bytes(int64_t n, int64_t m, size_t *bytes)
{
    if (!bytes) return REGOT_ERR_NULL;
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    const int64_t nblk = (n + kRowsPerScanBlock - 1) / kRowsPerScanBlock;
    *bytes = align_up((size_t)(nblk + 1) * sizeof(int64_t));
    return REGOT_OK;
}

int regot_hessian_lower_csc(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr,
                            const int32_t *col_idx, const double *val, int64_t capacity, const double *row_sum,
                            const double *col_sum, int64_t *h_col_ptr, int32_t *h_row_idx, double *h_val,
                            int64_t h_capacity, int64_t *info, int values_only, void *workspace,
                            size_t workspace_bytes, regot_stream_t stream)
{
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!(eta > 0.0) || !isfinite(eta)) return REGOT_ERR_ETA;
    if (capacity < 0 || h_capacity < 0 || tau != tau || (values_only != 0 && values_only != 1)) return REGOT_ERR_ARG;
    if (!row_ptr || !row_sum || !col_sum || !h_col_ptr || !info) return REGOT_ERR_NULL;
    if (capacity > 0 && (!col_idx || !val)) return REGOT_ERR_NULL;
    if (h_capacity > 0 && (!h_row_idx || !h_val)) return REGOT_ERR_NULL;
    if (misaligned(row_ptr, 8) || misaligned(val, 8) || misaligned(row_sum, 8) || misaligned(col_sum, 8) ||
        misaligned(h_col_ptr, 8) || misaligned(h_val, 8) || misaligned(info, 8) || misaligned(col_idx, 4) ||
        misaligned(h_row_idx, 4))
        return REGOT_ERR_ALIGN;
    size_t need = 0;
    (void)regot_hessian_workspace_bytes(n, m, &need);
    int st = check_workspace(workspace, workspace_bytes, need);
    if (st != REGOT_OK) return st;
    LowerArgs A{};
    A.n = (int)n;
    A.m = (int)m;
    A.eta = eta;
    A.tau = tau;
    A.row_ptr = row_ptr;
    A.col_idx = col_idx;
    A.val = val;
    A.capacity = capacity;
    A.row_sum = row_sum;
    A.col_sum = col_sum;
    A.h_col_ptr = h_col_ptr;
    A.h_row_idx = h_row_idx;
    A.h_val = h_val;
    A.h_capacity = h_capacity;
    A.info = info;
    A.blk = static_cast<int64_t *>(workspace);
    A.nblk = (int)((n + kRowsPerScanBlock - 1) / kRowsPerScanBlock);
    A.values_only = values_only;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!values_only) {
        hipLaunchKernelGGL(lower_count_kernel, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, A);
        hipLaunchKernelGGL(lower_scan_kernel, dim3(1), dim3(kThreads), 0, s, A);
    }
    int64_t beta_blocks = (m - 1 + kThreads - 1) / kThreads;
    if (beta_blocks < 1) beta_blocks = 1;
    hipLaunchKernelGGL(lower_fill_kernel, dim3((unsigned)(A.nblk + beta_blocks)), dim3(kThreads), 0, s, A);
    return hip_status();
}

int regot_dual_metrics(int64_t n, int64_t m, const double *a, const double *b, const double *alpha,
                       const double *beta, double eta, const double *row_sum, const double *col_sum,
                       double *metrics, void *workspace, size_t workspace_bytes, regot_stream_t stream)
{
    if (n < 0 || m < 0 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!(eta > 0.0) || !isfinite(eta)) return REGOT_ERR_ETA;
    if (!metrics || (n > 0 && (!a || !alpha || !row_sum)) || (m > 0 && (!b || !beta || !col_sum))) return REGOT_ERR_NULL;
    if (misaligned(a, 8) || misaligned(b, 8) || misaligned(alpha, 8) || misaligned(beta, 8) || misaligned(row_sum, 8) ||
        misaligned(col_sum, 8) || misaligned(metrics, 8))
        return REGOT_ERR_ALIGN;
    const Layout L = make_layout(n, m, -1);
    int st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;
    MetricArgs A{};
    A.n = n;
    A.m = m;
    A.a = a;
    A.b = b;
    A.alpha = alpha;
    A.beta = beta;
    A.row_sum = row_sum;
    A.col_sum = col_sum;
    A.eta = eta;
    A.part = at<double>(workspace, L.metric_part);
    A.metrics = metrics;
    int64_t parts = (n + m + 4 * kThreads - 1) / (4 * kThreads);
    if (parts < 1) parts = 1;
    if (parts > kMetricParts) parts = kMetricParts;
    A.parts = (int)parts;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(metric_parts_kernel, dim3((unsigned)parts), dim3(kThreads), 0, s, A);
    hipLaunchKernelGGL(metric_final_kernel, dim3(1), dim3(kLanes), 0, s, A);
    return hip_status();
}

int regot_choose_candidate(int64_t n, int64_t m, const double *obj_q, const double *obj_s, const double *alpha_q,
                           const double *beta_q, const double *alpha_s, const double *beta_s, double *alpha_out,
                           double *beta_out, int64_t *choice, regot_stream_t stream)
{
    if (n < 0 || m < 0 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!obj_q || !obj_s || !choice) return REGOT_ERR_NULL;
    if ((n > 0 && (!alpha_q || !alpha_s || !alpha_out)) || (m > 0 && (!beta_q || !beta_s || !beta_out)))
        return REGOT_ERR_NULL;
    if (misaligned(obj_q, 8) || misaligned(obj_s, 8) || misaligned(alpha_q, 8) || misaligned(beta_q, 8) ||
        misaligned(alpha_s, 8) || misaligned(beta_s, 8) || misaligned(alpha_out, 8) || misaligned(beta_out, 8) ||
        misaligned(choice, 8))
        return REGOT_ERR_ALIGN;
    ChooseArgs A{n, m, obj_q, obj_s, alpha_q, beta_q, alpha_s, beta_s, alpha_out, beta_out, choice};
    int64_t blocks = (n + m + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > 4 * kNumCU) blocks = 4 * kNumCU;
    hipLaunchKernelGGL(choose_candidate_kernel, dim3((unsigned)blocks), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), A);
    return hip_status();
}

int regot_pcg_workspace_bytes(int64_t n, int64_t m, size_t *bytes)
{
    if (!bytes) return REGOT_ERR_NULL;
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    *bytes = make_pcg_layout(n, m).total;
    return REGOT_OK;
}

int regot_pcg_solve(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr, const int32_t *col_idx,
                    const double *val, const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                    int64_t capacity, const double *row_sum, const double *col_sum, const double *rhs, double *x,
                    double rtol, int iterations, int restart, double *info, void *workspace,
                    size_t workspace_bytes, regot_stream_t stream)
{
    const double *const rhs1[1] = {rhs};
    double *const x1[1] = {x};
    return run_pcg<1>(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, capacity, row_sum, col_sum,
                      rhs1, x1, rtol, iterations, restart, info, workspace, workspace_bytes, stream);
}

int regot_pcg_solve_reduced(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr,
                            const int32_t *col_idx, const double *val, const int64_t *col_ptr, const int32_t *row_idx,
                            const double *val_csc, int64_t capacity, const double *row_sum, const double *col_sum,
                            const double *rhs, double *x, double rtol, int iterations, int restart, double *info,
                            void *workspace, size_t workspace_bytes, regot_stream_t stream)
{
    const double *const rhs1[1] = {rhs};
    double *const x1[1] = {x};
    return run_pcg_reduced<1>(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, capacity, row_sum,
                              col_sum, rhs1, x1, rtol, iterations, restart, info, workspace, workspace_bytes, stream);
}

int regot_pcg_solve2_reduced(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr,
                             const int32_t *col_idx, const double *val, const int64_t *col_ptr, const int32_t *row_idx,
                             const double *val_csc, int64_t capacity, const double *row_sum, const double *col_sum,
                             const double *rhs_a, const double *rhs_b, double *x_a, double *x_b, double rtol,
                             int iterations, int restart, double *info, void *workspace, size_t workspace_bytes,
                             regot_stream_t stream)
{
    if (x_a && x_a == x_b) return REGOT_ERR_ARG;
    const double *const rhs2[2] = {rhs_a, rhs_b};
    double *const x2[2] = {x_a, x_b};
    return run_pcg_reduced<2>(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, capacity, row_sum,
                              col_sum, rhs2, x2, rtol, iterations, restart, info, workspace, workspace_bytes, stream);
}

int regot_pcg_solve2(int64_t n, int64_t m, double eta, double tau, const int64_t *row_ptr, const int32_t *col_idx,
                     const double *val, const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                     int64_t capacity, const double *row_sum, const double *col_sum, const double *rhs_a,
                     const double *rhs_b, double *x_a, double *x_b, double rtol, int iterations, int restart,
                     double *info, void *workspace, size_t workspace_bytes, regot_stream_t stream)
{
    if (x_a && x_a == x_b) return REGOT_ERR_ARG;
    const double *const rhs2[2] = {rhs_a, rhs_b};
    double *const x2[2] = {x_a, x_b};
    return run_pcg<2>(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, capacity, row_sum, col_sum,
                      rhs2, x2, rtol, iterations, restart, info, workspace, workspace_bytes, stream);
}

int regot_splr_direction(int64_t n, int64_t m, const double *p, const double *q, const double *s_prev,
                         const double *y_prev, const double *v, double *d, double *info, void *workspace,
                         size_t workspace_bytes, regot_stream_t stream)
{
    if (n < 1 || m < 1 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (!p || !d || !info) return REGOT_ERR_NULL;
    const bool any = q || s_prev || y_prev || v;
    if (any && !(q && s_prev && y_prev && v)) return REGOT_ERR_NULL;
    if (misaligned(p, 8) || misaligned(q, 8) || misaligned(s_prev, 8) || misaligned(y_prev, 8) || misaligned(v, 8) ||
        misaligned(d, 8) || misaligned(info, 8))
        return REGOT_ERR_ALIGN;
    const PcgLayout L = make_pcg_layout(n, m);
    const int st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != REGOT_OK) return st;
    CombineArgs A{};
    A.N = n + m - 1;
    A.p = p;
    A.q = q;
    A.s = s_prev;
    A.y = y_prev;
    A.v = v;
    A.d = d;
    A.info = info;
    A.part = at<double>(workspace, L.part);
    int64_t blocks = (A.N + kThreads - 1) / kThreads;
    if (blocks > kPcgParts) blocks = kPcgParts;
    A.blocks = (int)blocks;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (any) hipLaunchKernelGGL(splr_dots_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, A);
    hipLaunchKernelGGL(splr_combine_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, A);
    return hip_status();
}

}  // extern "C"

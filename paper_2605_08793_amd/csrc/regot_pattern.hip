// regot_pattern_transpose: the sparsity pattern by columns (symbolic work, once per pattern;
// Sec. 4.2 keeps a pattern for S iterations; the transposed block of H_Omega in Sec. 3.1 eq. (7) reads
// it).  The interface is documented in include/regot.h.
//
// Steps, all kernels of this file:
//   1. count the entries of every column (integer atomics: the counts do not depend on their order);
//   2. exclusive scan of the counts -> col_ptr (per-block sums, a one-workgroup scan of those, apply);
//   3. every entry takes a place inside its column's segment in the order in which the atomics happen
//      to arrive, and leaves its CSR position p there;
//   4. every column's segment is sorted by p.  CSR positions grow with the row, and a column holds at
//      most one entry per row, so ascending p is ascending row: the result is the pattern by columns
//      with strictly ascending rows, whatever order step 3 ran in.  Short segments (the usual case:
//      about a hundred entries) are sorted by one wave in LDS (bitonic network); a column with more than
//      kWaveCap entries is put on a list and sorted by a whole workgroup: pieces of kBlockCap entries
//      in LDS, then merged pairwise in memory (every entry finds its place in the partner run by
//      a binary search; keys are distinct, so the merge is unambiguous);
//   5. with the final order known: row_idx[q] = row of entry p (the last i with row_ptr[i] <= p),
//      csc_pos[p] = q.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "regot.h"

namespace {

constexpr int64_t kMaxDim = 2147483647LL;
constexpr size_t kAlign = 256;
constexpr int kBlock = 256;
constexpr int kLanes = 64;
constexpr int kWavesPerBlock = kBlock / kLanes;
constexpr int kScanPer = 8;                      // counts per thread in the scan kernels
constexpr int kScanTile = kBlock * kScanPer;     // counts per workgroup
constexpr int kWaveCap = 1024;                   // longest segment a single wave sorts in LDS
constexpr int kBlockCap = 2048;                  // piece a workgroup sorts in LDS
constexpr unsigned kPad = 0xffffffffu;           // sorts behind every CSR position

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

struct TransposeLayout {
    size_t count, block_sum, place, place2, long_cols, long_count;
    int64_t scan_blocks, max_long;
    size_t total;
};

TransposeLayout make_transpose_layout(int64_t m, int64_t nnz)
{
    TransposeLayout L{};
    const size_t e = (size_t)(nnz > 0 ? nnz : 1);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L.scan_blocks = (m + 1 + kScanTile - 1) / kScanTile;
    L.max_long = nnz / (kWaveCap + 1) + 1;  // columns with more than kWaveCap entries
    if (L.max_long > m) L.max_long = m > 0 ? m : 1;
    L.count = take((size_t)(m + 1) * sizeof(int32_t));
    L.block_sum = take((size_t)(L.scan_blocks + 1) * sizeof(int64_t));
    L.place = take(e * sizeof(uint32_t));
    L.place2 = take(e * sizeof(uint32_t));
    L.long_cols = take((size_t)L.max_long * sizeof(int32_t));
    L.long_count = take(sizeof(int32_t));
    L.total = off;
    return L;
}

struct TransposeArgs {
    int64_t n, m, nnz;
    const int64_t *row_ptr;
    const int32_t *col_idx;
    int64_t *col_ptr;
    int32_t *row_idx;
    int64_t *csc_pos;
    int32_t *count;      // [m + 1]; entry m stays 0
    int64_t *block_sum;  // [scan_blocks + 1]
    uint32_t *place;     // [nnz] CSR positions, column by column
    uint32_t *place2;    // [nnz] second buffer of the merges
    int32_t *long_cols;  // [max_long]
    int32_t *long_count; // [1]
    int64_t scan_blocks;
    int64_t max_long;
};

__global__ __launch_bounds__(kBlock) void clear_kernel(TransposeArgs A)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i <= A.m) A.count[i] = 0;
    if (i == 0) *A.long_count = 0;
}

__global__ __launch_bounds__(kBlock) void count_kernel(TransposeArgs A)
{
    const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (p >= A.nnz) return;
    const int64_t j = A.col_idx[p];
    if (j >= 0 && j < A.m) atomicAdd(&A.count[j], 1);
}

// sum of the workgroup's kScanTile counts
__global__ __launch_bounds__(kBlock) void scan_sums_kernel(TransposeArgs A)
{
    __shared__ int64_t lds[kBlock];
    const int64_t first = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kScanPer;
    int64_t s = 0;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k)
        if (first + k <= A.m) s += A.count[first + k];
    lds[threadIdx.x] = s;
    __syncthreads();
    for (int d = kBlock / 2; d > 0; d >>= 1) {
        if ((int)threadIdx.x < d) lds[threadIdx.x] += lds[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) A.block_sum[blockIdx.x] = lds[0];
}

// exclusive scan across the workgroup; returns this thread's offset, *total = sum of all
__device__ __forceinline__ int64_t block_exclusive_scan(int64_t mine, int64_t *lds /* [kBlock] */, int64_t *total)
{
    lds[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < kBlock; d <<= 1) {
        const int64_t up = (int)threadIdx.x >= d ? lds[threadIdx.x - d] : 0;
        __syncthreads();
        lds[threadIdx.x] += up;
        __syncthreads();
    }
    const int64_t incl = lds[threadIdx.x];
    *total = lds[kBlock - 1];
    __syncthreads();
    return incl - mine;
}

// one workgroup: the per-block sums become their exclusive prefix
__global__ __launch_bounds__(kBlock) void scan_top_kernel(TransposeArgs A)
{
    __shared__ int64_t lds[kBlock];
    int64_t carry = 0;
    for (int64_t base = 0; base < A.scan_blocks; base += kBlock) {
        const int64_t i = base + threadIdx.x;
        const int64_t mine = i < A.scan_blocks ? A.block_sum[i] : 0;
        int64_t total;
        const int64_t excl = block_exclusive_scan(mine, lds, &total);
        if (i < A.scan_blocks) A.block_sum[i] = carry + excl;
        carry += total;
    }
}

// col_ptr from the counts and the blocks' offsets; the counts are cleared for step 3, which uses them as cursors
__global__ __launch_bounds__(kBlock) void scan_apply_kernel(TransposeArgs A)
{
    __shared__ int64_t lds[kBlock];
    const int64_t first = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kScanPer;
    int c[kScanPer];
    int64_t mine = 0;
#pragma unroll
    for (int k = 0; k < kScanPer; ++k) {
        c[k] = first + k <= A.m ? A.count[first + k] : 0;
        mine += c[k];
    }
    int64_t total;
    int64_t run = A.block_sum[blockIdx.x] + block_exclusive_scan(mine, lds, &total);
#pragma unroll
    for (int k = 0; k < kScanPer; ++k)
        if (first + k <= A.m) {
            A.col_ptr[first + k] = run;
            A.count[first + k] = 0;
            run += c[k];
        }
}

__global__ __launch_bounds__(kBlock) void place_kernel(TransposeArgs A)
{
    const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (p >= A.nnz) return;
    const int64_t j = A.col_idx[p];
    if (j >= 0 && j < A.m) {
        const int64_t at = A.col_ptr[j] + atomicAdd(&A.count[j], 1);
        if (at < A.nnz) A.place[at] = (uint32_t)p;
    } else {
        A.csc_pos[p] = -1;  // not an entry of any column
    }
}

// row of CSR position p: the last i with row_ptr[i] <= p
__device__ __forceinline__ int64_t row_of(const TransposeArgs &A, int64_t p)
{
    int64_t lo = 0, hi = A.n;  // invariant: row_ptr[lo] <= p, and (hi == n or row_ptr[hi] > p)
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (A.row_ptr[mid] <= p) lo = mid;
        else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void emit(const TransposeArgs &A, int64_t q, uint32_t p)
{
    if (p == kPad || (int64_t)p >= A.nnz) return;
    A.row_idx[q] = (int32_t)row_of(A, p);
    A.csc_pos[p] = q;
}

// Bitonic network over N = a power of two keys in LDS, run by T threads that all call this (T a power of two
// <= N / 2 ... or more: surplus threads idle); `sync` separates the stages.
template <typename Sync>
__device__ __forceinline__ void bitonic_sort(unsigned *keys, int N, int tid, int T, Sync sync)
{
    for (int k = 2; k <= N; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < N / 2; t += T) {
                // the t-th compare-exchange of this stage: partners i and i + j with bit j of i clear
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const unsigned a = keys[i], b = keys[i + j];
                const bool up = (i & k) == 0;
                if ((a > b) == up) {
                    keys[i] = b;
                    keys[i + j] = a;
                }
            }
            sync();
        }
}

// Step 4 and 5 for the short columns: one wave per column, four columns per workgroup at a time.
__global__ __launch_bounds__(kBlock) void sort_short_kernel(TransposeArgs A)
{
    __shared__ unsigned lds[kWavesPerBlock][kWaveCap];
    const int lane = threadIdx.x & (kLanes - 1), w = threadIdx.x >> 6;
    unsigned *keys = lds[w];
    // (a wave runs in lockstep, but the LDS traffic of one stage must be complete before the next reads it)
    auto wave_sync = [] { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); };
    for (int64_t j = (int64_t)blockIdx.x * kWavesPerBlock + w; j < A.m; j += (int64_t)gridDim.x * kWavesPerBlock) {
        const int64_t begin = A.col_ptr[j];
        const int64_t len = A.col_ptr[j + 1] - begin;
        if (len <= 0) continue;
        if (len > kWaveCap) {
            if (lane == 0) {
                const int slot = atomicAdd(A.long_count, 1);
                if (slot < A.max_long) A.long_cols[slot] = (int32_t)j;
            }
            continue;
        }
        int N = 2;
        while (N < len) N <<= 1;
        for (int i = lane; i < N; i += kLanes) keys[i] = i < len ? A.place[begin + i] : kPad;
        wave_sync();
        bitonic_sort(keys, N, lane, kLanes, wave_sync);
        for (int i = lane; i < (int)len; i += kLanes) emit(A, begin + i, keys[i]);
        wave_sync();
    }
}

// first position in the ascending run[0 .. len) whose key is not below `key`; the run was written by this
// workgroup's own stores, which are complete in the L2 after the barrier: read there, not in the first-level cache
__device__ __forceinline__ int64_t lower_bound_run(const uint32_t *run, int64_t len, uint32_t key)
{
    int64_t lo = 0, hi = len;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (__hip_atomic_load(run + mid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < key) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Step 4 and 5 for the columns on the list: one workgroup per column.
__global__ __launch_bounds__(kBlock) void sort_long_kernel(TransposeArgs A)
{
    __shared__ unsigned keys[kBlockCap];
    const int tid = threadIdx.x;
    auto block_sync = [] { __syncthreads(); };
    int listed = *A.long_count;
    if (listed > A.max_long) listed = (int)A.max_long;
    for (int t = blockIdx.x; t < listed; t += gridDim.x) {
        const int64_t j = A.long_cols[t];
        const int64_t begin = A.col_ptr[j];
        const int64_t len = A.col_ptr[j + 1] - begin;
        uint32_t *src = A.place + begin, *dst = A.place2 + begin;
        // pieces of kBlockCap keys, each sorted in LDS
        for (int64_t c0 = 0; c0 < len; c0 += kBlockCap) {
            const int64_t clen = len - c0 < kBlockCap ? len - c0 : kBlockCap;
            for (int i = tid; i < kBlockCap; i += kBlock) keys[i] = i < clen ? src[c0 + i] : kPad;
            __syncthreads();
            bitonic_sort(keys, kBlockCap, tid, kBlock, block_sync);
            for (int i = tid; i < (int)clen; i += kBlock) src[c0 + i] = keys[i];
            __syncthreads();
        }
        // merge neighbouring runs until one is left: an entry's place in the merged run is its place in its own
        // run plus the number of smaller keys in the partner run (keys are distinct)
        for (int64_t width = kBlockCap; width < len; width <<= 1) {
            for (int64_t i = tid; i < len; i += kBlock) {
                const int64_t run = i / width;
                const int64_t a0 = run * width, b0 = (run ^ 1) * width;
                const int64_t blen = b0 >= len ? 0 : (len - b0 < width ? len - b0 : width);
                const uint32_t key = __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int64_t other = blen > 0 ? lower_bound_run(src + b0, blen, key) : 0;
                const int64_t base = a0 < b0 ? a0 : b0;
                dst[base + (i - a0) + other] = key;
            }
            __syncthreads();
            uint32_t *tmp = src;
            src = dst;
            dst = tmp;
        }
        for (int64_t i = tid; i < len; i += kBlock)
            emit(A, begin + i, __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        __syncthreads();
    }
}

int check_dims(int64_t n, int64_t m, int64_t nnz)
{
    if (n < 0 || m < 0 || n > kMaxDim || m > kMaxDim) return REGOT_ERR_DIM;
    if (nnz < 0 || nnz > kMaxDim) return REGOT_ERR_ARG;
    return REGOT_OK;
}

}  // namespace

extern "C" {

int regot_pattern_transpose_workspace_bytes(int64_t n, int64_t m, int64_t nnz, size_t *bytes)
{
    if (!bytes) return REGOT_ERR_NULL;
    const int st = check_dims(n, m, nnz);
    if (st != REGOT_OK) return st;
    *bytes = make_transpose_layout(m, nnz).total;
    return REGOT_OK;
}

int regot_pattern_transpose(int64_t n, int64_t m, int64_t nnz, const int64_t *row_ptr, const int32_t *col_idx,
                            int64_t *col_ptr, int32_t *row_idx, int64_t *csc_pos, void *workspace,
                            size_t workspace_bytes, regot_stream_t stream)
{
    int st = check_dims(n, m, nnz);
    if (st != REGOT_OK) return st;
    if (!row_ptr || !col_ptr || (nnz > 0 && (!col_idx || !row_idx || !csc_pos))) return REGOT_ERR_NULL;
    if (misaligned(row_ptr, 8) || misaligned(col_ptr, 8) || misaligned(csc_pos, 8) || misaligned(col_idx, 4) ||
        misaligned(row_idx, 4))
        return REGOT_ERR_ALIGN;
    const TransposeLayout L = make_transpose_layout(m, nnz);
    if (!workspace) return REGOT_ERR_NULL;
    if (misaligned(workspace, kAlign)) return REGOT_ERR_ALIGN;
    if (workspace_bytes < L.total) return REGOT_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    TransposeArgs A{};
    A.n = n;
    A.m = m;
    A.nnz = nnz;
    A.row_ptr = row_ptr;
    A.col_idx = col_idx;
    A.col_ptr = col_ptr;
    A.row_idx = row_idx;
    A.csc_pos = csc_pos;
    A.count = reinterpret_cast<int32_t *>(ws + L.count);
    A.block_sum = reinterpret_cast<int64_t *>(ws + L.block_sum);
    A.place = reinterpret_cast<uint32_t *>(ws + L.place);
    A.place2 = reinterpret_cast<uint32_t *>(ws + L.place2);
    A.long_cols = reinterpret_cast<int32_t *>(ws + L.long_cols);
    A.long_count = reinterpret_cast<int32_t *>(ws + L.long_count);
    A.scan_blocks = L.scan_blocks;
    A.max_long = L.max_long;

    const unsigned col_blocks = (unsigned)((m + 1 + kBlock - 1) / kBlock);
    const unsigned entry_blocks = (unsigned)((nnz + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(clear_kernel, dim3(col_blocks), dim3(kBlock), 0, s, A);
    if (nnz > 0) hipLaunchKernelGGL(count_kernel, dim3(entry_blocks), dim3(kBlock), 0, s, A);
    hipLaunchKernelGGL(scan_sums_kernel, dim3((unsigned)L.scan_blocks), dim3(kBlock), 0, s, A);
    hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(kBlock), 0, s, A);
    hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)L.scan_blocks), dim3(kBlock), 0, s, A);
    if (nnz > 0 && m > 0) {
        hipLaunchKernelGGL(place_kernel, dim3(entry_blocks), dim3(kBlock), 0, s, A);
        int64_t short_blocks = (m + kWavesPerBlock - 1) / kWavesPerBlock;
        if (short_blocks > 16 * 256) short_blocks = 16 * 256;
        hipLaunchKernelGGL(sort_short_kernel, dim3((unsigned)short_blocks), dim3(kBlock), 0, s, A);
        const int64_t long_blocks = L.max_long < 1024 ? L.max_long : 1024;
        hipLaunchKernelGGL(sort_long_kernel, dim3((unsigned)long_blocks), dim3(kBlock), 0, s, A);
    }
    return hipGetLastError() == hipSuccess ? REGOT_OK : REGOT_ERR_HIP;
}

}  // extern "C"

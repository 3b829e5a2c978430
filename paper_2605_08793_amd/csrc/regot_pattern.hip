// regot_pattern_transpose: the sparsity pattern by columns (symbolic work, once per pattern;
// Sec. 4.2 keeps a pattern for S iterations; the transposed block of H_Omega in Sec. 3.1 eq. (7) reads
// it).  The interface is documented in include/regot.h.
//
// The pattern by columns is the list of CSR positions p sorted by (column, p): CSR positions grow with
// the row and a column holds at most one entry per row, so inside a column ascending p is ascending row.
// The positions start out in ascending order, so a STABLE sort by column alone gives that list: a
// least-significant-digit radix sort on the column index, 8 bits per pass, ceil(bits(m) / 8) passes (two
// for m < 65536), every kernel of this file:
//   0. entry_row[p] = row of CSR position p (one wave per row);
//   per pass:
//   1. every workgroup counts the digits of its tile of 2048 keys (LDS) -> table[digit][workgroup];
//   2. one workgroup per digit: exclusive scan of its row of the table, and the digit's total;
//   3. every workgroup ranks its keys stably (a wave takes 64 consecutive keys at a time; lanes with the
//      same digit find each other with eight ballots and rank by lane number behind the keys of that
//      digit the wave has already seen), orders the tile by digit in LDS and writes each digit's run to
//      its place: the digit's base + the table entry + the position inside the run;
//   then, on the sorted (column, p) list:
//   4. col_ptr[j] = number of keys below j (a binary search per column);
//   5. row_idx[q] = entry_row[p], csc_pos[p] = q.
// A col_idx outside [0, m) sorts as column m, behind every real column, and gets csc_pos = -1.
// No atomics on memory and no order that depends on timing: the same bits on every call.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "regot.h"

namespace {

constexpr int64_t kMaxDim = 2147483647LL;
constexpr size_t kAlign = 256;
constexpr int kBlock = 256;
constexpr int kLanes = 64;
constexpr int kWavesPerBlock = kBlock / kLanes;
constexpr int kItems = 8;                        // keys per thread
constexpr int kTile = kBlock * kItems;           // keys per workgroup
constexpr int kWaveKeys = kTile / kWavesPerBlock;  // consecutive keys a wave ranks
constexpr int kDigitBits = 8;
constexpr int kDigits = 1 << kDigitBits;
static_assert(kDigits == kBlock, "one thread per digit");
static_assert(kWaveKeys == kItems * kLanes, "a wave ranks kItems groups of 64 keys");

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

struct TransposeLayout {
    size_t table, digit_total, entry_row, key[2], pay[2];
    int64_t blocks;
    int passes;
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
    L.blocks = (int64_t)((e + kTile - 1) / kTile);
    int bits = 0;  // keys are 0 .. m
    while (bits < 32 && ((uint64_t)m >> bits) != 0) ++bits;
    L.passes = bits <= kDigitBits ? 1 : (bits + kDigitBits - 1) / kDigitBits;
    L.table = take((size_t)kDigits * (size_t)L.blocks * sizeof(uint32_t));
    L.digit_total = take(kDigits * sizeof(uint32_t));
    L.entry_row = take(e * sizeof(int32_t));
    for (int k = 0; k < 2; ++k) {
        L.key[k] = take(e * sizeof(uint32_t));
        L.pay[k] = take(e * sizeof(uint32_t));
    }
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
    uint32_t *table;        // [kDigits][blocks]
    uint32_t *digit_total;  // [kDigits]
    int32_t *entry_row;     // [nnz]
    int64_t blocks;
};

// one pass of the sort: FIRST reads the keys from col_idx (positions are the payload), else from key_in / pay_in
struct PassArgs {
    const uint32_t *key_in, *pay_in;
    uint32_t *key_out, *pay_out;
    int shift;
};

__device__ __forceinline__ uint32_t column_key(const TransposeArgs &A, int64_t p)
{
    const int64_t j = A.col_idx[p];
    return (uint32_t)(j >= 0 && j < A.m ? j : A.m);
}

template <bool FIRST>
__device__ __forceinline__ uint32_t load_key(const TransposeArgs &A, const PassArgs &P, int64_t i)
{
    return FIRST ? column_key(A, i) : P.key_in[i];
}

// step 0: one wave per row
__global__ __launch_bounds__(kBlock) void entry_row_kernel(TransposeArgs A)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    for (int64_t i = wave; i < A.n; i += (int64_t)gridDim.x * kWavesPerBlock) {
        int64_t p0 = A.row_ptr[i], p1 = A.row_ptr[i + 1];
        if (p0 < 0) p0 = 0;
        if (p1 > A.nnz) p1 = A.nnz;
        for (int64_t p = p0 + lane; p < p1; p += kLanes) A.entry_row[p] = (int32_t)i;
    }
}

// step 1
template <bool FIRST>
__global__ __launch_bounds__(kBlock) void digit_count_kernel(TransposeArgs A, PassArgs P)
{
    __shared__ unsigned hist[kDigits];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kTile;
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int64_t i = base + k * kBlock + threadIdx.x;
        if (i < A.nnz) atomicAdd(&hist[(load_key<FIRST>(A, P, i) >> P.shift) & (kDigits - 1)], 1u);
    }
    __syncthreads();
    A.table[(size_t)threadIdx.x * A.blocks + blockIdx.x] = hist[threadIdx.x];
}

// exclusive scan of one value per thread across the workgroup; *total = sum of all (lds: [kBlock])
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t mine, uint32_t *lds, uint32_t *total)
{
    lds[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < kBlock; d <<= 1) {
        const uint32_t up = (int)threadIdx.x >= d ? lds[threadIdx.x - d] : 0u;
        __syncthreads();
        lds[threadIdx.x] += up;
        __syncthreads();
    }
    const uint32_t incl = lds[threadIdx.x];
    *total = lds[kBlock - 1];
    __syncthreads();
    return incl - mine;
}

// step 2: workgroup d turns row d of the table into its exclusive prefix and leaves the row's sum
__global__ __launch_bounds__(kBlock) void digit_scan_kernel(TransposeArgs A)
{
    __shared__ uint32_t lds[kBlock];
    constexpr int kPer = 4;
    uint32_t *row = A.table + (size_t)blockIdx.x * A.blocks;
    uint32_t carry = 0;
    for (int64_t base = 0; base < A.blocks; base += kBlock * kPer) {
        const int64_t first = base + (int64_t)threadIdx.x * kPer;
        uint32_t c[kPer], mine = 0;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            c[k] = first + k < A.blocks ? row[first + k] : 0u;
            mine += c[k];
        }
        uint32_t total;
        uint32_t run = carry + block_exclusive_scan(mine, lds, &total);
#pragma unroll
        for (int k = 0; k < kPer; ++k)
            if (first + k < A.blocks) {
                row[first + k] = run;
                run += c[k];
            }
        carry += total;
    }
    if (threadIdx.x == 0) A.digit_total[blockIdx.x] = carry;
}

// step 3
template <bool FIRST>
__global__ __launch_bounds__(kBlock) void digit_scatter_kernel(TransposeArgs A, PassArgs P)
{
    __shared__ uint32_t seen[kWavesPerBlock][kDigits];  // keys of a digit a wave has ranked so far; then the wave's offset
    __shared__ uint32_t run_start[kDigits];             // where the digit's run starts inside the tile
    __shared__ uint32_t run_dest[kDigits];              // where it goes in the output
    __shared__ uint32_t scan_lds[kBlock];
    __shared__ uint32_t tile_key[kTile], tile_pay[kTile];
    const int lane = threadIdx.x & (kLanes - 1), w = threadIdx.x >> 6;
    const int64_t base = (int64_t)blockIdx.x * kTile;
    const int64_t left = A.nnz - base;
    const int count = (int)(left < kTile ? left : kTile);
    auto wave_sync = [] { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); __builtin_amdgcn_wave_barrier(); };

#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) seen[k][threadIdx.x] = 0;
    __syncthreads();

    // the wave's keys in input order: group g, lane l is key w * kWaveKeys + g * 64 + l of the tile
    uint32_t key[kItems], pay[kItems], rank[kItems];
#pragma unroll
    for (int g = 0; g < kItems; ++g) {
        const int t = w * kWaveKeys + g * kLanes + lane;
        const bool valid = t < count;
        key[g] = valid ? load_key<FIRST>(A, P, base + t) : 0u;
        pay[g] = valid ? (FIRST ? (uint32_t)(base + t) : P.pay_in[base + t]) : 0u;
    }
#pragma unroll
    for (int g = 0; g < kItems; ++g) {
        const int t = w * kWaveKeys + g * kLanes + lane;
        const bool valid = t < count;
        const unsigned d = (key[g] >> P.shift) & (kDigits - 1);
        // lanes that hold the same digit
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kDigitBits; ++b) {
            const bool set = ((d >> b) & 1u) != 0;
            const uint64_t m = __ballot(set);
            peers &= set ? m : ~m;
        }
        const int before = __builtin_popcountll(peers & ((1ull << lane) - 1ull));
        uint32_t first = 0;
        if (valid) first = seen[w][d];
        wave_sync();
        if (valid && before == 0) seen[w][d] = first + (uint32_t)__builtin_popcountll(peers);
        wave_sync();
        rank[g] = first + (uint32_t)before;
    }
    __syncthreads();

    // thread d: the waves' offsets inside the run of digit d, the run's place in the tile and in the output
    {
        const int d = threadIdx.x;
        uint32_t run = 0;
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) {
            const uint32_t c = seen[k][d];
            seen[k][d] = run;
            run += c;
        }
        uint32_t total;
        const uint32_t start = block_exclusive_scan(run, scan_lds, &total);
        const uint32_t digit_base = block_exclusive_scan(A.digit_total[d], scan_lds, &total);
        run_start[d] = start;
        run_dest[d] = digit_base + A.table[(size_t)d * A.blocks + blockIdx.x];
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < kItems; ++g) {
        const int t = w * kWaveKeys + g * kLanes + lane;
        if (t < count) {
            const unsigned d = (key[g] >> P.shift) & (kDigits - 1);
            const uint32_t at = run_start[d] + seen[w][d] + rank[g];
            tile_key[at] = key[g];
            tile_pay[at] = pay[g];
        }
    }
    __syncthreads();
    // neighbouring threads now hold neighbouring keys of a run
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int t = k * kBlock + threadIdx.x;
        if (t < count) {
            const uint32_t kk = tile_key[t];
            const unsigned d = (kk >> P.shift) & (kDigits - 1);
            const int64_t at = (int64_t)run_dest[d] + (t - (int)run_start[d]);
            if (at < A.nnz) {  // always; a guard against a table that does not add up
                P.key_out[at] = kk;
                P.pay_out[at] = tile_pay[t];
            }
        }
    }
}

// step 4: col_ptr[j] = number of sorted keys below j, j = 0 .. m
__global__ __launch_bounds__(kBlock) void col_ptr_kernel(TransposeArgs A, const uint32_t *sorted_key)
{
    const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j > A.m) return;
    int64_t lo = 0, hi = A.nnz;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if ((int64_t)sorted_key[mid] < j) lo = mid + 1;
        else hi = mid;
    }
    A.col_ptr[j] = lo;
}

// step 5
__global__ __launch_bounds__(kBlock) void emit_kernel(TransposeArgs A, const uint32_t *sorted_key, const uint32_t *sorted_pay)
{
    const int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (q >= A.nnz) return;
    const int64_t p = sorted_pay[q];
    if (p >= A.nnz) return;  // never: the payloads are a permutation of the positions
    if ((int64_t)sorted_key[q] < A.m) {
        A.row_idx[q] = A.entry_row[p];
        A.csc_pos[p] = q;
    } else {
        A.csc_pos[p] = -1;  // not an entry of any column
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
    A.table = reinterpret_cast<uint32_t *>(ws + L.table);
    A.digit_total = reinterpret_cast<uint32_t *>(ws + L.digit_total);
    A.entry_row = reinterpret_cast<int32_t *>(ws + L.entry_row);
    A.blocks = L.blocks;
    uint32_t *key[2] = {reinterpret_cast<uint32_t *>(ws + L.key[0]), reinterpret_cast<uint32_t *>(ws + L.key[1])};
    uint32_t *pay[2] = {reinterpret_cast<uint32_t *>(ws + L.pay[0]), reinterpret_cast<uint32_t *>(ws + L.pay[1])};

    const unsigned col_blocks = (unsigned)((m + 1 + kBlock - 1) / kBlock);
    if (nnz == 0) {
        // no keys: every column starts and ends at 0
        hipLaunchKernelGGL(col_ptr_kernel, dim3(col_blocks), dim3(kBlock), 0, s, A, (const uint32_t *)key[0]);
        return hipGetLastError() == hipSuccess ? REGOT_OK : REGOT_ERR_HIP;
    }
    if (n > 0) {
        int64_t row_blocks = (n + kWavesPerBlock - 1) / kWavesPerBlock;
        if (row_blocks > 16 * 256) row_blocks = 16 * 256;
        hipLaunchKernelGGL(entry_row_kernel, dim3((unsigned)row_blocks), dim3(kBlock), 0, s, A);
    }
    const unsigned tiles = (unsigned)L.blocks;
    for (int pass = 0; pass < L.passes; ++pass) {
        PassArgs P{};
        P.key_in = pass == 0 ? nullptr : key[(pass - 1) & 1];
        P.pay_in = pass == 0 ? nullptr : pay[(pass - 1) & 1];
        P.key_out = key[pass & 1];
        P.pay_out = pay[pass & 1];
        P.shift = pass * kDigitBits;
        if (pass == 0) hipLaunchKernelGGL(digit_count_kernel<true>, dim3(tiles), dim3(kBlock), 0, s, A, P);
        else hipLaunchKernelGGL(digit_count_kernel<false>, dim3(tiles), dim3(kBlock), 0, s, A, P);
        hipLaunchKernelGGL(digit_scan_kernel, dim3(kDigits), dim3(kBlock), 0, s, A);
        if (pass == 0) hipLaunchKernelGGL(digit_scatter_kernel<true>, dim3(tiles), dim3(kBlock), 0, s, A, P);
        else hipLaunchKernelGGL(digit_scatter_kernel<false>, dim3(tiles), dim3(kBlock), 0, s, A, P);
    }
    const uint32_t *sorted_key = key[(L.passes - 1) & 1], *sorted_pay = pay[(L.passes - 1) & 1];
    hipLaunchKernelGGL(col_ptr_kernel, dim3(col_blocks), dim3(kBlock), 0, s, A, sorted_key);
    hipLaunchKernelGGL(emit_kernel, dim3((unsigned)((nnz + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, A, sorted_key,
                       sorted_pay);
    return hipGetLastError() == hipSuccess ? REGOT_OK : REGOT_ERR_HIP;
}

}  // extern "C"

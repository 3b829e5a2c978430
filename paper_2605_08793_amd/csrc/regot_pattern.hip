// regot_pattern_transpose: the sparsity pattern by columns (symbolic work, once per pattern;
// Sec. 4.2 keeps a pattern for S iterations).  The interface is documented in include/regot.h.
//
// A CSR pattern is already sorted by (row, column).  A STABLE sort of its entries by column
// therefore lists every column's entries by ascending row, which is the pattern by columns.
// The sort is rocPRIM's radix sort of (column, entry index) pairs; the kernels around it are
// index arithmetic.
#include <cstring>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <rocprim/device/device_radix_sort.hpp>

#include "regot.h"

namespace {

constexpr int64_t kMaxDim = 2147483647LL;
constexpr size_t kAlign = 256;
constexpr int kBlock = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

struct TransposeLayout {
    size_t keys_out, index_in, perm, sort_temp;
    size_t sort_temp_bytes;
    size_t total;
};

// The sort's own temporary storage is bounded here without asking the device: a second copy of
// keys and values plus a fixed amount for its digit counters.  The call checks the bound against
// what rocPRIM actually asks for.
TransposeLayout make_transpose_layout(int64_t nnz)
{
    TransposeLayout L{};
    const size_t e = (size_t)(nnz > 0 ? nnz : 1);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L.keys_out = take(e * sizeof(int32_t));
    L.index_in = take(e * sizeof(int32_t));
    L.perm = take(e * sizeof(int32_t));
    L.sort_temp_bytes = 2 * e * sizeof(int32_t) + (8u << 20);
    L.sort_temp = take(L.sort_temp_bytes);
    L.total = off;
    return L;
}

__global__ void iota_kernel(int32_t *out, int64_t nnz)
{
    const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (p < nnz) out[p] = (int32_t)p;
}

// entry q of the column order is CSR entry perm[q]; its row is the last i with row_ptr[i] <= perm[q]
__global__ void place_kernel(int64_t n, int64_t nnz, const int64_t *row_ptr, const int32_t *perm, int32_t *row_idx,
                             int64_t *csc_pos)
{
    const int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (q >= nnz) return;
    const int64_t p = perm[q];
    int64_t lo = 0, hi = n;  // invariant: row_ptr[lo] <= p, and (hi == n or row_ptr[hi] > p)
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (row_ptr[mid] <= p) lo = mid;
        else hi = mid;
    }
    row_idx[q] = (int32_t)lo;
    if (p >= 0 && p < nnz) csc_pos[p] = q;
}

// col_ptr[j] = number of sorted keys below j
__global__ void col_ptr_kernel(int64_t m, int64_t nnz, const int32_t *keys_sorted, int64_t *col_ptr)
{
    const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j > m) return;
    int64_t lo = 0, hi = nnz;  // first position whose key is >= j
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (keys_sorted[mid] < (int32_t)j) lo = mid + 1;
        else hi = mid;
    }
    col_ptr[j] = lo;
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
    *bytes = make_transpose_layout(nnz).total;
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
    const TransposeLayout L = make_transpose_layout(nnz);
    if (!workspace) return REGOT_ERR_NULL;
    if (misaligned(workspace, kAlign)) return REGOT_ERR_ALIGN;
    if (workspace_bytes < L.total) return REGOT_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    int32_t *keys_out = reinterpret_cast<int32_t *>(ws + L.keys_out);
    int32_t *index_in = reinterpret_cast<int32_t *>(ws + L.index_in);
    int32_t *perm = reinterpret_cast<int32_t *>(ws + L.perm);
    void *sort_temp = ws + L.sort_temp;

    const unsigned col_blocks = (unsigned)((m + 1 + kBlock - 1) / kBlock);
    if (nnz > 0) {
        // columns are below m: only the bits m - 1 needs take part in the sort
        unsigned end_bit = 1;
        while (end_bit < 31 && ((int64_t)1 << end_bit) < m) ++end_bit;
        size_t need = 0;
        if (rocprim::radix_sort_pairs(nullptr, need, col_idx, keys_out, index_in, perm, (unsigned)nnz, 0u, end_bit, s) !=
            hipSuccess)
            return REGOT_ERR_HIP;
        if (need > L.sort_temp_bytes) return REGOT_ERR_WORKSPACE;
        const unsigned blocks = (unsigned)((nnz + kBlock - 1) / kBlock);
        hipLaunchKernelGGL(iota_kernel, dim3(blocks), dim3(kBlock), 0, s, index_in, nnz);
        size_t have = L.sort_temp_bytes;
        if (rocprim::radix_sort_pairs(sort_temp, have, col_idx, keys_out, index_in, perm, (unsigned)nnz, 0u, end_bit, s) !=
            hipSuccess)
            return REGOT_ERR_HIP;
        hipLaunchKernelGGL(place_kernel, dim3(blocks), dim3(kBlock), 0, s, n, nnz, row_ptr, perm, row_idx, csc_pos);
    }
    hipLaunchKernelGGL(col_ptr_kernel, dim3(col_blocks), dim3(kBlock), 0, s, m, nnz, keys_out, col_ptr);
    return hipGetLastError() == hipSuccess ? REGOT_OK : REGOT_ERR_HIP;
}

}  // extern "C"

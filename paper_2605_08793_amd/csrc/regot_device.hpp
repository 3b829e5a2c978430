// Device-side building blocks shared by the streaming kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace regot {

constexpr int kLanes = 64;                  // wavefront width on CDNA
constexpr int kU = 4;                       // 16-byte loads per lane per matrix row
constexpr int kPanel = kLanes * 2 * kU;     // columns one wave covers per row (512)
constexpr int kWaves = 4;                   // waves per workgroup
constexpr int kThreads = kLanes * kWaves;
constexpr int kRB = 4;                      // matrix rows a wave keeps in flight
constexpr int kChunk = 1024;                // staged CSR records per pool chunk (>= kPanel)
constexpr int kExpDegree = 11;

typedef double dbl2 __attribute__((ext_vector_type(2)));

// Everything the device exponential needs, prepared on the host per call.
// exp_eta(s) = exp(s / eta) is evaluated as 2^k * P(r) with
//   k = rint(s * log2(e)/eta),  r = s - k*(eta*ln2)   (two-term Cody-Waite, in units of s),
//   P(r) = sum_i (c_i / eta^i) r^i,  c_i the near-minimax coefficients of exp on |x| <= ln2/2.
// Folding 1/eta into the constants saves the separate division of s by eta.
struct ExpParams {
    double c1;                 // log2(e) / eta
    double lhi, llo;           // eta*ln2 split in two doubles
    double q[kExpDegree + 1];  // c_i / eta^i
};

__device__ __forceinline__ double exp_eta(double s, const ExpParams &P)
{
    double t = s * P.c1;
    double k = __builtin_rint(t);
    double r = __builtin_fma(-k, P.lhi, s);
    r = __builtin_fma(-k, P.llo, r);
    double p = P.q[kExpDegree];
#pragma unroll
    for (int i = kExpDegree - 1; i >= 0; --i) p = __builtin_fma(p, r, P.q[i]);
    int ki;
    // saturating convert: a huge |k| becomes INT_MIN/INT_MAX and ldexp then gives 0 / inf
    asm("v_cvt_i32_f64 %0, %1" : "=v"(ki) : "v"(k));
    return __builtin_ldexp(p, ki);
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kLanes);
    return v;
}

__device__ __forceinline__ double wave_max(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, kLanes));
    return v;
}

// number of set bits of `mask` in lanes below the calling lane
__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The column tile of one lane: columns col0 + u*128 + 2*lane + e, u < kU, e < 2.
// FULL: all kPanel columns of the panel exist.  ALIGNED: 16-byte loads are legal.
template <bool ALIGNED, bool FULL, int NR>
__device__ __forceinline__ void load_rows(const double *__restrict__ Mlane, int64_t ldM, int64_t row0,
                                          const bool (&cv)[kU][2], double (&v)[NR][kU][2])
{
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const double *prow = Mlane + (row0 + r) * ldM;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const double *ptr = prow + u * (2 * kLanes);
            if constexpr (FULL && ALIGNED) {
                dbl2 x = __builtin_nontemporal_load(reinterpret_cast<const dbl2 *>(ptr));
                v[r][u][0] = x.x;
                v[r][u][1] = x.y;
            } else if constexpr (FULL) {
                v[r][u][0] = __builtin_nontemporal_load(ptr);
                v[r][u][1] = __builtin_nontemporal_load(ptr + 1);
            } else {
                v[r][u][0] = cv[u][0] ? __builtin_nontemporal_load(ptr) : 0.0;
                v[r][u][1] = cv[u][1] ? __builtin_nontemporal_load(ptr + 1) : 0.0;
            }
        }
    }
}

}  // namespace regot

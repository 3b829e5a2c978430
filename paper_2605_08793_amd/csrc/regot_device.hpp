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
constexpr int kExpDegree = 10;

typedef double dbl2 __attribute__((ext_vector_type(2)));

// Everything the device exponential needs, prepared on the host per call.
// exp_eta(s) = exp(s / eta) is evaluated as 2^k * P(r) with
//   k = rint(s * log2(e)/eta),  r = s - k*(eta*ln2)   (one fused multiply-add, in units of s),
//   P(r) = sum_i (c_i / eta^i) r^i,  c_i the near-minimax coefficients of exp on |x| <= ln2/2.
// Folding 1/eta into the constants saves the separate division of s by eta.
// Accuracy: the degree-10 polynomial is within 2.9e-16 of exp; rounding eta*ln2 to one double shifts
// r/eta by at most |k| ln2 2^-53, i.e. a relative error |x| 2^-53 in exp(x), x = s/eta -- the same size
// as the error any implementation makes that first rounds the quotient x = s/eta to a double.
struct ExpParams {
    double c1;                 // log2(e) / eta
    double l;                  // eta*ln2
    double q[kExpDegree + 1];  // c_i / eta^i
};

__device__ __forceinline__ double exp_eta(double s, const ExpParams &P)
{
    double t = s * P.c1;
    double k = __builtin_rint(t);
    double r = __builtin_fma(-k, P.l, s);
    double p = P.q[kExpDegree];
#pragma unroll
    for (int i = kExpDegree - 1; i >= 0; --i) p = __builtin_fma(p, r, P.q[i]);
    int ki;
    // saturating convert: a huge |k| becomes INT_MIN/INT_MAX and ldexp then gives 0 / inf
    asm("v_cvt_i32_f64 %0, %1" : "=v"(ki) : "v"(k));
    return __builtin_ldexp(p, ki);
}

// exp(s / eta) for ANY s.  exp_eta is exact in the IEEE sense only where its range reduction works: for an
// infinite s (an infinite cost: a forbidden assignment) the reduction forms inf - inf, and for finite s with
// |s / eta| beyond ~2^31 ln 2 it cancels catastrophically.  Here both tails are cut off where the result is 0
// or +inf anyway (2^-1100 and 2^1100 lie outside the range of a double); a NaN stays a NaN.  The streaming
// kernels call this only where a sum they formed with exp_eta came out not finite (rare, wave-uniform branch),
// so the common path pays one comparison per row, not two per entry.
__device__ __forceinline__ double exp_eta_any(double s, const ExpParams &P)
{
    const double t = s * P.c1;
    const double e = exp_eta(s, P);
    return t < -1100.0 ? 0.0 : (t > 1100.0 ? __builtin_inf() : e);
}

// true for NaN and for +-inf
__device__ __forceinline__ bool not_finite(double x) { return !(__builtin_fabs(x) < __builtin_inf()); }

// ---- cross-lane primitives ------------------------------------------------------------
// v_mov_b32 with a DPP lane pattern, applied to both halves of a double.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

constexpr int kDppXor1 = 0xB1;         // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each group of 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each row of 16

struct OpSum {
    static __device__ __forceinline__ double apply(double a, double b) { return a + b; }
};
struct OpMax {
    static __device__ __forceinline__ double apply(double a, double b) { return fmax(a, b); }
};

// combine the 16 lanes of each DPP row; every lane of the row ends with the row's result
template <typename Op>
__device__ __forceinline__ double row16_reduce(double v)
{
    v = Op::apply(v, dpp_f64<kDppXor1>(v));
    v = Op::apply(v, dpp_f64<kDppXor2>(v));
    v = Op::apply(v, dpp_f64<kDppHalfMirror>(v));
    v = Op::apply(v, dpp_f64<kDppMirror>(v));
    return v;
}

// x: lanes 0-31 keep x, lanes 32-63 receive y[lane-32];  y: lanes 0-31 receive x[lane+32], lanes 32-63 keep y
__device__ __forceinline__ void swap32(double &x, double &y)
{
    auto lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(x), (unsigned)__double2loint(y), false, false);
    auto hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(x), (unsigned)__double2hiint(y), false, false);
    x = __hiloint2double((int)hi[0], (int)lo[0]);
    y = __hiloint2double((int)hi[1], (int)lo[1]);
}

// odd 16-lane rows of x are exchanged with even 16-lane rows of y
__device__ __forceinline__ void swap16(double &x, double &y)
{
    auto lo = __builtin_amdgcn_permlane16_swap((unsigned)__double2loint(x), (unsigned)__double2loint(y), false, false);
    auto hi = __builtin_amdgcn_permlane16_swap((unsigned)__double2hiint(x), (unsigned)__double2hiint(y), false, false);
    x = __hiloint2double((int)hi[0], (int)lo[0]);
    y = __hiloint2double((int)hi[1], (int)lo[1]);
}

// Reduce four per-lane values (one per matrix row) across the wave at once.  The two swap
// steps halve the data while they halve the lanes, so the whole thing costs about as much as
// one plain 64-lane reduction.  On return every lane holds the wave-wide result of row
// quad_row(lane): lanes 0-15 row 0, 16-31 row 2, 32-47 row 1, 48-63 row 3.
template <typename Op>
__device__ __forceinline__ double wave_reduce4(double a0, double a1, double a2, double a3)
{
    swap32(a0, a1);
    swap32(a2, a3);
    double b0 = Op::apply(a0, a1);  // lanes < 32: row 0, lanes >= 32: row 1
    double b1 = Op::apply(a2, a3);  // lanes < 32: row 2, lanes >= 32: row 3
    swap16(b0, b1);
    return row16_reduce<Op>(Op::apply(b0, b1));
}

__device__ __forceinline__ int quad_row(int lane) { return ((lane >> 5) & 1) | (((lane >> 4) & 1) << 1); }

// value of lane `src` (a compile-time-free uniform index) broadcast to the wave
__device__ __forceinline__ double read_lane(double v, int src)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ int64_t read_lane_i64(int64_t v, int src)
{
    const int lo = __builtin_amdgcn_readlane((int)(uint32_t)v, src);
    const int hi = __builtin_amdgcn_readlane((int)(v >> 32), src);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// plain 64-lane reduction of one value; every lane gets the result
template <typename Op>
__device__ __forceinline__ double wave_reduce1(double v)
{
    v = row16_reduce<Op>(v);
    const double r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
    return Op::apply(Op::apply(r0, r1), Op::apply(r2, r3));
}

// sum over the workgroup, fixed order; result valid in every thread
__device__ __forceinline__ double block_sum(double v, double *lds /* [kWaves] */)
{
    v = wave_reduce1<OpSum>(v);
    __syncthreads();
    if ((threadIdx.x & (kLanes - 1)) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = lds[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r += lds[w];
    return r;
}

// number of set bits of `mask` in lanes below the calling lane
__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// How a workgroup treats the columns of its panel.
//   kPanelFull     all kPanel columns exist and belong to this panel
//   kPanelOverlap  the ragged last panel of a matrix with m >= kPanel: it is shifted left to start at
//                  m - kPanel, so all loads are unconditional, and the columns it shares with the
//                  panel before it are masked out of every result
//   kPanelPartial  m < kPanel: loads are guarded per element
//   kPanelOverlapEven  the same with m even: the shifted panel still starts at an even column, so
//                  16-byte loads stay legal
enum PanelMode { kPanelFull = 0, kPanelOverlap = 1, kPanelPartial = 2, kPanelOverlapEven = 3 };
__host__ __device__ constexpr bool is_overlap(int mode) { return mode == kPanelOverlap || mode == kPanelOverlapEven; }

// The column tile of one lane: columns col0 + u*128 + 2*lane + e, u < kU, e < 2.
// VEC16: 16-byte loads are legal.  GUARDED: only elements with cv[u][e] set may be touched.
// Groups u outside [u_lo, u_hi) own no column of the panel: they are not loaded (v = 0).
template <bool VEC16, bool GUARDED, int NR>
__device__ __forceinline__ void load_rows(const double *__restrict__ Mlane, int64_t ldM, int64_t row0,
                                          const bool (&cv)[kU][2], int u_lo, int u_hi, double (&v)[NR][kU][2])
{
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const double *prow = Mlane + (row0 + r) * ldM;
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            if (u < u_lo || u >= u_hi) {
                v[r][u][0] = v[r][u][1] = 0.0;
                continue;
            }
            const double *ptr = prow + u * (2 * kLanes);
            if constexpr (GUARDED) {
                v[r][u][0] = cv[u][0] ? __builtin_nontemporal_load(ptr) : 0.0;
                v[r][u][1] = cv[u][1] ? __builtin_nontemporal_load(ptr + 1) : 0.0;
            } else if constexpr (VEC16) {
                dbl2 x = __builtin_nontemporal_load(reinterpret_cast<const dbl2 *>(ptr));
                v[r][u][0] = x.x;
                v[r][u][1] = x.y;
            } else {
                v[r][u][0] = __builtin_nontemporal_load(ptr);
                v[r][u][1] = __builtin_nontemporal_load(ptr + 1);
            }
        }
    }
}

// Column bookkeeping of one lane for its panel.
template <int MODE>
struct PanelCols {
    int col0;          // first column the loads touch
    int u_lo, u_hi;    // 128-column groups [u_lo, u_hi) hold the panel's own columns (wave-uniform)
    bool cv[kU][2];    // column counts for this panel (always true in kPanelFull)
    __device__ __forceinline__ PanelCols(int p, int m, int lane)
    {
        const int ncol = min(kPanel, m - p * kPanel);  // columns that belong to this panel
        col0 = is_overlap(MODE) ? m - kPanel : p * kPanel;
        u_lo = is_overlap(MODE) ? (kPanel - ncol) / (2 * kLanes) : 0;
        u_hi = MODE == kPanelPartial ? (ncol + 2 * kLanes - 1) / (2 * kLanes) : kU;
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int c = u * (2 * kLanes) + 2 * lane + e;
                cv[u][e] = MODE == kPanelFull ? true : is_overlap(MODE) ? c >= kPanel - ncol : c < ncol;
            }
    }
    // does group u hold any column of this panel (always, in a full panel)
    __device__ __forceinline__ bool live(int u) const { return MODE == kPanelFull || (u >= u_lo && u < u_hi); }
    // does local column c (0 .. kPanel-1) belong to this panel
    static __device__ __forceinline__ bool owns(int c, int p, int m)
    {
        const int ncol = min(kPanel, m - p * kPanel);
        return MODE == kPanelFull ? true : is_overlap(MODE) ? c >= kPanel - ncol : c < ncol;
    }
};

// which mode the workgroup of panel p runs in
__device__ __forceinline__ int panel_mode(int p, int m)
{
    if (m - p * kPanel >= kPanel) return kPanelFull;
    return m >= kPanel ? ((m & 1) ? kPanelOverlap : kPanelOverlapEven) : kPanelPartial;
}

}  // namespace regot

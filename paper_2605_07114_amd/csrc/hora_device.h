// Device-side helpers shared by the HORA kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hora.h"

namespace hora {

constexpr int kWave = 64;
constexpr int kThreads = 256;              // threads per workgroup in every kernel here
constexpr int kWaves = kThreads / kWave;   // 4

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef double v2d __attribute__((ext_vector_type(2)));
typedef long long v2l __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

// Positive binary64 values order like their bit patterns read as unsigned integers.
__device__ __forceinline__ unsigned long long gain_bits(double g) {
    return (unsigned long long)__double_as_longlong(g);
}

// Marginal-gain recurrence (Sec. 3.2, stable update below Eq. 5).  One multiply, then
// one divide per step; `lf` is l as a double, `s` is alpha+beta.  The order of the
// operations is part of the result: these values break ties between prompts.
__device__ __forceinline__ double gain_first(double a, double s) { return a / s; }
__device__ __forceinline__ double gain_next(double m, double b, double s, double lf) {
    return (m * (b + lf)) / (s + (lf + 1.0));
}
// Survival product of the hit utility (App. A): E(l+1) = E(l) (beta+l)/(alpha+beta+l).
__device__ __forceinline__ double surv_next(double e, double b, double s, double lf) {
    return (e * (b + lf)) / (s + lf);
}

template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// ---------------------------------------------------------------------------------
// Wavefront prefix sums on the DPP cross-lane path (no LDS traffic).  The classic GCN
// sequence: shifts by 1, 2, 3 inside a row of 16 lanes, by 4 and 8 with bank masks, then
// the two row broadcasts that carry row totals across the four rows.
// Lanes that a mask disables, or whose source lies outside the row, contribute 0.
// ---------------------------------------------------------------------------------
template <int kCtrl, int kRowMask, int kBankMask>
__device__ __forceinline__ int dpp_take(int v) {
    return __builtin_amdgcn_update_dpp(0, v, kCtrl, kRowMask, kBankMask, true);
}

__device__ __forceinline__ int wave_incl_scan_i32(int v) {
    int t = v + dpp_take<0x111, 0xf, 0xf>(v);      // row_shr:1
    t += dpp_take<0x112, 0xf, 0xf>(v);             // row_shr:2
    t += dpp_take<0x113, 0xf, 0xf>(v);             // row_shr:3
    t += dpp_take<0x114, 0xf, 0xe>(t);             // row_shr:4, banks 1-3
    t += dpp_take<0x118, 0xf, 0xc>(t);             // row_shr:8, banks 2-3
    t += dpp_take<0x142, 0xa, 0xf>(t);             // row_bcast:15 into rows 1 and 3
    t += dpp_take<0x143, 0xc, 0xf>(t);             // row_bcast:31 into rows 2 and 3
    return t;
}

// Inclusive scan of non-negative 64-bit values below 2^50 as two 32-bit scans
// (low 22 bits and the rest), so that no partial sum over 64 lanes overflows.
__device__ __forceinline__ long long wave_incl_scan_i64(long long v) {
    const int lo = wave_incl_scan_i32((int)(v & 0x3fffff));
    const int hi = wave_incl_scan_i32((int)(v >> 22));
    return (long long)lo + ((long long)hi << 22);
}

// Inclusive scan of any 64-bit values whose sums fit 64 bits, as three 32-bit scans (pieces of
// 22, 21 and 21 bits: a piece's sum over 64 lanes stays below 2^28).
__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long v) {
    const unsigned lo = (unsigned)wave_incl_scan_i32((int)(v & 0x3fffffull));
    const unsigned mid = (unsigned)wave_incl_scan_i32((int)((v >> 22) & 0x1fffffull));
    const unsigned hi = (unsigned)wave_incl_scan_i32((int)(v >> 43));
    return (unsigned long long)lo + ((unsigned long long)mid << 22) + ((unsigned long long)hi << 43);
}

__device__ __forceinline__ unsigned long long wave_total_u64(unsigned long long v) {
    const unsigned long long t = wave_incl_scan_u64(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(t & 0xffffffffull), kWave - 1);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(t >> 32), kWave - 1);
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ int wave_last_i32(int v) { return __builtin_amdgcn_readlane(v, kWave - 1); }

__device__ __forceinline__ long long wave_total_i64(long long v) {   // same range as the scan
    const int lo = wave_last_i32(wave_incl_scan_i32((int)(v & 0x3fffff)));
    const int hi = wave_last_i32(wave_incl_scan_i32((int)(v >> 22)));
    return (long long)lo + ((long long)hi << 22);
}

// Number of lanes below this one whose bit is set in a wavefront ballot.
__device__ __forceinline__ int lanes_below(unsigned long long ballot) {
    return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(ballot >> 32),
                                          __builtin_amdgcn_mbcnt_lo((unsigned)ballot, 0u));
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        unsigned long long o = (unsigned long long)__shfl_xor((long long)v, d, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// Exclusive scan over the kThreads threads of a workgroup; `total` gets the sum.
// `lds` points at kWaves elements of LDS that the caller may reuse afterwards.
template <typename T>
__device__ __forceinline__ T block_excl_scan(T v, T* lds, T& total) {
    T inc = wave_incl_scan(v);
    const int w = wave_id();
    if (lane_id() == kWave - 1) lds[w] = inc;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
        T x = lds[i];
        if (i < w) base += x;
        tot += x;
    }
    __syncthreads();
    total = tot;
    return base + inc - v;
}

template <typename T>
__device__ __forceinline__ T block_sum(T v, T* lds) {
    v = wave_sum(v);
    if (lane_id() == 0) lds[wave_id()] = v;
    __syncthreads();
    T tot = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) tot += lds[i];
    __syncthreads();
    return tot;
}

__device__ __forceinline__ void report(int32_t* dev_status, int code) {
    // every writer stores an error code; which one lands is immaterial
    *reinterpret_cast<volatile int32_t*>(dev_status) = code;
}

}  // namespace hora

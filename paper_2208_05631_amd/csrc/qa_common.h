// Internal helpers of libqadagrad (gfx950 only).  Not part of the public interface.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qadagrad.h"

namespace qa {

constexpr int kThreads = 256;          // work-group size of every tile kernel: 4 wave64
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr int kTile = 4096;            // coordinates per work-group tile = 256 code words
constexpr int kTileWords = kTile / 16;

// ---- host-side argument checks ---------------------------------------------------------

inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
inline int ilog2(int64_t v) { int l = 0; while ((int64_t(1) << l) < v) ++l; return l; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int64_t words_of(int64_t d) { return (d + 15) / 16; }
inline int64_t tiles_of(int64_t d) { return (d + kTile - 1) / kTile; }
inline int64_t buckets_of(int64_t d, int64_t bucket) {
  return bucket > 0 ? (d + bucket - 1) / bucket : 1;
}

// Layout rules shared by every entry point that takes a qa_layout.
inline int check_layout(const qa_layout* L) {
  if (!L) return QA_ERR_INVALID_ARG;
  if (L->d < 1 || L->d >= (int64_t(1) << 40)) return QA_ERR_INVALID_ARG;
  if (L->M < 1 || L->M > 4096) return QA_ERR_INVALID_ARG;
  if (L->bucket != 0 && (L->bucket < 64 || !is_pow2(L->bucket))) return QA_ERR_INVALID_ARG;
  if (!(L->thr_coef > 0.0f) || !(L->thr_coef < 1e30f)) return QA_ERR_INVALID_ARG;
  if (L->code_stride < words_of(L->d)) return QA_ERR_INVALID_ARG;
  if (L->scale_stride < buckets_of(L->d, L->bucket)) return QA_ERR_INVALID_ARG;
  return QA_OK;
}

// Internal flag of quantize_launch (never accepted from the C ABI): the tile sums of |v| are
// already in the workspace, whose first M*ntiles doubles hold them (worker-major), so the first
// pass over the input is skipped.  Used when the producer of the input computed them on the way.
constexpr uint32_t kQuantAbsPartialsGiven = 0x80000000u;
inline int launch_status() { return hipGetLastError() == hipSuccess ? QA_OK : QA_ERR_LAUNCH; }

// ---- device-side reductions (binary64, fixed order: run-to-run deterministic) -----------

#if defined(__HIPCC__)

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  return __shfl_xor(v, mask, kWave);
}

// ---- wave64 sums with DPP (no LDS traffic): every lane receives the sum of all 64 lanes ----
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);   // every lane has a source
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const int lo = dpp_i32<CTRL>(__double2loint(v)), hi = dpp_i32<CTRL>(__double2hiint(v));
  return __hiloint2double(hi, lo);
}
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

__device__ __forceinline__ double readlane_f64(double v, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum_f64(double v) {
  v += dpp_f64<kDppQuadXor1>(v);
  v += dpp_f64<kDppQuadXor2>(v);
  v += dpp_f64<kDppRowHalfMirror>(v);
  v += dpp_f64<kDppRowMirror>(v);        // every lane: sum of its row of 16
  return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  v += (uint32_t)dpp_i32<kDppQuadXor1>((int)v);
  v += (uint32_t)dpp_i32<kDppQuadXor2>((int)v);
  v += (uint32_t)dpp_i32<kDppRowHalfMirror>((int)v);
  v += (uint32_t)dpp_i32<kDppRowMirror>((int)v);
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
         (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

// The same pattern for any associative, commutative operation on 32-bit integers.
template <typename F>
__device__ __forceinline__ int wave_reduce_i32(int v, F f) {
  v = f(v, dpp_i32<kDppQuadXor1>(v));
  v = f(v, dpp_i32<kDppQuadXor2>(v));
  v = f(v, dpp_i32<kDppRowHalfMirror>(v));
  v = f(v, dpp_i32<kDppRowMirror>(v));
  return f(f(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
           f(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// Sum over the whole 256-thread work-group, returned to every thread.  One barrier; `lds`
// (kWaves doubles) must not be reused by another call before a later barrier.
__device__ __forceinline__ double block_sum_f64(double v, double* lds) {
  v = wave_sum_f64(v);
  if ((threadIdx.x % kWave) == 0) lds[threadIdx.x / kWave] = v;
  __syncthreads();
  return (lds[0] + lds[1]) + (lds[2] + lds[3]);
}

// Sum of `v` over aligned segments of `seg` consecutive threads (seg a power of two,
// 1 <= seg <= 256); every thread receives the sum of its own segment.  `lds` points to at
// least kWaves doubles of shared memory that no one else uses across the call.
// Contains barriers when seg > 64: every thread of the work-group must call it.
__device__ __forceinline__ double segment_sum(double v, int seg, double* lds) {
  const int lim = seg < kWave ? seg : kWave;
  for (int off = 1; off < lim; off <<= 1) v += shfl_xor_f64(v, off);
  if (seg > kWave) {
    const int wave = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x % kWave) == 0) lds[wave] = v;
    __syncthreads();
    const int wps = seg / kWave;              // waves per segment: 2 or 4
    const int w0 = wave & ~(wps - 1);
    double t = lds[w0];
    for (int k = 1; k < wps; ++k) t += lds[w0 + k];
    v = t;
  }
  return v;
}

__device__ __forceinline__ uint32_t segment_sum_u32(uint32_t v, int seg, uint32_t* lds) {
  const int lim = seg < kWave ? seg : kWave;
  for (int off = 1; off < lim; off <<= 1) v += __shfl_xor(v, off, kWave);
  if (seg > kWave) {
    const int wave = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x % kWave) == 0) lds[wave] = v;
    __syncthreads();
    const int wps = seg / kWave;
    const int w0 = wave & ~(wps - 1);
    uint32_t t = lds[w0];
    for (int k = 1; k < wps; ++k) t += lds[w0 + k];
    v = t;
  }
  return v;
}

// This thread's share of part[i0 .. i1): elements i0 + threadIdx.x + k*256, sixteen loads in
// flight at a time (a fixed order: the result does not depend on scheduling).  These sums run
// in a single work-group per bucket, so the number of dependent rounds of loads is their time.
constexpr int kPartialLoads = 16;
// For the kernels that call them: one or two waves per SIMD is all they ever run at, and saying so
// keeps the compiler from serialising the loads to save registers (it did: one load, one wait).
#define QA_FEW_WAVES __attribute__((amdgpu_waves_per_eu(1, 2)))
__device__ __forceinline__ double fold_partials(const double (&acc)[kPartialLoads]) {
  double r[kPartialLoads / 2];
#pragma unroll
  for (int u = 0; u < kPartialLoads / 2; ++u) r[u] = acc[2 * u] + acc[2 * u + 1];
#pragma unroll
  for (int w = kPartialLoads / 4; w >= 1; w /= 2)
#pragma unroll
    for (int u = 0; u < w; ++u) r[u] = r[2 * u] + r[2 * u + 1];
  return r[0];
}
template <typename T>
__device__ __forceinline__ double strided_partial_sum(const T* __restrict__ part, int64_t i0,
                                                      int64_t i1) {
  double acc[kPartialLoads];
#pragma unroll
  for (int u = 0; u < kPartialLoads; ++u) acc[u] = 0.0;
  int64_t i = i0 + threadIdx.x;
  for (; i + (kPartialLoads - 1) * kThreads < i1; i += kPartialLoads * kThreads) {
    T v[kPartialLoads];
#pragma unroll
    for (int u = 0; u < kPartialLoads; ++u) v[u] = part[i + u * kThreads];
#pragma unroll
    for (int u = 0; u < kPartialLoads; ++u) acc[u] += (double)v[u];
  }
  for (; i < i1; i += kThreads) acc[0] += (double)part[i];
  return fold_partials(acc);
}
// The same for a pair of arrays (sums and counts of the same tiles), their loads interleaved.
template <typename T, typename U>
__device__ __forceinline__ void strided_partial_sums(const T* __restrict__ pa, const U* __restrict__ pb,
                                                     int64_t i0, int64_t i1, double* sa, double* sb) {
  double acc[kPartialLoads], bcc[kPartialLoads];
#pragma unroll
  for (int u = 0; u < kPartialLoads; ++u) { acc[u] = 0.0; bcc[u] = 0.0; }
  int64_t i = i0 + threadIdx.x;
  for (; i + (kPartialLoads - 1) * kThreads < i1; i += kPartialLoads * kThreads) {
    T v[kPartialLoads];
    U w[kPartialLoads];
#pragma unroll
    for (int u = 0; u < kPartialLoads; ++u) { v[u] = pa[i + u * kThreads]; w[u] = pb[i + u * kThreads]; }
#pragma unroll
    for (int u = 0; u < kPartialLoads; ++u) { acc[u] += (double)v[u]; bcc[u] += (double)w[u]; }
  }
  for (; i < i1; i += kThreads) { acc[0] += (double)pa[i]; bcc[0] += (double)pb[i]; }
  *sa = fold_partials(acc);
  *sb = fold_partials(bcc);
}

// Threshold and scale from the binary64 sums, rounded once (Sections 3.4-3.5).
__device__ __forceinline__ float threshold_from_sum(double S1, float thr_coef, int64_t n) {
  return (float)(((double)thr_coef * S1) / (double)n);
}
__device__ __forceinline__ float scale_from_sum(double S2, uint64_t cnt) {
  return cnt ? (float)(S2 / (double)cnt) : 0.0f;
}

// Ternary code as the 2-bit field 00 / 01 / 11; NaN compares false on both sides -> 00.
__device__ __forceinline__ uint32_t ternary_field(float v, float Delta) {
  return v > Delta ? 1u : (v < -Delta ? 3u : 0u);
}

#endif  // __HIPCC__

}  // namespace qa

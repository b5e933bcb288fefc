// Exact least-squares threshold (Section 3.4: rank the magnitudes and try each one as the
// threshold) for buckets longer than one 4096-tile and for one threshold over a whole vector.
// The per-tile form (an in-register ranking network) lives with the quantizer; this is the
// device-wide form for gfx950, used by qa_quantize_pack with QA_THRESH_EXACT when a bucket spans
// tiles.  Not on the method's hot path: Section 3.5 introduces the 0.75 mean|v| rule precisely to
// avoid this ranking.
//
// Per worker:
//   1. 64-bit keys (bucket index << 31 | 0x7fffffff - bits(|v|)) are sorted in ascending order
//      with the library's device radix sort: buckets stay in place (bucket k's keys end up in
//      positions [k b, min((k+1) b, d)) again) and inside a bucket the magnitudes descend.  The
//      keys are formed on the fly from the gradient by the sort's input iterator.
//   2. tile sums of the sorted magnitudes (binary64) -> exclusive scan over each bucket's tiles ->
//      per position k the sum of the k largest, the objective (sum)^2 / k for every k that does not
//      split equal magnitudes and keeps no zero -> arg max (smallest k among equal objectives) per
//      tile, then per bucket.
//   3. the threshold written is the largest magnitude NOT kept, sorted[k*] (0 if everything
//      non-zero is kept or the bucket is all zero), to be compared with strictly.
// The quantizer's ordinary passes then run with these thresholds given.
//
// The sums of the k largest are associated tile by tile here and strictly left to right in a plain
// loop; where two candidates' objectives agree to within that rounding difference (about 1e-16
// relative) the two may pick different k.  For n components the objectives of neighbouring k near
// the optimum differ by about 1/k^2 relative, so this becomes likely beyond some 1e7 components per
// bucket and is not a matter of correctness: both kept sets are optimal to binary64 resolution.
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/iterator/counting_iterator.hpp>
#include <rocprim/iterator/transform_iterator.hpp>

#include "qa_common.h"

namespace qa {

// Key = (bucket index << 31) | (0x7fffffff - bits(|v|)); with a single bucket (one threshold for
// the whole vector) the bucket index is 0 and the key type is 32 bits wide: half the bytes in
// every pass of the sort.
template <typename K>
struct SortKeyOf {
  const float* g;
  int shift;                                             // log2(bucket); 62 for one bucket
  __host__ __device__ K operator()(int64_t i) const {
    uint32_t u;
    const float v = g[i];
    memcpy(&u, &v, 4);
    const uint32_t low = 0x7fffffffu - (u & 0x7fffffffu);
    if (sizeof(K) == 4) return (K)low;
    return (K)(((uint64_t)(i >> shift) << 31) | (uint64_t)low);
  }
};

template <typename K>
struct ExactArgs {
  const K* keys;                                         // sorted
  int64_t d, ntiles, nb, tiles_per_bucket, bucket_len;   // bucket_len = d for one bucket
  double* tsum;                                          // per tile: sum of its magnitudes
  double* tbase;                                         // per tile: sum of the bucket's magnitudes before it
  double* tobj;                                          // per tile: best objective (-1: no candidate)
  int64_t* tk;                                           // per tile: its k (count kept, within the bucket)
  float* thresholds;                                     // this worker's row
};

template <typename K>
__device__ __forceinline__ float magnitude_of(K key) {
  return __uint_as_float(0x7fffffffu - ((uint32_t)key & 0x7fffffffu));
}

// every thread receives the sum over the threads before it; *total = sum over the work-group
__device__ __forceinline__ double block_exclusive_scan_f64(double v, double* lds, double* total) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  double incl = v;
  for (int off = 1; off < kWave; off <<= 1) {
    const double o = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += o;
  }
  __syncthreads();                                       // earlier readers of lds are done
  if (lane == kWave - 1) lds[wave] = incl;
  __syncthreads();
  double before = 0.0, all = 0.0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) before += lds[w];
    all += lds[w];
  }
  *total = all;
  return before + (incl - v);
}

// (obj, k) with the largest obj, the smallest k among equal obj, over the work-group, to thread 0
__device__ __forceinline__ bool better(double o2, int64_t k2, double o, int64_t k) {
  return o2 > o || (o2 == o && k2 < k);
}
__device__ __forceinline__ void block_argmax(double& obj, int64_t& k, double* lds_o, int64_t* lds_k) {
  for (int off = 1; off < kWave; off <<= 1) {
    const double o2 = __shfl_xor(obj, off, kWave);
    const int64_t k2 = (int64_t)__shfl_xor((long long)k, off, kWave);
    if (better(o2, k2, obj, k)) { obj = o2; k = k2; }
  }
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  __syncthreads();
  if (lane == 0) { lds_o[wave] = obj; lds_k[wave] = k; }
  __syncthreads();
  obj = lds_o[0]; k = lds_k[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w)
    if (better(lds_o[w], lds_k[w], obj, k)) { obj = lds_o[w]; k = lds_k[w]; }
}

template <typename K>
__global__ __launch_bounds__(kThreads) void exact_tile_sum_kernel(ExactArgs<K> a) {
  __shared__ double lds_d[kWaves];
  const int64_t tile = blockIdx.x;
  const int64_t i0 = tile * kTile + 16 * (int64_t)threadIdx.x;
  double s = 0.0;
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if (i0 + j < a.d) s += (double)magnitude_of(a.keys[i0 + j]);
  s = block_sum_f64(s, lds_d);
  if (threadIdx.x == 0) a.tsum[tile] = s;
}

// one work-group per bucket: tbase[tile] = sum of tsum over the bucket's earlier tiles, in tile order
template <typename K>
__global__ __launch_bounds__(kThreads) void exact_scan_kernel(ExactArgs<K> a) {
  __shared__ double lds_d[kWaves];
  const int64_t t0 = (int64_t)blockIdx.x * a.tiles_per_bucket;
  const int64_t t1 = t0 + a.tiles_per_bucket < a.ntiles ? t0 + a.tiles_per_bucket : a.ntiles;
  constexpr int kRun = 8;
  double running = 0.0;
  for (int64_t i = t0; i < t1; i += (int64_t)kThreads * kRun) {
    const int64_t j0 = i + (int64_t)threadIdx.x * kRun;
    double c[kRun], mine = 0.0;
#pragma unroll
    for (int u = 0; u < kRun; ++u) {
      c[u] = j0 + u < t1 ? a.tsum[j0 + u] : 0.0;
      mine += c[u];
    }
    double total;
    double ex = block_exclusive_scan_f64(mine, lds_d, &total);
#pragma unroll
    for (int u = 0; u < kRun; ++u) {
      if (j0 + u < t1) a.tbase[j0 + u] = running + ex;
      ex += c[u];
    }
    running += total;
  }
}

// per tile: the best candidate k among its positions
template <typename K>
__global__ __launch_bounds__(kThreads) void exact_objective_kernel(ExactArgs<K> a) {
  __shared__ double lds_d[kWaves];
  __shared__ double lds_o[kWaves];
  __shared__ int64_t lds_k[kWaves];
  const int64_t tile = blockIdx.x;
  const int64_t kb = tile / a.tiles_per_bucket;
  const int64_t lo = kb * a.bucket_len;                                      // the bucket
  const int64_t hi = lo + a.bucket_len < a.d ? lo + a.bucket_len : a.d;
  const int64_t i0 = tile * kTile + 16 * (int64_t)threadIdx.x;
  float m[17];                                           // the thread's 16 magnitudes and the one after
#pragma unroll
  for (int j = 0; j < 17; ++j) m[j] = i0 + j < hi ? magnitude_of(a.keys[i0 + j]) : -1.0f;
  double p[16], run = 0.0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    run += i0 + j < hi ? (double)m[j] : 0.0;
    p[j] = run;
  }
  double total;
  const double before = a.tbase[tile] + block_exclusive_scan_f64(run, lds_d, &total);
  double best = -1.0;
  int64_t best_k = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    // keeping the k largest is a candidate if the k-th is non-zero and differs from the (k+1)-th
    // (m[j + 1] is -1 past the bucket's end: the last position always qualifies)
    const int64_t k = i0 + j + 1 - lo;
    if (i0 + j < hi && m[j] > 0.0f && m[j + 1] != m[j]) {
      const double s = before + p[j];
      const double obj = s * s / (double)k;
      if (obj > best) { best = obj; best_k = k; }
    }
  }
  block_argmax(best, best_k, lds_o, lds_k);
  if (threadIdx.x == 0) { a.tobj[tile] = best; a.tk[tile] = best_k; }
}

// per bucket: the best tile's k, and the largest magnitude not kept
template <typename K>
__global__ __launch_bounds__(kThreads) void exact_pick_kernel(ExactArgs<K> a) {
  __shared__ double lds_o[kWaves];
  __shared__ int64_t lds_k[kWaves];
  const int64_t kb = blockIdx.x;
  const int64_t t0 = kb * a.tiles_per_bucket;
  const int64_t t1 = t0 + a.tiles_per_bucket < a.ntiles ? t0 + a.tiles_per_bucket : a.ntiles;
  double best = -1.0;
  int64_t best_k = 0;
  for (int64_t i = t0 + threadIdx.x; i < t1; i += kThreads) {
    const double o = a.tobj[i];
    const int64_t k = a.tk[i];
    if (o >= 0.0 && better(o, k, best, best_k)) { best = o; best_k = k; }
  }
  block_argmax(best, best_k, lds_o, lds_k);
  if (threadIdx.x == 0) {
    const int64_t lo = kb * a.bucket_len;
    const int64_t hi = lo + a.bucket_len < a.d ? lo + a.bucket_len : a.d;
    float Delta = 0.0f;
    if (best >= 0.0 && lo + best_k < hi) Delta = magnitude_of(a.keys[lo + best_k]);
    a.thresholds[kb] = Delta;
  }
}

static inline size_t xalign(size_t v) { return (v + 255) & ~size_t(255); }

static bool bucket_spans_tiles(const qa_layout* L) {
  return L->bucket == 0 ? tiles_of(L->d) > 1 : L->bucket > kTile;
}

// Bytes this file's passes need beyond the quantizer's own workspace: sorted keys, the per-tile
// arrays and the sort's temporary storage (another buffer of keys plus its histograms; measured
// 8.17 bytes per key, declared here as 9 bytes per key plus 4 MiB and checked against the sort's
// own figure at the call).
size_t exact_sort_workspace_bytes(const qa_layout* L) {
  if (!bucket_spans_tiles(L)) return 0;
  const size_t d = (size_t)L->d, nt = (size_t)tiles_of(L->d);
  return xalign(d * 8) + 4 * xalign(nt * 8) + xalign(d * 8 + d + (size_t(4) << 20));
}

template <typename K>
static int exact_sorted_run(const qa_layout* L, const float* g, int64_t g_stride, float* thresholds,
                            void* ws, size_t ws_bytes, hipStream_t stream) {
  const size_t d = (size_t)L->d, nt = (size_t)tiles_of(L->d);
  char* p = static_cast<char*>(ws);
  K* keys = reinterpret_cast<K*>(p);  p += xalign(d * 8);
  ExactArgs<K> a{};
  a.keys = keys; a.d = L->d; a.ntiles = (int64_t)nt; a.nb = buckets_of(L->d, L->bucket);
  a.bucket_len = L->bucket ? L->bucket : L->d;
  a.tiles_per_bucket = L->bucket ? L->bucket / kTile : (int64_t)nt;
  a.tsum = reinterpret_cast<double*>(p);   p += xalign(nt * 8);
  a.tbase = reinterpret_cast<double*>(p);  p += xalign(nt * 8);
  a.tobj = reinterpret_cast<double*>(p);   p += xalign(nt * 8);
  a.tk = reinterpret_cast<int64_t*>(p);    p += xalign(nt * 8);
  void* temp = p;
  const size_t temp_have = ws_bytes - (size_t)(p - static_cast<char*>(ws));
  const int shift = L->bucket ? ilog2(L->bucket) : 62;
  const unsigned end_bit = 31u + (unsigned)(a.nb > 1 ? ilog2(a.nb) : 0);
  const dim3 block(kThreads);
  for (int m = 0; m < L->M; ++m) {
    auto in = rocprim::make_transform_iterator(rocprim::counting_iterator<int64_t>(0),
                                               SortKeyOf<K>{g + (int64_t)m * g_stride, shift});
    size_t temp_need = 0;
    if (rocprim::radix_sort_keys(nullptr, temp_need, in, keys, d, 0u, end_bit, stream) != hipSuccess)
      return QA_ERR_LAUNCH;
    if (temp_need > temp_have) return QA_ERR_WORKSPACE;
    if (rocprim::radix_sort_keys(temp, temp_need, in, keys, d, 0u, end_bit, stream) != hipSuccess)
      return QA_ERR_LAUNCH;
    a.thresholds = thresholds + (int64_t)m * L->scale_stride;
    hipLaunchKernelGGL(exact_tile_sum_kernel<K>, dim3((unsigned)nt), block, 0, stream, a);
    hipLaunchKernelGGL(exact_scan_kernel<K>, dim3((unsigned)a.nb), block, 0, stream, a);
    hipLaunchKernelGGL(exact_objective_kernel<K>, dim3((unsigned)nt), block, 0, stream, a);
    hipLaunchKernelGGL(exact_pick_kernel<K>, dim3((unsigned)a.nb), block, 0, stream, a);
  }
  return launch_status();
}

int exact_thresholds_sorted(const qa_layout* L, const float* g, int64_t g_stride, float* thresholds,
                            void* ws, size_t ws_bytes, hipStream_t stream) {
  if (!bucket_spans_tiles(L)) return QA_ERR_INVALID_ARG;
  if (L->d >= (int64_t(1) << 32)) return QA_ERR_TOO_LARGE;
  if (!ws || ws_bytes < exact_sort_workspace_bytes(L) || !aligned(ws, 256)) return QA_ERR_WORKSPACE;
  if (buckets_of(L->d, L->bucket) == 1)
    return exact_sorted_run<uint32_t>(L, g, g_stride, thresholds, ws, ws_bytes, stream);
  return exact_sorted_run<uint64_t>(L, g, g_stride, thresholds, ws, ws_bytes, stream);
}

}  // namespace qa

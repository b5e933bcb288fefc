// Threshold quantizer + 2-bit encoding (Sections 3.4-3.5 of arXiv 2208.05631) for gfx950.
//
// Tile = 4096 elements of one worker's gradient per 256-thread work-group.  Thread t holds
// four float4 groups f = j*256 + t (j = 0..3), i.e. elements 4f..4f+3 of the tile, so that
// every global load instruction of a wave reads 1 KiB of consecutive memory.
//
//   bucket <= 4096 : one kernel; sums, threshold, scale and codes of a tile's buckets are
//                    formed in registers/LDS; the gradient is read once (4 B/elem + 0.25 B out).
//   bucket  > 4096 or 0 (whole vector): tile partial sums -> finalize threshold -> codes and
//                    tile partial (count, sum) -> finalize scale; the gradient is read twice.
#include <mutex>

#include "qa_common.h"

namespace qa {

struct QuantArgs {
  const float* g;
  int64_t g_stride;
  int64_t d;
  int64_t W;               // ceil(d/16)
  uint32_t* codes;
  int64_t code_stride;
  float* scales;
  float* thresholds;       // user array, may be null
  int64_t scale_stride;
  int log2b;               // log2(bucket); unused when bucket == 0
  float thr_coef;
  int thresh_given;
  // two-pass path
  double* part_sum;        // [M][ntiles]
  uint32_t* part_cnt;      // [M][ntiles]
  float* thr_ws;           // [M][nb]
  int64_t ntiles;
  int64_t tiles_per_bucket;  // ntiles when bucket == 0
  int64_t nb;
  int64_t bucket_len;        // elements per bucket (d when bucket == 0)
};

// Load the thread's 4 float4 groups of tile `tile`; elements at or beyond d read as +0.
__device__ __forceinline__ void load_tile(const float* __restrict__ g, int64_t d, int64_t tile,
                                          float v[4][4]) {
  const int64_t base = tile * kTile;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t i = base + (int64_t)(j * kThreads + (int)threadIdx.x) * 4;
    if (i + 3 < d) {
      const float4 q = *reinterpret_cast<const float4*>(g + i);
      v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[j][e] = (i + e < d) ? g[i + e] : 0.0f;
    }
  }
}

// The same with streaming (non-temporal) loads for tiles that lie wholly below d: for passes after
// which the element is not needed again soon.
__device__ __forceinline__ void load_tile_stream(const float* __restrict__ g, int64_t d, int64_t tile,
                                                 float v[4][4]) {
  if ((tile + 1) * kTile <= d) {
    typedef float floatx4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const floatx4 q = __builtin_nontemporal_load(
          reinterpret_cast<const floatx4*>(g + tile * kTile + (j * kThreads + (int)threadIdx.x) * 4));
      v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
    }
  } else {
    load_tile(g, d, tile, v);
  }
}

// Ternary fields of the thread's 16 elements -> the four code words of its quad (group j of
// lanes 4q..4q+3 is code word j*64 + t/4 of the tile); lane (t & 3) == j stores word j.
__device__ __forceinline__ void pack_and_store(const float v[4][4], const float Delta[4],
                                               uint32_t* __restrict__ codes_m, int64_t tile,
                                               int64_t W) {
  const int t = threadIdx.x;
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t b = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) b |= ternary_field(v[j][e], Delta[j]) << (2 * e);
    uint32_t w = b << (8 * (t & 3));
    w |= (uint32_t)dpp_i32<kDppQuadXor1>((int)w);
    w |= (uint32_t)dpp_i32<kDppQuadXor2>((int)w);
    if ((t & 3) == j) mine = w;
  }
  const int64_t widx = tile * kTileWords + (t & 3) * 64 + (t >> 2);
  if (widx < W) codes_m[widx] = mine;
}

__device__ __forceinline__ void kept_sums(const float v[4], float Delta, double* s_out,
                                          uint32_t* c_out) {
  double s = 0.0;
  uint32_t c = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float av = fabsf(v[e]);
    if (av > Delta) { s += (double)av; ++c; }
  }
  *s_out = s; *c_out = c;
}

// ---- 64 <= bucket < 4096 : single pass, several buckets per tile --------------------------------
//
// Slice j of the tile (elements j*1024 .. j*1024+1023) is held four elements per thread, so a
// bucket of b <= 1024 elements is SEG = b/4 consecutive threads of one slice, and a bucket of 2048
// is two whole slices.  Sums over 16 lanes use DPP, 32 and 64 lanes one more cross-row step, and
// larger segments one LDS exchange for all four slices at once: no barrier for b <= 256, one per
// phase otherwise.  Every thread receives the sums of its own buckets.
template <int SEG>
__device__ __forceinline__ double lanes_sum_f64(double v) {
  v += dpp_f64<kDppQuadXor1>(v);
  v += dpp_f64<kDppQuadXor2>(v);
  v += dpp_f64<kDppRowHalfMirror>(v);
  v += dpp_f64<kDppRowMirror>(v);                        // sum of the row of 16
  if (SEG == 32) v += shfl_xor_f64(v, 16);
  if (SEG >= 64)
    v = (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
  return v;
}
template <int SEG>
__device__ __forceinline__ uint32_t lanes_sum_u32(uint32_t v) {
  v += (uint32_t)dpp_i32<kDppQuadXor1>((int)v);
  v += (uint32_t)dpp_i32<kDppQuadXor2>((int)v);
  v += (uint32_t)dpp_i32<kDppRowHalfMirror>((int)v);
  v += (uint32_t)dpp_i32<kDppRowMirror>((int)v);
  if (SEG == 32) v += (uint32_t)__shfl_xor((int)v, 16, kWave);
  if (SEG >= 64)
    v = (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
        (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return v;
}

// s[j], c[j]: this thread's part of slice j -> the sums over its bucket.  LOG2B = log2(bucket).
// lds: 16 doubles and 16 words nobody else uses; the caller's threads all take part.
template <int LOG2B, bool WITH_COUNT>
__device__ __forceinline__ void bucket_sums(double s[4], uint32_t c[4], double* lds_s, uint32_t* lds_c) {
  constexpr int SEG = LOG2B >= 10 ? 256 : (1 << LOG2B) / 4;     // threads per bucket within a slice
  constexpr int LANES = SEG < 64 ? SEG : 64;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    s[j] = lanes_sum_f64<LANES>(s[j]);
    if (WITH_COUNT) c[j] = lanes_sum_u32<LANES>(c[j]);
  }
  if (SEG > 64) {
    const int wave = threadIdx.x / kWave;
    __syncthreads();                                     // earlier readers of lds are done
    if ((threadIdx.x % kWave) == 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lds_s[j * kWaves + wave] = s[j];
        if (WITH_COUNT) lds_c[j * kWaves + wave] = c[j];
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (SEG == 128) {                                  // waves {0,1} and {2,3}
        const int w0 = wave & ~1;
        s[j] = lds_s[j * kWaves + w0] + lds_s[j * kWaves + w0 + 1];
        if (WITH_COUNT) c[j] = lds_c[j * kWaves + w0] + lds_c[j * kWaves + w0 + 1];
      } else {
        s[j] = (lds_s[j * kWaves] + lds_s[j * kWaves + 1]) + (lds_s[j * kWaves + 2] + lds_s[j * kWaves + 3]);
        if (WITH_COUNT)
          c[j] = lds_c[j * kWaves] + lds_c[j * kWaves + 1] + lds_c[j * kWaves + 2] + lds_c[j * kWaves + 3];
      }
    }
    if (LOG2B == 11) {                                   // a bucket is two slices
      const double s01 = s[0] + s[1], s23 = s[2] + s[3];
      s[0] = s[1] = s01; s[2] = s[3] = s23;
      if (WITH_COUNT) {
        const uint32_t c01 = c[0] + c[1], c23 = c[2] + c[3];
        c[0] = c[1] = c01; c[2] = c[3] = c23;
      }
    }
  }
}

template <int LOG2B>
__global__ __launch_bounds__(kThreads) void quantize_bucket_kernel(QuantArgs a) {
  __shared__ double lds_s[4 * kWaves];
  __shared__ uint32_t lds_c[4 * kWaves];
  constexpr int b = 1 << LOG2B;
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const float* g = a.g + (int64_t)m * a.g_stride;
  const int t = threadIdx.x;
  const bool whole = (tile + 1) * kTile <= a.d;          // the vector does not end inside the tile

  float v[4][4];
  if (whole) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      typedef float floatx4 __attribute__((ext_vector_type(4)));
      const floatx4 q = __builtin_nontemporal_load(
          reinterpret_cast<const floatx4*>(g + tile * kTile + (j * kThreads + t) * 4));
      v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
    }
  } else {
    load_tile(g, a.d, tile, v);
  }
  float Delta[4];
  const int64_t k0 = tile * (kTile >> LOG2B);            // first bucket of the tile
  int kb[4];                                             // bucket of slice j within the tile
#pragma unroll
  for (int j = 0; j < 4; ++j) kb[j] = ((j * kThreads + t) * 4) >> LOG2B;

  if (!a.thresh_given) {
    double S1[4];
    uint32_t unused[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      S1[j] = (double)fabsf(v[j][0]);
#pragma unroll
      for (int e = 1; e < 4; ++e) S1[j] += (double)fabsf(v[j][e]);
    }
    bucket_sums<LOG2B, false>(S1, unused, lds_s, lds_c);
    // Every bucket of the tile is complete unless the vector ends inside the tile; dividing by
    // the power of two b is then an exact scaling, the same value as the division.
    if (whole) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        Delta[j] = (float)(((double)a.thr_coef * S1[j]) * (1.0 / (double)b));
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t lo = (k0 + kb[j]) << LOG2B;
        const int64_t n = (a.d - lo) < (int64_t)b ? (a.d - lo) : (int64_t)b;   // true length
        Delta[j] = n > 0 ? threshold_from_sum(S1[j], a.thr_coef, n) : 0.0f;
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      Delta[j] = k0 + kb[j] < a.nb ? a.thresholds[(int64_t)m * a.scale_stride + k0 + kb[j]] : 0.0f;
  }

  // kept sums, counts and 2-bit fields; for Delta >= 0 the field of a kept element is
  // 01 | sign << 1, a negative (given) threshold takes the two plain comparisons
  double S2[4];
  uint32_t C[4];
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const bool plain = Delta[j] < 0.0f;
    double s2 = 0.0;
    uint32_t c = 0, bits = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float av = fabsf(v[j][e]);
      const bool keep = av > Delta[j];
      s2 += (double)(keep ? av : 0.0f);
      c += keep ? 1u : 0u;
      const uint32_t pat = 1u | ((__float_as_uint(v[j][e]) >> 30) & 2u);
      const uint32_t f = plain ? ternary_field(v[j][e], Delta[j]) : (keep ? pat : 0u);
      bits |= f << (2 * e);
    }
    S2[j] = s2; C[j] = c;
    uint32_t w = bits << (8 * (t & 3));
    w |= (uint32_t)dpp_i32<kDppQuadXor1>((int)w);
    w |= (uint32_t)dpp_i32<kDppQuadXor2>((int)w);
    if ((t & 3) == j) mine = w;
  }
  {
    const int64_t widx = tile * kTileWords + (t & 3) * 64 + (t >> 2);
    if (widx < a.W) (a.codes + (int64_t)m * a.code_stride)[widx] = mine;
  }
  bucket_sums<LOG2B, true>(S2, C, lds_s, lds_c);

  // The thread holding a bucket's first element hands (sum, count, threshold) of the bucket to
  // LDS; thread k of the work-group then divides for bucket k of the tile, so that a wave runs
  // the binary64 division once instead of once per slice.
  constexpr int kBucketsPerTile = kTile >> LOG2B;
  __shared__ double out_s[kBucketsPerTile];
  __shared__ uint32_t out_c[kBucketsPerTile];
  __shared__ float out_d[kBucketsPerTile];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e0 = (j * kThreads + t) * 4;               // first element of this thread in slice j
    if ((e0 & (b - 1)) == 0) {
      out_s[e0 >> LOG2B] = S2[j]; out_c[e0 >> LOG2B] = C[j]; out_d[e0 >> LOG2B] = Delta[j];
    }
  }
  __syncthreads();
  if (t < kBucketsPerTile) {
    const int64_t k = tile * kBucketsPerTile + t;
    if (k < a.nb) {
      a.scales[(int64_t)m * a.scale_stride + k] = scale_from_sum(out_s[t], out_c[t]);
      if (a.thresholds && !a.thresh_given) a.thresholds[(int64_t)m * a.scale_stride + k] = out_d[t];
    }
  }
}

// ---- bucket == 4096 == the tile : single pass, two work-group reductions ---------------------

// Kept-magnitude sum, kept count (wave-wide, from the compare masks on the scalar unit) and the
// 2-bit fields of one float4 group.  For Delta >= 0 (always, unless a caller hands in a negative
// threshold)  v > Delta or v < -Delta  <=>  |v| > Delta, and the field is 01 | sign << 1.
__device__ __forceinline__ uint32_t quantize4(const float v[4], float Delta, bool plain_compare,
                                              double& s2, uint32_t& wave_cnt) {
  uint32_t b = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float av = fabsf(v[e]);
    const bool keep = av > Delta;
    wave_cnt += (uint32_t)__popcll(__ballot(keep));
    s2 += (double)(keep ? av : 0.0f);
    uint32_t f;
    if (plain_compare) {
      f = ternary_field(v[e], Delta);
    } else {
      const uint32_t pat = 1u | ((__float_as_uint(v[e]) >> 30) & 2u);
      f = keep ? pat : 0u;
    }
    b |= f << (2 * e);
  }
  return b;
}

__global__ __launch_bounds__(kThreads) void quantize_tile_kernel(QuantArgs a) {
  __shared__ double lds_s1[kWaves];
  __shared__ double lds_s2[kWaves];
  __shared__ uint32_t lds_c[kWaves];
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const int t = threadIdx.x;
  const int64_t lo = tile * kTile;
  const float* g = a.g + (int64_t)m * a.g_stride;
  float v[4][4];
  if (lo + kTile <= a.d) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // the gradient is read exactly once: nontemporal
      typedef float floatx4 __attribute__((ext_vector_type(4)));
      const floatx4 q = __builtin_nontemporal_load(
          reinterpret_cast<const floatx4*>(g + lo + (j * kThreads + t) * 4));
      v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
    }
  } else {
    load_tile(g, a.d, tile, v);
  }

  float Delta;
  if (!a.thresh_given) {
    double sj[4];                                        // four independent chains
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      sj[j] = (double)fabsf(v[j][0]);
#pragma unroll
      for (int e = 1; e < 4; ++e) sj[j] += (double)fabsf(v[j][e]);
    }
    const double S1 = block_sum_f64((sj[0] + sj[1]) + (sj[2] + sj[3]), lds_s1);
    const int64_t n = (a.d - lo) < (int64_t)kTile ? (a.d - lo) : (int64_t)kTile;
    Delta = threshold_from_sum(S1, a.thr_coef, n);
  } else {
    Delta = a.thresholds[(int64_t)m * a.scale_stride + tile];
  }
  const bool plain_compare = Delta < 0.0f;               // uniform; only with a given threshold

  double s2j[4] = {0.0, 0.0, 0.0, 0.0};
  uint32_t wave_cnt = 0;
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t b = quantize4(v[j], Delta, plain_compare, s2j[j], wave_cnt);
    uint32_t w = b << (8 * (t & 3));
    w |= (uint32_t)dpp_i32<kDppQuadXor1>((int)w);
    w |= (uint32_t)dpp_i32<kDppQuadXor2>((int)w);
    if ((t & 3) == j) mine = w;
  }
  const int64_t widx = tile * kTileWords + (t & 3) * 64 + (t >> 2);
  if (widx < a.W) (a.codes + (int64_t)m * a.code_stride)[widx] = mine;

  const double s2 = wave_sum_f64((s2j[0] + s2j[1]) + (s2j[2] + s2j[3]));
  if ((t % kWave) == 0) { lds_s2[t / kWave] = s2; lds_c[t / kWave] = wave_cnt; }
  __syncthreads();
  if (t == 0) {
    const double S2 = (lds_s2[0] + lds_s2[1]) + (lds_s2[2] + lds_s2[3]);
    const uint32_t C = lds_c[0] + lds_c[1] + lds_c[2] + lds_c[3];
    a.scales[(int64_t)m * a.scale_stride + tile] = scale_from_sum(S2, C);
    if (a.thresholds && !a.thresh_given) a.thresholds[(int64_t)m * a.scale_stride + tile] = Delta;
  }
}

// ---- exact optimal threshold by ranking (Section 3.4: the magnitudes are sorted and each one
//      is tried as the threshold) for one 4096-tile ----------------------------------------------
//
// |v| of the tile is sorted in descending order (bitonic network on the bit patterns, which
// order like the non-negative floats), prefix sums are formed in binary64, and the k that
// maximises (sum of the k largest)^2 / k is taken among the k that do not split equal
// magnitudes.  The threshold written is the largest magnitude NOT kept (0 if none), to be
// compared with strictly like the approximate one.
//
// The network runs on 16 keys per thread held in registers.  Position i of the 4096 has 12 bits;
// a thread owns the 16 positions that differ in four of them ("free" bits) and the other eight
// come from its thread index.  Three ownerships cover every stage: free bits 0-3, 4-7 or 8-11.
// A stage that exchanges across bit b is done by the ownership whose free bits hold b, as a
// register min/max; keys move between ownerships through LDS (two buffers, used alternately, so
// one barrier per move is enough: a buffer is rewritten only after the barrier that follows
// every thread's last read of it).  Rows of 16 are padded to 17 words against bank conflicts.
constexpr int kSortPitch = kTile + kTile / 16;

template <int OWN> __device__ __forceinline__ int sort_position(int t, int r) {
  if (OWN == 0) return t * 16 + r;
  if (OWN == 1) return (t & 15) | (r << 4) | ((t >> 4) << 8);
  return t | (r << 8);
}

// The stages of phase P (blocks of 2^P positions, alternately descending and ascending) that
// exchange across the lowest NST free bits of ownership OWN, highest first.  A block that must
// come out ascending is sorted descending on complemented keys.  FLIP: complement here, around
// the stages (phases 1-4, where the block bit is a compile-time bit of r or t & 1); otherwise the
// caller keeps the keys of ascending blocks complemented for the whole phase (an exchange never
// leaves its block, so a key's state stays right for the position it moves to).
template <int OWN, int P, int NST, bool FLIP>
__device__ __forceinline__ void sort_stages(uint32_t (&e)[16], int t) {
  if (FLIP) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      e[r] ^= (uint32_t)(-((sort_position<OWN>(t, r) >> P) & 1));
  }
#pragma unroll
  for (int lb = NST - 1; lb >= 0; --lb)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (!(r & (1 << lb))) {
        const uint32_t x = e[r], y = e[r | (1 << lb)];
        e[r] = x > y ? x : y;
        e[r | (1 << lb)] = x > y ? y : x;
      }
  if (FLIP) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      e[r] ^= (uint32_t)(-((sort_position<OWN>(t, r) >> P) & 1));
  }
}

template <int FROM, int TO>
__device__ __forceinline__ void sort_move(uint32_t (&e)[16], int t, uint32_t* buf) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = sort_position<FROM>(t, r);
    buf[i + (i >> 4)] = e[r];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = sort_position<TO>(t, r);
    e[r] = buf[i + (i >> 4)];
  }
}

// Phase P of the network for P >= 5, entered and left in ownership 0 (positions 16t + r: the
// block bit P is bit P-4 of t, the same for the thread's 16 keys).  On entry the keys carry the
// complement state of phase P-1 (PREV_FLIPPED) or none; they leave in the state of phase P, which
// for the last phase is "none" (FINAL: every block of 2^P comes out descending; for P = 12 that
// is the one block there is).  n counts the moves made so far and picks the buffer.
template <int P, bool PREV_FLIPPED, bool FINAL>
__device__ __forceinline__ void sort_phase(uint32_t (&e)[16], int t, uint32_t (*buf)[kSortPitch],
                                           int& n) {
  {
    const uint32_t now = FINAL ? 0u : (t >> (P - 4)) & 1u, before = PREV_FLIPPED ? (t >> (P - 5)) & 1u : 0u;
    const uint32_t m = (uint32_t)(-(int)(now ^ before));
#pragma unroll
    for (int r = 0; r < 16; ++r) e[r] ^= m;
  }
  if constexpr (P > 8) {
    sort_move<0, 2>(e, t, buf[n++ & 1]);
    sort_stages<2, P, P - 8, false>(e, t);
    sort_move<2, 1>(e, t, buf[n++ & 1]);
    sort_stages<1, P, 4, false>(e, t);
  } else {
    sort_move<0, 1>(e, t, buf[n++ & 1]);
    sort_stages<1, P, P - 4, false>(e, t);
  }
  sort_move<1, 0>(e, t, buf[n++ & 1]);
  sort_stages<0, P, 4, false>(e, t);
}

// LOG2B: log2 of the bucket (6..12): the network stops after phase LOG2B, which leaves every
// bucket of the tile sorted on its own; the prefix sums and the search then run per bucket, over
// the 2^(LOG2B-4) consecutive threads that hold it.
template <int LOG2B>
__global__ __launch_bounds__(kThreads) void exact_threshold_kernel(QuantArgs a) {
  static_assert(LOG2B >= 6 && LOG2B <= 12, "bucket of 64 .. 4096 components");
  constexpr int kSeg = 1 << (LOG2B - 4);                 // threads per bucket
  constexpr int kSegLanes = kSeg < kWave ? kSeg : kWave; // ... of them inside one wave
  constexpr int kSegWaves = kSeg / kSegLanes;            // waves per bucket: 1, 2 or 4
  __shared__ uint32_t buf[2][kSortPitch];
  __shared__ uint32_t lds_first[kThreads];
  __shared__ double lds_tot[kWaves];
  __shared__ double lds_obj[kWaves];
  __shared__ int lds_k[kWaves];
  __shared__ float lds_next[kWaves];
  const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  uint32_t e[16];                 // which 16 of the tile a thread starts with does not matter
  {
    float v[4][4];
    load_tile(a.g + (int64_t)m * a.g_stride, a.d, tile, v);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int c = 0; c < 4; ++c) e[j * 4 + c] = __float_as_uint(fabsf(v[j][c]));
  }
  // load_tile hands thread t the float4 groups j*256 + t, i.e. components of up to four buckets
  // when the bucket is smaller than the tile: bring every key to ownership 0 (positions
  // 16t .. 16t+15) first, so that a thread's keys and every later exchange stay inside a bucket
  int n = 0;
  if constexpr (LOG2B < 12) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = ((r >> 2) * kThreads + t) * 4 + (r & 3);
      buf[0][i + (i >> 4)] = e[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = 16 * t + r;
      e[r] = buf[0][i + (i >> 4)];
    }
    n = 1;
  }
  sort_stages<0, 1, 1, true>(e, t);
  sort_stages<0, 2, 2, true>(e, t);
  sort_stages<0, 3, 3, true>(e, t);
  sort_stages<0, 4, 4, true>(e, t);
  sort_phase<5, false, false>(e, t, buf, n);
  sort_phase<6, true, LOG2B == 6>(e, t, buf, n);
  if constexpr (LOG2B >= 7) sort_phase<7, true, LOG2B == 7>(e, t, buf, n);
  if constexpr (LOG2B >= 8) sort_phase<8, true, LOG2B == 8>(e, t, buf, n);
  if constexpr (LOG2B >= 9) sort_phase<9, true, LOG2B == 9>(e, t, buf, n);
  if constexpr (LOG2B >= 10) sort_phase<10, true, LOG2B == 10>(e, t, buf, n);
  if constexpr (LOG2B >= 11) sort_phase<11, true, LOG2B == 11>(e, t, buf, n);
  if constexpr (LOG2B >= 12) sort_phase<12, true, true>(e, t, buf, n);
  // the thread now holds positions 16t .. 16t+15 of the tile, each bucket in descending order
  const int ts = t & (kSeg - 1);                         // this thread's place among its bucket's threads
  lds_first[t] = e[0];
  __syncthreads();
  float av[17];
#pragma unroll
  for (int j = 0; j < 16; ++j) av[j] = __uint_as_float(e[j]);
  av[16] = ts < kSeg - 1 ? __uint_as_float(lds_first[t + 1]) : 0.0f;
  double run[16];
  run[0] = (double)av[0];
#pragma unroll
  for (int j = 1; j < 16; ++j) run[j] = run[j - 1] + (double)av[j];
  double incl = run[15];
#pragma unroll
  for (int off = 1; off < kSegLanes; off <<= 1) {
    const double o = __shfl_up(incl, off, kWave);
    if ((lane & (kSegLanes - 1)) >= off) incl += o;
  }
  double before = incl - run[15];
  if constexpr (kSegWaves > 1) {
    if (lane == kWave - 1) lds_tot[wave] = incl;
    __syncthreads();
    for (int w = wave & ~(kSegWaves - 1); w < wave; ++w) before += lds_tot[w];
  }
  // best candidate of this thread (smallest k among equal objectives); k = 0: none
  double best = -1.0;
  int best_k = 0;
  float best_next = 0.0f;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int k = 16 * ts + j + 1;
    if (av[j] > 0.0f && av[j] > av[j + 1]) {
      const double r = before + run[j];
      const double obj = r * r / (double)k;
      if (obj > best) { best = obj; best_k = k; best_next = av[j + 1]; }
    }
  }
#pragma unroll
  for (int off = 1; off < kSegLanes; off <<= 1) {
    const double o = __shfl_xor(best, off, kWave);
    const int ok = __shfl_xor(best_k, off, kWave);
    const float on = __shfl_xor(best_next, off, kWave);
    if (o > best || (o == best && ok < best_k)) { best = o; best_k = ok; best_next = on; }
  }
  if constexpr (kSegWaves > 1) {
    if (lane == 0) { lds_obj[wave] = best; lds_k[wave] = best_k; lds_next[wave] = best_next; }
    __syncthreads();
    if (ts == 0)
      for (int w = wave + 1; w < wave + kSegWaves; ++w) {
        const double o = lds_obj[w];
        const int ok = lds_k[w];
        if (o > best || (o == best && ok < best_k)) { best = o; best_k = ok; best_next = lds_next[w]; }
      }
  }
  if (ts == 0) {
    const int64_t k = tile * (kTile >> LOG2B) + (t >> (LOG2B - 4));   // bucket index
    if (k < a.nb) a.thresholds[(int64_t)m * a.scale_stride + k] = best_k > 0 ? best_next : 0.0f;
  }
}

// ---- bucket > 4096 or whole vector : two passes -----------------------------------------------

// pass 1: part_sum[m][tile] = sum |v| over the tile
__global__ __launch_bounds__(kThreads) void quantize_abs_partial_kernel(QuantArgs a) {
  __shared__ double lds_d[kWaves];
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  float v[4][4];
  // streaming: the second pass over the gradient comes after all of it has gone by
  load_tile_stream(a.g + (int64_t)m * a.g_stride, a.d, tile, v);
  double s = 0.0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) s += (double)fabsf(v[j][e]);
  s = block_sum_f64(s, lds_d);
  if (threadIdx.x == 0) a.part_sum[(int64_t)m * a.ntiles + tile] = s;
}

// finalize 1: one work-group per (bucket, worker): threshold from the tile partials
__global__ __launch_bounds__(kThreads) QA_FEW_WAVES void quantize_threshold_finalize_kernel(QuantArgs a) {
  __shared__ double lds_d[kWaves];
  const int64_t k = blockIdx.x;
  const int m = blockIdx.y;
  const int64_t t0 = k * a.tiles_per_bucket;
  const int64_t t1 = (t0 + a.tiles_per_bucket) < a.ntiles ? (t0 + a.tiles_per_bucket) : a.ntiles;
  double s = strided_partial_sum(a.part_sum + (int64_t)m * a.ntiles, t0, t1);
  s = segment_sum(s, kThreads, lds_d);
  if (threadIdx.x == 0) {
    const int64_t lo = k * a.bucket_len;
    const int64_t n = (a.d - lo) < a.bucket_len ? (a.d - lo) : a.bucket_len;
    const float Delta = threshold_from_sum(s, a.thr_coef, n);
    a.thr_ws[(int64_t)m * a.nb + k] = Delta;
    if (a.thresholds) a.thresholds[(int64_t)m * a.scale_stride + k] = Delta;
  }
}

// pass 2: codes of the tile and its partial (count, sum) of kept magnitudes
__global__ __launch_bounds__(kThreads) void quantize_codes_partial_kernel(QuantArgs a) {
  __shared__ double lds_d[kWaves];
  __shared__ uint32_t lds_u[kWaves];
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const int64_t k = tile / a.tiles_per_bucket;
  const float D = a.thresh_given ? a.thresholds[(int64_t)m * a.scale_stride + k]
                                 : a.thr_ws[(int64_t)m * a.nb + k];
  float v[4][4];
  load_tile_stream(a.g + (int64_t)m * a.g_stride, a.d, tile, v);
  double s = 0.0;
  uint32_t c = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    double sj; uint32_t cj;
    kept_sums(v[j], D, &sj, &cj);
    s += sj; c += cj;
  }
  s = wave_sum_f64(s);
  c = wave_sum_u32(c);
  if ((threadIdx.x % kWave) == 0) { lds_d[threadIdx.x / kWave] = s; lds_u[threadIdx.x / kWave] = c; }
  const float Delta[4] = {D, D, D, D};
  pack_and_store(v, Delta, a.codes + (int64_t)m * a.code_stride, tile, a.W);
  __syncthreads();
  if (threadIdx.x == 0) {
    a.part_sum[(int64_t)m * a.ntiles + tile] = (lds_d[0] + lds_d[1]) + (lds_d[2] + lds_d[3]);
    a.part_cnt[(int64_t)m * a.ntiles + tile] = lds_u[0] + lds_u[1] + lds_u[2] + lds_u[3];
  }
}

// finalize 2: scale of each (bucket, worker)
__global__ __launch_bounds__(kThreads) QA_FEW_WAVES void quantize_scale_finalize_kernel(QuantArgs a) {
  __shared__ double lds_d[kWaves];
  __shared__ double lds_c[kWaves];
  const int64_t k = blockIdx.x;
  const int m = blockIdx.y;
  const int64_t t0 = k * a.tiles_per_bucket;
  const int64_t t1 = (t0 + a.tiles_per_bucket) < a.ntiles ? (t0 + a.tiles_per_bucket) : a.ntiles;
  // counts are integers < 2^53: exact in binary64
  double s, c;
  strided_partial_sums(a.part_sum + (int64_t)m * a.ntiles, a.part_cnt + (int64_t)m * a.ntiles, t0, t1, &s, &c);
  s = segment_sum(s, kThreads, lds_d);
  c = segment_sum(c, kThreads, lds_c);
  if (threadIdx.x == 0)
    a.scales[(int64_t)m * a.scale_stride + k] = scale_from_sum(s, (uint64_t)c);
}

// ---- stochastic ternary quantizer (TernGrad: max-norm scale, keep probability |v|/s) ----------
//
// Uniform numbers: Philox4x32-10 keyed by the 64-bit seed, counter (j low, j high, worker, step)
// with j the index of the float4 group, so one generator call serves the four components of a
// group (component i takes output word i % 4).  u = (r >> 8) * 2^-24; keep iff u < |v| / s with
// the division in binary32.  The max is exact, so its reduction order is free.

struct StochArgs {
  QuantArgs q;
  uint32_t seed_lo, seed_hi, step;
  int pass;                 // two-pass path: 0 = bucket max, 1 = codes
};

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;      // one 32x32->64 multiply each
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ float tile_abs_max(const float v[4][4]) {
  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) { const float a = fabsf(v[j][e]); s = a > s ? a : s; }   // NaN never wins
  return s;
}

__device__ __forceinline__ float wave_max_f32(float s) {
  float o;
  o = __int_as_float(dpp_i32<kDppQuadXor1>(__float_as_int(s))); s = o > s ? o : s;
  o = __int_as_float(dpp_i32<kDppQuadXor2>(__float_as_int(s))); s = o > s ? o : s;
  o = __int_as_float(dpp_i32<kDppRowHalfMirror>(__float_as_int(s))); s = o > s ? o : s;
  o = __int_as_float(dpp_i32<kDppRowMirror>(__float_as_int(s))); s = o > s ? o : s;
  float r = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), 0));
#pragma unroll
  for (int l = 16; l < 64; l += 16) {
    o = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), l));
    r = o > r ? o : r;
  }
  return r;
}

// codes of the tile, float4 group j of every thread with scale sj[j]; element (j, e) of thread t
// is vector index base + 4*(j*256+t)+e
__device__ __forceinline__ void stochastic_codes(const StochArgs& a, const float v[4][4],
                                                 const float sj[4], int64_t tile, int m) {
  const int t = threadIdx.x;
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float s = sj[j];
    const float rs = __builtin_amdgcn_rcpf(s);
    const uint64_t grp = (uint64_t)tile * (kTile / 4) + (uint64_t)(j * kThreads + t);
    uint32_t r[4];
    philox4x32_10((uint32_t)grp, (uint32_t)(grp >> 32), (uint32_t)m, a.step, a.seed_lo, a.seed_hi, r);
    // keep iff u < fl(|v| / s).  The hardware reciprocal gives |v|/s to a few ulp; only when u
    // lies within that margin of it (probability ~1e-6) is the correctly rounded quotient needed.
    float u[4], av[4];
    bool keep[4], unsure = false;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      u[e] = (float)(r[e] >> 8) * 0x1p-24f;
      av[e] = fabsf(v[j][e]);
      const float pa = av[e] * rs;
      const float lo = pa * 0.999999f, hi = pa * 1.000001f;
      keep[e] = u[e] < lo;
      unsure |= !(u[e] < lo) && !(u[e] > hi);            // also NaN/Inf products
    }
    if (__any(unsure)) {
#pragma unroll
      for (int e = 0; e < 4; ++e) keep[e] = u[e] < av[e] / s;
    }
    uint32_t b = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) b |= (keep[e] ? (v[j][e] < 0.0f ? 3u : 1u) : 0u) << (2 * e);
    uint32_t w = b << (8 * (t & 3));
    w |= (uint32_t)dpp_i32<kDppQuadXor1>((int)w);
    w |= (uint32_t)dpp_i32<kDppQuadXor2>((int)w);
    if ((t & 3) == j) mine = w;
  }
  const int64_t widx = tile * kTileWords + (t & 3) * 64 + (t >> 2);
  if (widx < a.q.W) (a.q.codes + (int64_t)m * a.q.code_stride)[widx] = mine;
}

// bucket == tile (4096, or one scale per vector with d <= 4096): one pass
__global__ __launch_bounds__(kThreads) void quantize_stochastic_tile_kernel(StochArgs a) {
  __shared__ float lds_m[kWaves];
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  float v[4][4];
  load_tile_stream(a.q.g + (int64_t)m * a.q.g_stride, a.q.d, tile, v);
  float s = wave_max_f32(tile_abs_max(v));
  if ((threadIdx.x % kWave) == 0) lds_m[threadIdx.x / kWave] = s;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) s = lds_m[w] > s ? lds_m[w] : s;
  if (threadIdx.x == 0) a.q.scales[(int64_t)m * a.q.scale_stride + tile] = s;
  const float sj[4] = {s, s, s, s};
  stochastic_codes(a, v, sj, tile, m);
}

// Maximum over aligned segments of `seg` consecutive threads (a power of two, 16 <= seg <= 256);
// every thread receives its segment's maximum.  Barriers when seg > 64: all threads must call.
__device__ __forceinline__ float segment_max_f32(float v, int seg, float* lds) {
  const int lim = seg < kWave ? seg : kWave;
  for (int off = 1; off < lim; off <<= 1) {
    const float o = __shfl_xor(v, off, kWave);
    v = o > v ? o : v;
  }
  if (seg > kWave) {
    const int wave = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x % kWave) == 0) lds[wave] = v;
    __syncthreads();
    const int wps = seg / kWave, w0 = wave & ~(wps - 1);
    float r = lds[w0];
    for (int k = 1; k < wps; ++k) r = lds[w0 + k] > r ? lds[w0 + k] : r;
    v = r;
  }
  return v;
}

// buckets of 64 .. 2048 elements: float4 group f = j*256 + t of the tile lies in the tile's bucket
// f / (bucket/4), so a bucket is a segment of bucket/4 consecutive threads of one j (two j's for
// 2048).  Not tuned: one segmented maximum per j.
__global__ __launch_bounds__(kThreads) void quantize_stochastic_bucket_kernel(StochArgs a) {
  __shared__ float lds_m[kWaves];
  const int t = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  float v[4][4];
  load_tile_stream(a.q.g + (int64_t)m * a.q.g_stride, a.q.d, tile, v);
  const int groups = (int)(a.q.bucket_len / 4);          // float4 groups per bucket: 16 .. 512
  const int seg = groups < kThreads ? groups : kThreads;
  float sj[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float s = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) { const float av = fabsf(v[j][e]); s = av > s ? av : s; }
    sj[j] = segment_max_f32(s, seg, lds_m);
  }
  if (groups > kThreads) {                               // 2048: j = 0,1 and j = 2,3 share a bucket
    const float lo = sj[0] > sj[1] ? sj[0] : sj[1], hi = sj[2] > sj[3] ? sj[2] : sj[3];
    sj[0] = sj[1] = lo; sj[2] = sj[3] = hi;
  }
  if ((t & (seg - 1)) == 0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int f = j * kThreads + t;
      if (f % groups == 0) {
        const int64_t kb = tile * (kTile / a.q.bucket_len) + f / groups;
        if (kb < a.q.nb) a.q.scales[(int64_t)m * a.q.scale_stride + kb] = sj[j];
      }
    }
  }
  stochastic_codes(a, v, sj, tile, m);
}

// bucket > 4096 or one scale per large vector: pass 0 folds tile maxima into scales[] (which
// the host zeroed) with integer atomic max on the bit pattern of the non-negative float;
// pass 1 reads the finished scale and writes the codes.
__global__ __launch_bounds__(kThreads) void quantize_stochastic_twopass_kernel(StochArgs a) {
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const int64_t k = tile / a.q.tiles_per_bucket;
  float v[4][4];
  load_tile_stream(a.q.g + (int64_t)m * a.q.g_stride, a.q.d, tile, v);
  float* sc = a.q.scales + (int64_t)m * a.q.scale_stride + k;
  if (a.pass == 0) {
    const float s = wave_max_f32(tile_abs_max(v));
    if ((threadIdx.x % kWave) == 0) atomicMax(reinterpret_cast<unsigned int*>(sc), __float_as_uint(s));
  } else {
    const float s = *sc;
    const float sj[4] = {s, s, s, s};
    stochastic_codes(a, v, sj, tile, m);
  }
}

__global__ __launch_bounds__(kThreads) void zero_scales_kernel(float* scales, int64_t stride, int64_t nb) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < nb) scales[(int64_t)blockIdx.y * stride + k] = 0.0f;
}

// ---- host side -------------------------------------------------------------------------------

static inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t exact_sort_workspace_bytes(const qa_layout* L);
int exact_thresholds_sorted(const qa_layout* L, const float* g, int64_t g_stride, float* thresholds,
                            void* ws, size_t ws_bytes, hipStream_t stream);

size_t quantize_workspace_bytes(const qa_layout* L) {
  if (L->bucket != 0 && L->bucket <= kTile) return 0;
  if (L->bucket == 0 && tiles_of(L->d) == 1) return 0;   // one tile: one pass
  const int64_t nt = tiles_of(L->d), nb = buckets_of(L->d, L->bucket);
  return align256((size_t)L->M * nt * sizeof(double)) + align256((size_t)L->M * nt * sizeof(uint32_t)) +
         align256((size_t)L->M * nb * sizeof(float));
}

// Where the multi-pass quantizer keeps its per-tile sums, counts and per-bucket thresholds inside
// its workspace (all worker-major).
void quantize_workspace_parts(const qa_layout* L, void* ws, double** part_sum, uint32_t** part_cnt,
                              float** thr) {
  char* p = static_cast<char*>(ws);
  const int64_t nt = tiles_of(L->d);
  *part_sum = reinterpret_cast<double*>(p);
  p += align256((size_t)L->M * nt * sizeof(double));
  *part_cnt = reinterpret_cast<uint32_t*>(p);
  p += align256((size_t)L->M * nt * sizeof(uint32_t));
  *thr = reinterpret_cast<float*>(p);
}

int quantize_launch(const qa_layout* L, const float* g, int64_t g_stride, uint32_t* codes,
                    float* scales, float* thresholds, uint32_t flags, void* ws, size_t ws_bytes,
                    hipStream_t stream) {
  QuantArgs a{};
  a.g = g; a.g_stride = g_stride; a.d = L->d; a.W = words_of(L->d);
  a.codes = codes; a.code_stride = L->code_stride;
  a.scales = scales; a.thresholds = thresholds; a.scale_stride = L->scale_stride;
  a.thr_coef = L->thr_coef;
  a.thresh_given = (flags & QA_THRESH_GIVEN) ? 1 : 0;
  a.ntiles = tiles_of(L->d);
  a.nb = buckets_of(L->d, L->bucket);
  const dim3 block(kThreads);
  if (a.ntiles > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  const dim3 grid_tiles((unsigned)a.ntiles, (unsigned)L->M);
  const bool one_pass = (L->bucket != 0 && L->bucket <= kTile) || (L->bucket == 0 && a.ntiles == 1);
  if ((flags & QA_THRESH_EXACT) && !one_pass) {
    // buckets that span tiles: device-wide ranking, in the part of the workspace that follows
    // the multi-pass quantizer's own
    const size_t own = quantize_workspace_bytes(L), more = exact_sort_workspace_bytes(L);
    if (!ws || ws_bytes < own + more) return QA_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
    const int rc = exact_thresholds_sorted(L, g, g_stride, thresholds, static_cast<char*>(ws) + own,
                                           ws_bytes - own, stream);
    if (rc != QA_OK) return rc;
    a.thresh_given = 1;                                  // the passes below read what it wrote
  } else if (flags & QA_THRESH_EXACT) {
    // one ranking network per tile: buckets that fit a tile
    switch (L->bucket ? ilog2(L->bucket) : 12) {
      case 6: hipLaunchKernelGGL(exact_threshold_kernel<6>, grid_tiles, block, 0, stream, a); break;
      case 7: hipLaunchKernelGGL(exact_threshold_kernel<7>, grid_tiles, block, 0, stream, a); break;
      case 8: hipLaunchKernelGGL(exact_threshold_kernel<8>, grid_tiles, block, 0, stream, a); break;
      case 9: hipLaunchKernelGGL(exact_threshold_kernel<9>, grid_tiles, block, 0, stream, a); break;
      case 10: hipLaunchKernelGGL(exact_threshold_kernel<10>, grid_tiles, block, 0, stream, a); break;
      case 11: hipLaunchKernelGGL(exact_threshold_kernel<11>, grid_tiles, block, 0, stream, a); break;
      default: hipLaunchKernelGGL(exact_threshold_kernel<12>, grid_tiles, block, 0, stream, a); break;
    }
    a.thresh_given = 1;                                  // the passes below read what it wrote
  }

  if (L->bucket != 0 && L->bucket <= kTile) {
    a.log2b = ilog2(L->bucket);
    a.bucket_len = L->bucket;
    switch (a.log2b) {
      case 6: hipLaunchKernelGGL(quantize_bucket_kernel<6>, grid_tiles, block, 0, stream, a); break;
      case 7: hipLaunchKernelGGL(quantize_bucket_kernel<7>, grid_tiles, block, 0, stream, a); break;
      case 8: hipLaunchKernelGGL(quantize_bucket_kernel<8>, grid_tiles, block, 0, stream, a); break;
      case 9: hipLaunchKernelGGL(quantize_bucket_kernel<9>, grid_tiles, block, 0, stream, a); break;
      case 10: hipLaunchKernelGGL(quantize_bucket_kernel<10>, grid_tiles, block, 0, stream, a); break;
      case 11: hipLaunchKernelGGL(quantize_bucket_kernel<11>, grid_tiles, block, 0, stream, a); break;
      default: hipLaunchKernelGGL(quantize_tile_kernel, grid_tiles, block, 0, stream, a); break;
    }
    return launch_status();
  }
  if (L->bucket == 0 && a.ntiles == 1) {                 // the whole vector is one tile: one pass
    a.log2b = ilog2(kTile);
    a.bucket_len = kTile;
    hipLaunchKernelGGL(quantize_tile_kernel, grid_tiles, block, 0, stream, a);
    return launch_status();
  }

  const size_t need = quantize_workspace_bytes(L);
  if (!ws || ws_bytes < need) return QA_ERR_WORKSPACE;
  if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
  quantize_workspace_parts(L, ws, &a.part_sum, &a.part_cnt, &a.thr_ws);
  a.bucket_len = L->bucket ? L->bucket : L->d;
  a.tiles_per_bucket = L->bucket ? L->bucket / kTile : a.ntiles;
  a.log2b = L->bucket ? ilog2(L->bucket) : 0;
  const dim3 grid_buckets((unsigned)a.nb, (unsigned)L->M);

  if (!a.thresh_given) {
    if (!(flags & kQuantAbsPartialsGiven))
      hipLaunchKernelGGL(quantize_abs_partial_kernel, grid_tiles, block, 0, stream, a);
    hipLaunchKernelGGL(quantize_threshold_finalize_kernel, grid_buckets, block, 0, stream, a);
  }
  hipLaunchKernelGGL(quantize_codes_partial_kernel, grid_tiles, block, 0, stream, a);
  hipLaunchKernelGGL(quantize_scale_finalize_kernel, grid_buckets, block, 0, stream, a);
  return launch_status();
}

// The multi-pass quantizer's finalize kernels alone, for a producer that leaves the partial sums in
// the quantizer's workspace itself and never materialises the quantizer's input (the steps that
// form Q(SynQ) from the messages).  which = 0: thresholds from the partial sums of |v| (also
// written to thresholds[] if given); which = 1: scales from the partial sums and counts of the
// kept |v|.  n_partials = 0: one partial per 4096-tile, as the quantizer's own passes leave them;
// otherwise the layout must have a single bucket, whose n_partials partials (each over some whole
// tiles, in order) are at the start of the arrays.
int quantize_finalize_launch(const qa_layout* L, int which, int64_t n_partials, float* scales,
                             float* thresholds, void* ws, size_t ws_bytes, hipStream_t stream) {
  const size_t need = quantize_workspace_bytes(L);
  if (need == 0 || !ws || ws_bytes < need) return QA_ERR_WORKSPACE;   // (need == 0: a one-pass layout)
  if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
  QuantArgs a{};
  a.d = L->d; a.W = words_of(L->d);
  a.scales = scales; a.thresholds = thresholds; a.scale_stride = L->scale_stride;
  a.thr_coef = L->thr_coef;
  a.ntiles = tiles_of(L->d);
  a.nb = buckets_of(L->d, L->bucket);
  quantize_workspace_parts(L, ws, &a.part_sum, &a.part_cnt, &a.thr_ws);
  a.bucket_len = L->bucket ? L->bucket : L->d;
  a.tiles_per_bucket = L->bucket ? L->bucket / kTile : a.ntiles;
  if (n_partials != 0) {
    if (a.nb != 1 || n_partials < 1 || n_partials > a.ntiles || L->M != 1) return QA_ERR_INVALID_ARG;
    a.ntiles = n_partials; a.tiles_per_bucket = n_partials;
  }
  const dim3 grid_buckets((unsigned)a.nb, (unsigned)L->M), block(kThreads);
  if (which == 0) hipLaunchKernelGGL(quantize_threshold_finalize_kernel, grid_buckets, block, 0, stream, a);
  else hipLaunchKernelGGL(quantize_scale_finalize_kernel, grid_buckets, block, 0, stream, a);
  return launch_status();
}

// ---- scratch that the library owns, for callers that cannot hand over a workspace -------------
//
// The multi-pass quantizer keeps per-tile partial sums, counts and the thresholds between its
// launches.  qa_quantize_pack_static keeps them in this array instead of a caller's workspace.
// Every GPU the library runs on holds its own copy until the process ends; its device address
// is looked up once per device and that address (never the symbol itself) is what host code
// hands to the kernels.
constexpr size_t kScratchBytes = size_t(4) << 20;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[kMaxDevices];    // device address of `scratch` on each GPU, 0 = not yet asked

// Address of the current device's copy of `scratch`.
static int scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return QA_ERR_LAUNCH;
  }
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return QA_ERR_LAUNCH;
    }
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return QA_OK;
}

}  // namespace qa

extern "C" int qa_quantize_pack_static(const qa_layout* layout, const float* g, int64_t g_stride,
                                       uint32_t* codes, float* scales, float* thresholds,
                                       uint32_t flags, void* stream) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  if (!g || !codes || !scales) return QA_ERR_INVALID_ARG;
  if (flags & ~(QA_THRESH_GIVEN | QA_THRESH_EXACT)) return QA_ERR_INVALID_ARG;
  if ((flags & QA_THRESH_GIVEN) && (flags & QA_THRESH_EXACT)) return QA_ERR_INVALID_ARG;
  if ((flags & (QA_THRESH_GIVEN | QA_THRESH_EXACT)) && !thresholds) return QA_ERR_INVALID_ARG;
  if (g_stride < layout->d || (g_stride % 4) != 0) return QA_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(codes, 4) || !aligned(scales, 4) || !aligned(thresholds, 4))
    return QA_ERR_ALIGNMENT;
  const size_t need = quantize_workspace_bytes(layout);
  if (need > kScratchBytes) return QA_ERR_TOO_LARGE;
  // the device-wide ranking needs a sort's worth of scratch: not from this array
  if ((flags & QA_THRESH_EXACT) && exact_sort_workspace_bytes(layout) != 0) return QA_ERR_TOO_LARGE;
  void* ws = nullptr;
  if (need) {
    rc = scratch_address(&ws);
    if (rc != QA_OK) return rc;
  }
  // every partial that a later launch reads is written by an earlier launch of the same call:
  // nothing in the array has to start at zero
  return quantize_launch(layout, g, g_stride, codes, scales, thresholds, flags, ws,
                         need ? kScratchBytes : 0, static_cast<hipStream_t>(stream));
}

extern "C" int qa_quantize_pack(const qa_layout* layout, const float* g, int64_t g_stride,
                                uint32_t* codes, float* scales, float* thresholds, uint32_t flags,
                                void* ws, size_t ws_bytes, void* stream) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  if (!g || !codes || !scales) return QA_ERR_INVALID_ARG;
  if (flags & ~(QA_THRESH_GIVEN | QA_THRESH_EXACT)) return QA_ERR_INVALID_ARG;
  if ((flags & QA_THRESH_GIVEN) && (flags & QA_THRESH_EXACT)) return QA_ERR_INVALID_ARG;
  if ((flags & (QA_THRESH_GIVEN | QA_THRESH_EXACT)) && !thresholds) return QA_ERR_INVALID_ARG;
  if (g_stride < layout->d || (g_stride % 4) != 0) return QA_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(codes, 4) || !aligned(scales, 4) || !aligned(thresholds, 4))
    return QA_ERR_ALIGNMENT;
  return quantize_launch(layout, g, g_stride, codes, scales, thresholds, flags, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

extern "C" int qa_quantize_pack_stochastic(const qa_layout* layout, const float* g, int64_t g_stride,
                                           uint32_t* codes, float* scales, uint64_t seed,
                                           uint32_t step, void* stream_) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  if (!g || !codes || !scales) return QA_ERR_INVALID_ARG;
  if (g_stride < layout->d || (g_stride % 4) != 0) return QA_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(codes, 4) || !aligned(scales, 4)) return QA_ERR_ALIGNMENT;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  StochArgs a{};
  a.q.g = g; a.q.g_stride = g_stride; a.q.d = layout->d; a.q.W = words_of(layout->d);
  a.q.codes = codes; a.q.code_stride = layout->code_stride;
  a.q.scales = scales; a.q.scale_stride = layout->scale_stride;
  a.q.ntiles = tiles_of(layout->d);
  a.q.nb = buckets_of(layout->d, layout->bucket);
  a.seed_lo = (uint32_t)seed; a.seed_hi = (uint32_t)(seed >> 32); a.step = step;
  if (a.q.ntiles > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  const dim3 block(kThreads), grid((unsigned)a.q.ntiles, (unsigned)layout->M);
  if (layout->bucket != 0 && layout->bucket < kTile) {
    a.q.bucket_len = layout->bucket;
    hipLaunchKernelGGL(quantize_stochastic_bucket_kernel, grid, block, 0, stream, a);
    return launch_status();
  }
  if (layout->bucket == kTile || a.q.ntiles == 1) {
    hipLaunchKernelGGL(quantize_stochastic_tile_kernel, grid, block, 0, stream, a);
    return launch_status();
  }
  a.q.tiles_per_bucket = layout->bucket ? layout->bucket / kTile : a.q.ntiles;
  hipLaunchKernelGGL(zero_scales_kernel, dim3((unsigned)((a.q.nb + kThreads - 1) / kThreads),
                                              (unsigned)layout->M), block, 0, stream, scales,
                     layout->scale_stride, a.q.nb);
  a.pass = 0;
  hipLaunchKernelGGL(quantize_stochastic_twopass_kernel, grid, block, 0, stream, a);
  a.pass = 1;
  hipLaunchKernelGGL(quantize_stochastic_twopass_kernel, grid, block, 0, stream, a);
  return launch_status();
}

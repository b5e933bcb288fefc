// Server average and fused QCMD / QRDA adagrad steps (Section 3.2 and Algorithm 1 of
// arXiv 2208.05631) for gfx950.
//
// Tile = 4096 coordinates = 256 code words per 256-thread work-group; thread t owns code
// word t of the tile, i.e. 16 consecutive coordinates, for every worker.  A wave therefore
// reads 256 consecutive bytes of each worker's code stream per load instruction.
// Per coordinate the kernel forms  acc = sum_m s_m * c_m  in binary64 (each product is exact),
// gbar = (float)(acc / M), optionally re-quantizes gbar per bucket inside the tile, and applies
// the accumulator + closed-form update, touching x, G (and z) exactly once.
// The same kernel also takes its code words from sparse-encoded messages (expanded on the fly)
// and, in aggregate mode with the second quantization, emits q_t as a coded message.
// A second quantization whose buckets span tiles takes several launches (of this kernel, or of
// requant_sums_kernel when every message has one scale) with the quantizer's finalize kernels
// in between: see step_common.
#include <cmath>
#include <cstring>

#include "qa_segments.h"
#include "qa_sparse.h"

namespace qa {

enum StepMode { kAggregate = 0, kQcmd = 1, kQrda = 2 };
// The second quantization q = Q(SynQ): none; formed inside the kernel (buckets that fit the tile);
// or with the threshold and scale of each bucket handed in (buckets that span tiles and one
// scale per vector, whose sums earlier launches of the same kernel have left in the workspace).
enum Requant { kRqNone = 0, kRqInTile = 1, kRqGiven = 2 };

struct StepArgs {
  const uint32_t* codes;
  const float* scales;
  int64_t code_stride, scale_stride;
  int64_t d, W;
  int M;
  int log2b;          // log2(bucket), or -1 for one scale per vector
  double inv_M;       // exact 1/M when M is a power of two, unused otherwise
  int M_pow2;
  int tile_uniform;   // all coordinates of a 4096-tile share their scales
  int span_limit;     // max exponent span of a tile's scales for which any order is exact
  float* x; float* G; float* z; float* gbar;
  double* abs_partials;   // aggregate mode, optional: sum of |gbar| of each tile (first pass of a quantizer)
  // Second quantization over buckets of rq_tiles tiles each (kRqGiven; the vector's tiles when it
  // has one scale): threshold and scale of every bucket, and (aggregate mode, optional, instead of
  // gbar) each tile's sum and count of the |gbar| above its bucket's threshold
  const float* rq_thr; const float* rq_scale;
  double* kept_sum; uint32_t* kept_cnt;
  int64_t rq_tiles;
  float eta, lam_eta, delta, t_lam, thr_coef;
  // Tiles whose scales all have biased exponents in [fast_emin, fast_emax] (and pass the span
  // test) may take the short forms of sqrt and division in the update: every numerator and
  // denominator then lies where the full forms do no rescaling (set by set_fast_limits)
  int fast_emin, fast_emax;
  uint32_t fast_r_lo, fast_r_span;   // QRDA: bit patterns bounding the positive r = |z| - t*lambda
  SegTable seg;       // tensor-list launches: work-group = piece, one scale column per tensor
  // sparse-encoded messages (kernels with SPARSE): `codes` holds the compact per-bucket streams,
  // worker m's indicator words start at ind + m*ind_stride (stride 0: one indicator for all)
  const uint32_t* ind;
  int64_t ind_stride;
  // aggregate mode with the second quantization: q_t leaves as a one-worker message instead of gbar
  uint32_t* q_codes;
  float* q_scales;
  float* q_thresholds;   // optional
  uint32_t* ind_syn;     // optional, sparse messages: OR of the workers' indicators
};

// 10 -> 00 so that the reserved pattern reads as zero; 01 and 11 are unchanged.
__device__ __forceinline__ uint32_t sanitize(uint32_t w) {
  const uint32_t lo = w & 0x55555555u;
  return lo | ((w & (lo << 1)));
}

// Accumulator and closed-form update of one coordinate (equations Hq, QCMD, QRDA): binary32,
// one rounding per operation, in this order.  accumulate() forms the new G (and z), solve_x()
// the new parameter from them.
template <int MODE, bool TRACK_Z>
__device__ __forceinline__ void accumulate(float q, float& G, float& z) {
  const float q2 = q * q;
  G = G + q2;
  if (MODE == kQrda || TRACK_Z) z = z + q;
}
// G, z: the values after accumulate(); x: the parameter before the step (QCMD)
template <int MODE>
__device__ __forceinline__ float solve_x(const StepArgs& a, float q, float x, float G, float z) {
  const float H = a.delta + sqrtf(G);
  if (MODE == kQcmd) {
    const float step = (a.eta * q) / H;
    const float u = x - step;
    const float tau = a.lam_eta / H;
    const float r = fabsf(u) - tau;
    return r > 0.0f ? copysignf(r, u) : 0.0f;
  } else {
    const float r = fabsf(z) - a.t_lam;
    const float mag = (a.eta * r) / H;
    return r > 0.0f ? -copysignf(mag, z) : 0.0f;
  }
}
template <int MODE, bool TRACK_Z>
__device__ __forceinline__ void update_coordinate(const StepArgs& a, float q, float& x, float& G,
                                                  float& z) {
  accumulate<MODE, TRACK_Z>(q, G, z);
  x = solve_x<MODE>(a, q, x, G, z);
}

// ---- short forms of the correctly rounded sqrt and division ----------------------------------
//
// The compiler expands binary32 sqrt and division into: rescale the operands if they lie near
// the ends of the exponent range, a hardware estimate, fused corrections, undo the rescaling,
// special values.  For operands well inside the range the rescaling steps do nothing, so the
// same estimate and the same corrections alone give the same, correctly rounded, bits.  The
// functions below are those cores; callers establish the ranges (per tile from the exponents
// of the scales, per lane for what comes from the caller's state) and fall back to the full
// forms otherwise.
//
//   sqrt_core(G)      : G == 0 or 2^-96 <= G < 2^126
//   div_core(a, H, r) : r = recip_core(H), 2^-64 <= H < 2^64, a == 0 or 2^-62 <= |a| < 2^59 with
//                       |a| / H < 2^95 (quotient and reciprocal normal, exponents < 96 apart)
__device__ __forceinline__ float sqrt_core(float G) {
  const float s = __builtin_amdgcn_sqrtf(G);            // within one ulp
  const float down = __int_as_float(__float_as_int(s) - 1);
  const float up = __int_as_float(__float_as_int(s) + 1);
  const float r_down = __builtin_fmaf(-down, s, G);
  const float r_up = __builtin_fmaf(-up, s, G);
  float out = r_down <= 0.0f ? down : s;
  out = r_up > 0.0f ? up : out;
  return out;
}
__device__ __forceinline__ float recip_core(float H) {
  const float r = __builtin_amdgcn_rcpf(H);
  const float e = __builtin_fmaf(-H, r, 1.0f);
  return __builtin_fmaf(e, r, r);
}
__device__ __forceinline__ float div_core(float a, float H, float r) {
  const float q0 = a * r;
  const float e0 = __builtin_fmaf(-H, q0, a);
  const float q1 = __builtin_fmaf(e0, r, q0);
  const float e1 = __builtin_fmaf(-H, q1, a);
  return __builtin_fmaf(e1, r, q1);
}

constexpr uint32_t kBitsTwoToMinus96 = 0x0F800000u;
constexpr uint32_t kBitsTwoTo126 = 0x7E800000u;

// solve_x with the short forms.  `bad` is set when this lane's G (or, for QRDA, its positive r)
// lies outside the ranges above: the caller then discards the result of the whole wave's group
// and takes solve_x instead.
template <int MODE>
__device__ __forceinline__ float solve_x_core(const StepArgs& a, float q, float x, float G, float z,
                                              bool& bad) {
  const uint32_t gb = __float_as_uint(G);
  bad |= (gb - 1u) < (kBitsTwoToMinus96 - 1u);           // 0 < G < 2^-96
  bad |= gb >= kBitsTwoTo126;                           // huge, Inf, NaN, negative
  const float H = a.delta + sqrt_core(G);
  const float rcp = recip_core(H);
  if (MODE == kQcmd) {
    const float step = div_core(a.eta * q, H, rcp);
    const float u = x - step;
    const float tau = div_core(a.lam_eta, H, rcp);
    const float r = fabsf(u) - tau;
    return r > 0.0f ? copysignf(r, u) : 0.0f;
  } else {
    const float r = fabsf(z) - a.t_lam;
    bad |= r > 0.0f && !((__float_as_uint(r) - a.fast_r_lo) < a.fast_r_span);
    const float mag = div_core(a.eta * r, H, rcp);
    return r > 0.0f ? -copysignf(mag, z) : 0.0f;
  }
}

// ---- the step kernel ----------------------------------------------------------------------------
//
// Tile-uniform scales (bucket >= 4096 or one scale per vector): table-driven sum over the workers.
// When the exponents of the non-zero scales of the tile's bucket span few enough binades, every
// partial sum of  sum_m s_m*c_m  is exactly representable in binary64 (all are multiples of
// 2^(e_min-23) and below M*2^(e_max+1)), so the order of the additions does not matter.  The
// kernel then sums workers four at a time: the 2-bit codes of workers 4g..4g+3 for one
// coordinate are gathered into one byte by word-wide bit operations and the byte indexes a
// 256-entry binary64 table (built per tile in LDS) holding the exact partial sum of those four
// workers.  Tiles that fail the span test (or hold Inf/NaN scales) take the ordered loop, and so
// do launches with buckets smaller than the tile (each thread's 16 coordinates share a bucket,
// the tile does not: per-thread scales, second quantization by segmented sums).
//
// The code words of a chunk of workers are requested together, before the scale test and the
// table build; G, x, z (coalesced float4 mapping f = j*256 + t) are requested after the last
// look-up.  Four waves per SIMD cover each other's latencies.
constexpr int kMaxGroups = 4;                           // 16 workers per table set: 8 KiB of LDS

struct State4 { float4 v[4]; };

// Codes are read exactly once and the state is not touched again before the next step:
// both bypass the caches' retention (nontemporal), which measurably raises HBM throughput here.
typedef float floatx4 __attribute__((ext_vector_type(4)));
// One code word per lane through a buffer descriptor: `row` is the same for the whole wave and
// stays in scalar registers (stepping from one worker's row to the next is scalar arithmetic),
// byte_off is this lane's offset, offsets at or beyond row_bytes read as 0.  Streaming
// (non-temporal) access: every code word is read exactly once.
__device__ __forceinline__ uint32_t stream_load(const uint32_t* row, uint32_t byte_off,
                                                uint32_t row_bytes) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(row), 0, (int)row_bytes, 0x00020000 /* 32-bit data, raw addressing */);
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 2 /* nt */);
}
// The same without the streaming hint, for words that several lanes or waves read.
__device__ __forceinline__ uint32_t cached_load(const uint32_t* row, uint32_t byte_off,
                                                uint32_t row_bytes) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(row), 0, (int)row_bytes, 0x00020000);
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0);
}
// A whole tile row of one worker (256 code words) straight into LDS with one instruction of one
// wave, no vector registers involved: lane l brings bytes [16 l, 16 l + 16) of the row to the same
// offsets of lds_row; bytes at or beyond row_bytes arrive as 0.  The data is in LDS once the
// issuing wave's count of outstanding vector-memory operations has reached zero; other waves see
// it after a barrier that follows that.
typedef __attribute__((address_space(3))) void* lds_void_ptr;
__device__ __forceinline__ void stream_row_to_lds(const uint32_t* row, uint32_t row_bytes,
                                                  uint32_t* lds_row) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(row), 0, (int)row_bytes, 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void_ptr)lds_row, 16,
                                           (int)(threadIdx.x % kWave) * 16, 0, 0, 2 /* nt */);
}
__device__ __forceinline__ void wait_vector_memory() {
  __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0), the other counters untouched
}
// Work-group barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for
// outstanding vector-memory operations, so rows on their way into LDS stay in flight across it.
// (A fence would wait for them: to the compiler they are pending writes to LDS.)  The asm
// statement is also a compiler-level memory barrier: no LDS access moves across it.
__device__ __forceinline__ void barrier_lds_only() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ void stream_store4(float* p, const float4& v) {
  floatx4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<floatx4*>(p));
}

// float4 groups j*256+t of the tile; only coordinates in [lo, hi) are touched (lo is a multiple
// of 16), the others read as 0.  full_tile: [lo, hi) is the whole tile.
__device__ __forceinline__ void load_state(const float* __restrict__ p, int64_t tile_base,
                                           int64_t lo, int64_t hi, bool full_tile, State4& s) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t i = tile_base + (int64_t)(j * kThreads + (int)threadIdx.x) * 4;
    if (full_tile || (i >= lo && i + 3 < hi)) {
      const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p + i));
      s.v[j] = make_float4(v.x, v.y, v.z, v.w);
    } else {
      float e[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) e[c] = (i + c >= lo && i + c < hi) ? p[i + c] : 0.0f;
      s.v[j] = make_float4(e[0], e[1], e[2], e[3]);
    }
  }
}

__device__ __forceinline__ void store_state(float* __restrict__ p, int64_t tile_base, int64_t lo,
                                            int64_t hi, bool full_tile, const State4& s) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t i = tile_base + (int64_t)(j * kThreads + (int)threadIdx.x) * 4;
    if (full_tile || (i >= lo && i + 3 < hi)) {
      stream_store4(p + i, s.v[j]);
    } else {
      const float e[4] = {s.v[j].x, s.v[j].y, s.v[j].z, s.v[j].w};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (i + c >= lo && i + c < hi) p[i + c] = e[c];
    }
  }
}

// 8 * (byte R of v): the byte offset of a table entry, in one instruction (shift with a byte
// select on its source).  `three` holds the shift count in a vector register.
template <int R>
__device__ __forceinline__ uint32_t byte_times_8(uint32_t v, uint32_t three) {
  uint32_t out;
  if constexpr (R == 0)
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0"
        : "=v"(out) : "v"(three), "v"(v));
  else if constexpr (R == 1)
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1"
        : "=v"(out) : "v"(three), "v"(v));
  else if constexpr (R == 2)
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2"
        : "=v"(out) : "v"(three), "v"(v));
  else
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3"
        : "=v"(out) : "v"(three), "v"(v));
  return out;
}

// One group of four workers a, b, c, d: gather their codes per coordinate into bytes, look the
// partial sums up, add.  Coordinate 4r+c of the thread's 16 sits in byte r of zq[c].
//
// Index byte of a coordinate: bits 0..3 = "non-zero" bits (low code bits) of a, b, c, d,
// bits 4..7 = their "negative" bits (high code bits).  With 8-byte entries the LDS bank of an
// entry is chosen by the low five index bits, so the all-zero entry and the eight entries with a
// single non-zero worker (the bulk of the look-ups when codes are sparse) lie in different banks,
// except +c/-c and +d/-d which pair up.  With the four 2-bit codes side by side instead, every
// entry of worker d alone would share its bank with the all-zero entry that most lanes read.
// Cost: 8 merges that split the words into low-bit and high-bit pairs, then the 16 merges of a
// 4 x 2-bit gather; then per coordinate one address instruction, one LDS read and one binary64
// addition.
__device__ __forceinline__ void gather_group(uint32_t wa, uint32_t wb, uint32_t wc, uint32_t wd,
                                             uint32_t zq[4]) {
  // field i (bits 2i, 2i+1) of p0 = low bits of (a, b) for coordinate i; p1: (c, d); p2, p3: high bits
  const uint32_t p0 = (wa & 0x55555555u) | ((wb << 1) & 0xAAAAAAAAu);
  const uint32_t p1 = (wc & 0x55555555u) | ((wd << 1) & 0xAAAAAAAAu);
  const uint32_t p2 = ((wa >> 1) & 0x55555555u) | (wb & 0xAAAAAAAAu);
  const uint32_t p3 = ((wc >> 1) & 0x55555555u) | (wd & 0xAAAAAAAAu);
  const uint32_t xe = (p0 & 0x33333333u) | ((p1 << 2) & 0xCCCCCCCCu);
  const uint32_t xo = ((p0 >> 2) & 0x33333333u) | (p1 & 0xCCCCCCCCu);
  const uint32_t ye = (p2 & 0x33333333u) | ((p3 << 2) & 0xCCCCCCCCu);
  const uint32_t yo = ((p2 >> 2) & 0x33333333u) | (p3 & 0xCCCCCCCCu);
  zq[0] = (xe & 0x0F0F0F0Fu) | ((ye << 4) & 0xF0F0F0F0u);
  zq[1] = (xo & 0x0F0F0F0Fu) | ((yo << 4) & 0xF0F0F0F0u);
  zq[2] = ((xe >> 4) & 0x0F0F0F0Fu) | (ye & 0xF0F0F0F0u);
  zq[3] = ((xo >> 4) & 0x0F0F0F0Fu) | (yo & 0xF0F0F0F0u);
}
// the 16 look-ups and additions of one group from its gathered index words
__device__ __forceinline__ void lookup_indices(const uint32_t zq[4], const double* __restrict__ T,
                                               double acc[16]) {
  const uint32_t three = 3u;
  const char* Tb = reinterpret_cast<const char*>(T);
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    acc[c] += *reinterpret_cast<const double*>(Tb + byte_times_8<0>(zq[c], three));
    acc[4 + c] += *reinterpret_cast<const double*>(Tb + byte_times_8<1>(zq[c], three));
    acc[8 + c] += *reinterpret_cast<const double*>(Tb + byte_times_8<2>(zq[c], three));
    acc[12 + c] += *reinterpret_cast<const double*>(Tb + byte_times_8<3>(zq[c], three));
  }
}

// Workers are taken in chunks of 4*G (G groups of four, one table per group).
//   NGT = 4 or 2: G = NGT and M is a multiple of 4*NGT: every chunk is complete, straight-line code.
//   NGT = 0: any M, chunks of 16 workers with run-time guards.
//   NGT = 1: any M, chunks of 4 workers with run-time guards (for M <= 4, e.g. the one-worker
//            message of a separately formed second quantization).
// Chunks of 16 rather than 64 workers, and the state requested only after the look-ups, keep the
// kernel at about 100-120 vector registers, i.e. four waves per SIMD: measured faster than
// holding all 64 code words (and the state) in registers with two waves per SIMD.
//
// SPARSE: the messages arrive in the sparse encoding (indicator + compact stream per 4096-bucket)
// and are expanded to dense code words on the fly, a chunk of workers at a time: a thread's 16
// coordinates are the 16 indicator bits of half an indicator word; the position of its first
// marked component in the bucket's stream is the number of marked components before it (counts of
// two workers share one 32-bit prefix scan over the work-group); the codes are fetched from the
// stream and spread to the marked fields through the deposit table.  The result is the word the
// stand-alone decoder would have written, and everything after it is the dense path.
template <int MODE, bool TRACK_Z, int RQ, int NGT, bool SPARSE = false>
__global__ __launch_bounds__(kThreads) void step_lut_kernel(StepArgs a) {
  constexpr bool REQUANT = RQ == kRqInTile;
  static_assert(!SPARSE || NGT == 0, "sparse input: chunks of 16 workers with guards");
  constexpr bool FULL = NGT > 1;
  constexpr int kGroupsPerChunk = NGT >= 1 ? NGT : kMaxGroups;
  constexpr int kChunk = 4 * kGroupsPerChunk;
  // The server's kernel that sends Q(SynQ) stages complete chunks of code words through LDS (see
  // the loop over chunks below).  It ends before the hand-over of q, so its tables' array is small.
  constexpr bool kStaged = MODE == kAggregate && REQUANT && FULL && !SPARSE;
  constexpr int kTabDoubles = kGroupsPerChunk * 256;
  constexpr int kHandoverDoubles = (MODE == kAggregate && REQUANT) ? 0 : kTile / 2;
  constexpr int kTabEntries = kTabDoubles > kHandoverDoubles ? kTabDoubles : kHandoverDoubles;
  __shared__ double tab[kTabEntries];                   // also carries q (4096 floats) at the end
  __shared__ uint32_t stage[kStaged ? kChunk * kTileWords : 1];
  __shared__ double s_scale[kChunk];
  __shared__ double lds_d[kWaves];
  __shared__ double lds_d2[kWaves];
  __shared__ uint32_t lds_u[kWaves];
  __shared__ int lds_e[3 * kWaves];
  __shared__ uint8_t dep[SPARSE ? 16 * 256 : 16];
  __shared__ uint32_t lds_scan[kWaves][SPARSE ? kChunk / 2 : 1];
  const int t = threadIdx.x;
  if (SPARSE)                                             // visible after the first barrier below
    reinterpret_cast<uint4*>(dep)[t] = reinterpret_cast<const uint4*>(kDepositLut.v)[t];
  // the work-group's tile, its live coordinates [lo, hi) and its column of scales
  int64_t tile, lo, hi, k;
  if (a.seg.piece_tile) {
    const Piece pc = load_piece(a.seg, blockIdx.x, a.d);
    tile = pc.tile; lo = pc.lo; hi = pc.hi; k = pc.seg;
  } else {
    tile = blockIdx.x;
    lo = tile * kTile;
    hi = lo + kTile < a.d ? lo + kTile : a.d;
    k = a.log2b >= 0 ? (lo >> a.log2b) : 0;                            // same for the whole tile
  }
  const int64_t tile_base = tile * kTile;
  const bool full_tile = hi - lo == kTile;
  // words of this tile that exist; lanes beyond read the last one (in bounds) and are masked
  const int64_t words_here = a.W - tile * kTileWords;
  const int tw = words_here >= kTileWords ? t : (t < (int)words_here ? t : (int)words_here - 1);
  // Buckets smaller than the tile: every thread's 16 coordinates still share one bucket, but the
  // tile does not; such launches take the worker-ordered sum below with per-thread scales.
  const bool own_scales = !a.tile_uniform;               // uniform over the launch
  const float* sc = a.scales + (own_scales ? ((tile_base + 16 * (int64_t)tw) >> a.log2b) : k);
  const uint32_t tw4 = (uint32_t)tw * 4u;
  const uint32_t row_bytes = 4u * (uint32_t)(words_here >= kTileWords ? kTileWords : words_here);
  const uint32_t* ctile = a.codes + tile * kTileWords;                 // uniform base

  // ---- request the first chunk of code words ----
  uint32_t w[kChunk];
  // wave v brings rows v*kChunk/4 .. of the chunk that starts at worker m0 into the staging area
  auto stage_request = [&](int m0) {
    const int wave = __builtin_amdgcn_readfirstlane(t / kWave);   // known uniform: scalar addressing
#pragma unroll
    for (int i = 0; i < kChunk / kWaves; ++i) {
      const int r = wave * (kChunk / kWaves) + i;
      stream_row_to_lds(ctile + (int64_t)(m0 + r) * a.code_stride, row_bytes, stage + r * kTileWords);
    }
  };
  if (kStaged) {
    if (!own_scales) stage_request(0);
  } else if (!SPARSE) {
    const int left = own_scales ? 0 : a.M;
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      w[i] = ((FULL && !own_scales) || i < left)
                 ? stream_load(ctile + (int64_t)i * a.code_stride, tw4, row_bytes) : 0u;
  }

  // ---- can the sum over workers be reordered? (exponent span of the tile's scales) ----
  int emax = 0, emin = 255, bad = own_scales ? 1 : 0;
  for (int m = t; m < (own_scales ? 0 : a.M); m += kThreads) {
    const uint32_t u = __float_as_uint(sc[(int64_t)m * a.scale_stride]);
    if ((u << 1) == 0u) continue;
    int f = (int)((u >> 23) & 0xFFu);
    if (f == 255) bad = 1;
    f = f < 1 ? 1 : f;
    emax = f > emax ? f : emax;
    emin = f < emin ? f : emin;
  }
  if (!SPARSE) {
    emax = wave_reduce_i32(emax, [](int p, int q) { return p > q ? p : q; });
    emin = wave_reduce_i32(emin, [](int p, int q) { return p < q ? p : q; });
    bad = wave_reduce_i32(bad, [](int p, int q) { return p | q; });
  } else {                                                // (the sparse variants: fewer registers this way)
    for (int off = 1; off < kWave; off <<= 1) {
      const int o1 = __shfl_xor(emax, off, kWave), o2 = __shfl_xor(emin, off, kWave);
      bad |= __shfl_xor(bad, off, kWave);
      emax = o1 > emax ? o1 : emax;
      emin = o2 < emin ? o2 : emin;
    }
  }
  if ((t % kWave) == 0) {
    lds_e[t / kWave] = emax; lds_e[kWaves + t / kWave] = emin; lds_e[2 * kWaves + t / kWave] = bad;
  }
  __syncthreads();
#pragma unroll
  for (int v = 0; v < kWaves; ++v) {
    emax = lds_e[v] > emax ? lds_e[v] : emax;
    emin = lds_e[kWaves + v] < emin ? lds_e[kWaves + v] : emin;
    bad |= lds_e[2 * kWaves + v];
  }
  const bool reorder_ok = !bad && (emax - emin) <= a.span_limit;
  // may the update use the short sqrt / division? (decided here so that emin, emax die early)
  bool try_core = reorder_ok && emin >= a.fast_emin && emax <= a.fast_emax;

  double acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.0;

  // decoded codes of the four workers for index byte t (see lookup_group): bit j = non-zero,
  // bit 4+j = negative; the reserved pattern (negative without non-zero) reads as 0
  double dj[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) dj[j] = ((t >> j) & 1) ? (((t >> (4 + j)) & 1) ? -1.0 : 1.0) : 0.0;
  // The chunk that starts at worker m0 in three parts.  gather(): the code words become index
  // words, four per group, in the same registers' worth of space, so the code words are dead
  // afterwards and the next chunk's can be requested into them before the tables are built:
  // memory requests stay in flight during the table build and the look-ups at no register cost.
  uint32_t zq[kChunk];
  // Thread i < kChunk fetches worker (chunk start + i)'s scale for the tile.
  auto chunk_scale = [&](int m0) -> float {
    return (t < kChunk && m0 + t < a.M && !own_scales) ? sc[(int64_t)(m0 + t) * a.scale_stride] : 0.0f;
  };
  float sc_ahead = kStaged ? chunk_scale(0) : 0.0f;     // (staged loop only: elsewhere it measured slower)
  auto gather = [&](const uint32_t (&wc)[kChunk]) {
#pragma unroll
    for (int g = 0; g < kGroupsPerChunk; ++g)
      gather_group(wc[4 * g], wc[4 * g + 1], wc[4 * g + 2], wc[4 * g + 3], zq + 4 * g);
  };
  auto tables_and_lookups = [&](int m0) {
    const int left = a.M - m0;
    const int ng = (FULL || left >= kChunk) ? kGroupsPerChunk : (left + 3) / 4;
    if (m0 > 0) __syncthreads();                         // readers of the previous tables are done
    if (t < kChunk) s_scale[t] = (double)chunk_scale(m0);
    __syncthreads();
    for (int g = 0; g < ng; ++g) {
      const double e = fma(dj[3], s_scale[4 * g + 3],
                           fma(dj[2], s_scale[4 * g + 2],
                               fma(dj[1], s_scale[4 * g + 1], dj[0] * s_scale[4 * g])));
      tab[g * 256 + t] = e;
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < kGroupsPerChunk; ++g)
      if (FULL || g < ng) lookup_indices(zq + 4 * g, tab + g * 256, acc);
  };
  auto chunk = [&](const uint32_t (&wc)[kChunk], int m0) {
    gather(wc);
    tables_and_lookups(m0);
  };

  if (SPARSE) {
    const int wave = t / kWave;
    // indicator words of this tile that exist; half-word t&1 of word t/2 covers the thread's 16
    // coordinates; bits at or beyond d are not components
    const int64_t NW = (a.d + 31) / 32;
    const int64_t iw_here = NW - tile * (kTile / 32);
    const uint32_t ind_bytes = 4u * (uint32_t)(iw_here >= kTile / 32 ? kTile / 32 : iw_here);
    const uint32_t* itile = a.ind + tile * (kTile / 32);
    const uint32_t ind_off = (uint32_t)(t >> 1) * 4u;
    const int64_t live = a.d - (tile_base + 16 * (int64_t)t);
    const uint32_t live_mask = live >= 16 ? 0xFFFFu : (live > 0 ? (1u << live) - 1u : 0u);
    uint32_t syn = 0;                                    // the synchronous indicator of the thread's 16
    for (int m0 = 0; m0 < a.M; m0 += kChunk) {
      const int left = a.M - m0;
      uint32_t mk[kChunk];
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        const uint32_t iv =
            i < left ? stream_load(itile + (int64_t)(m0 + i) * a.ind_stride, ind_off, ind_bytes) : 0u;
        mk[i] = (iv >> (16 * (t & 1))) & live_mask;
        syn |= mk[i];
      }
      // marked components before this thread's, per worker (two 16-bit counts per scan; a tile
      // holds at most 4096)
      uint32_t ex[kChunk / 2];
      if (m0 > 0) __syncthreads();                       // readers of the previous totals are done
#pragma unroll
      for (int p = 0; p < kChunk / 2; ++p) {
        const uint32_t own = (uint32_t)__popc(mk[2 * p]) | ((uint32_t)__popc(mk[2 * p + 1]) << 16);
        const uint32_t incl = wave_inclusive_scan_u32(own);
        if ((t % kWave) == kWave - 1) lds_scan[wave][p] = incl;
        ex[p] = incl - own;
      }
      __syncthreads();
#pragma unroll
      for (int p = 0; p < kChunk / 2; ++p)
#pragma unroll
        for (int v = 0; v < kWaves - 1; ++v) ex[p] += v < wave ? lds_scan[v][p] : 0u;
      // the thread's n <= 16 codes start at code `before` of the worker's stream for this bucket:
      // word before/16 and, if they cross a word boundary, the next one.  Offsets beyond the
      // words that exist for this tile read as 0 (never needed: the stream holds every marked
      // component of the tile)
      uint32_t s_lo[kChunk], s_hi[kChunk];
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        const uint32_t before = (ex[i / 2] >> (16 * (i & 1))) & 0xFFFFu;
        const uint32_t* area = ctile + (int64_t)(m0 + i) * a.code_stride;
        s_lo[i] = i < left ? cached_load(area, (before >> 4) * 4u, row_bytes) : 0u;
        s_hi[i] = i < left ? cached_load(area, (before >> 4) * 4u + 4u, row_bytes) : 0u;
      }
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        const uint32_t before = (ex[i / 2] >> (16 * (i & 1))) & 0xFFFFu;
        uint32_t win = __builtin_amdgcn_alignbit(s_hi[i], s_lo[i], 2u * (before & 15u));
        uint32_t out = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint32_t nib = (mk[i] >> (4 * q)) & 15u;
          out |= (uint32_t)dep[nib * 256 + (win & 0xFFu)] << (8 * q);
          win >>= 2 * __popc(nib);
        }
        w[i] = out;
      }
      if (reorder_ok) {
        chunk(w, m0);
      } else {
        // ordered sum, as it is written: worker m0, m0+1, ...
#pragma unroll
        for (int u = 0; u < kChunk; ++u)
          if (u < left) {
            const uint32_t wv = sanitize(w[u]);
            const double sv = (double)sc[(int64_t)(m0 + u) * a.scale_stride];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const int c = ((int)(wv << (30 - 2 * j))) >> 30;
              acc[j] = fma((double)c, sv, acc[j]);
            }
          }
      }
    }
    if (a.ind_syn) {                                     // uniform; word t/2 = the halves of threads t, t^1
      const uint32_t other = (uint32_t)dpp_i32<kDppQuadXor1>((int)syn);
      const int64_t iw = tile * (kTile / 32) + (t >> 1);
      if ((t & 1) == 0 && iw < NW) a.ind_syn[iw] = syn | (other << 16);
    }
  } else if (kStaged && reorder_ok) {
    // The next chunk's code words travel from memory into LDS while this chunk's tables are built
    // and read, at no cost in vector registers: six waves per SIMD with requests in flight nearly
    // all the time (measured at d = 2^30, M = 64: 3.48 ms against 3.63 ms with register loads;
    // the kernel that writes the average out, already at the rate of a plain copy, gained nothing).
    for (int m0 = 0; m0 < a.M; m0 += kChunk) {
      wait_vector_memory();                              // this wave's rows of the chunk have landed
      __syncthreads();                                   // ... everyone's; the previous tables are free
#pragma unroll
      for (int i = 0; i < kChunk; ++i) w[i] = stage[i * kTileWords + t];
      if (t < kChunk) s_scale[t] = (double)sc_ahead;
      gather(w);
      __syncthreads();                                   // the staging area has been read by all
      sc_ahead = chunk_scale(m0 + kChunk);
      if (m0 + kChunk < a.M) stage_request(m0 + kChunk);
#pragma unroll
      for (int g = 0; g < kGroupsPerChunk; ++g) {
        const double e = fma(dj[3], s_scale[4 * g + 3],
                             fma(dj[2], s_scale[4 * g + 2],
                                 fma(dj[1], s_scale[4 * g + 1], dj[0] * s_scale[4 * g])));
        tab[g * 256 + t] = e;
      }
      barrier_lds_only();                                // tables complete; the rows stay in flight
#pragma unroll
      for (int g = 0; g < kGroupsPerChunk; ++g) lookup_indices(zq + 4 * g, tab + g * 256, acc);
    }
  } else if (reorder_ok) {
    // The kernels that go on to update the state request the next chunk right after the gather.
    // The aggregate-only kernels do not: they are small enough for five waves per SIMD, which
    // the longer live ranges would cost them (measured: 3.65 ms against 3.96 ms at d = 2^30, M = 64).
    constexpr bool kEarlyLoads = MODE != kAggregate;
    for (int m0 = 0; m0 < a.M; m0 += kChunk) {
      if (!kEarlyLoads && m0 > 0) {
        const int left = a.M - m0;
        const uint32_t* cc = ctile + (int64_t)m0 * a.code_stride;
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
          w[i] = (FULL || i < left) ? stream_load(cc + (int64_t)i * a.code_stride, tw4, row_bytes) : 0u;
      }
      gather(w);
      const int left = a.M - (m0 + kChunk);                // workers after this chunk
      if (kEarlyLoads && left > 0) {
        const uint32_t* cc = ctile + (int64_t)(m0 + kChunk) * a.code_stride;
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
          w[i] = (FULL || i < left) ? stream_load(cc + (int64_t)i * a.code_stride, tw4, row_bytes) : 0u;
      }
      tables_and_lookups(m0);
    }
  } else {
    // ordered loop, as the sum is written: worker 0, 1, 2, ...; eight code words are requested
    // at a time so that their latencies overlap
    if (kStaged) wait_vector_memory();                   // rows requested into LDS above: unused here
    for (int m0 = 0; m0 < a.M; m0 += 8) {
      uint32_t wv[8];
      double sv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool in = m0 + u < a.M;
        const int m = in ? m0 + u : a.M - 1;
        wv[u] = sanitize(stream_load(ctile + (int64_t)m * a.code_stride, tw4, row_bytes));
        sv[u] = (double)sc[(int64_t)m * a.scale_stride];
        if (!in) { wv[u] = 0u; sv[u] = 0.0; }             // adds +0
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int c = ((int)(wv[u] << (30 - 2 * j))) >> 30;
          acc[j] = fma((double)c, sv[u], acc[j]);
        }
    }
  }

  // The state is requested only now: held in registers during the look-ups it would cost a wave
  // per SIMD, and the other waves of the SIMD cover its latency.
  State4 sG, sx, sz;
  if (MODE != kAggregate) {
    load_state(a.G, tile_base, lo, hi, full_tile, sG);
    if (MODE == kQcmd) load_state(a.x, tile_base, lo, hi, full_tile, sx);
    // with the second quantization still to come, z (needed last) is requested after it
    if ((MODE == kQrda || TRACK_Z) && !(REQUANT && MODE == kQcmd))
      load_state(a.z, tile_base, lo, hi, full_tile, sz);
  }

  float q[16];
  if (a.M_pow2) {
#pragma unroll
    for (int j = 0; j < 16; ++j) q[j] = (float)(acc[j] * a.inv_M);
  } else {
    const double Md = (double)a.M;
#pragma unroll
    for (int j = 0; j < 16; ++j) q[j] = (float)(acc[j] / Md);
  }
  if (!full_tile) {                                       // dead lanes lie at or beyond hi
    const int64_t i0 = tile_base + 16 * (int64_t)t;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (i0 + j < lo || i0 + j >= hi) q[j] = 0.0f;
  }

  if (MODE == kAggregate && a.abs_partials) {             // uniform
    double s1 = 0.0;
#pragma unroll
    for (int j = 0; j < 16; ++j) s1 += (double)fabsf(q[j]);
    s1 = block_sum_f64(s1, lds_d);
    if (t == 0) a.abs_partials[tile] = s1;
  }
  if (MODE == kAggregate && RQ == kRqNone && a.kept_sum) {   // uniform
    const float Delta = a.rq_thr[tile / a.rq_tiles];
    double s2 = 0.0;
    uint32_t cnt = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float av = fabsf(q[j]);                       // dead lanes hold zeros
      if (av > Delta) { s2 += (double)av; ++cnt; }
    }
    s2 = wave_sum_f64(s2);
    cnt = wave_sum_u32(cnt);
    if ((t % kWave) == 0) { lds_d2[t / kWave] = s2; lds_u[t / kWave] = cnt; }
    __syncthreads();
    if (t == 0) {
      a.kept_sum[tile] = (lds_d2[0] + lds_d2[1]) + (lds_d2[2] + lds_d2[3]);
      a.kept_cnt[tile] = (lds_u[0] + lds_u[1]) + (lds_u[2] + lds_u[3]);
    }
    return;
  }
  if (MODE == kAggregate && RQ == kRqNone && !a.gbar) return;   // uniform: only the sums were wanted

  if (RQ == kRqGiven) {
    static_assert(RQ != kRqGiven || MODE != kAggregate, "the server's call writes the average out");
    const int64_t k2 = tile / a.rq_tiles;
    const float Delta = a.rq_thr[k2], s = a.rq_scale[k2];
    // q = +-s comes from the whole bucket, not from this tile: the short forms of the update also
    // need s itself inside the window that was checked for the tile's own scales
    const int es = (int)((__float_as_uint(s) >> 23) & 0xFFu);
    if (!(s == 0.0f || (es >= a.fast_emin && es <= a.fast_emax))) try_core = false;
#pragma unroll
    for (int j = 0; j < 16; ++j) q[j] = q[j] > Delta ? s : (q[j] < -Delta ? -s : 0.0f);
  }

  if (REQUANT) {
    // second quantization of the average, per bucket: the whole tile, or (buckets smaller than
    // the tile) a segment of bucket/16 consecutive threads
    const int seg = own_scales ? (1 << a.log2b) / 16 : kThreads;
    int64_t n = hi - lo;
    if (own_scales) {
      const int64_t b = (int64_t)1 << a.log2b;
      const int64_t blo = ((tile_base + 16 * (int64_t)t) >> a.log2b) << a.log2b;
      n = (a.d - blo) < b ? (a.d - blo) : b;              // true length of the thread's bucket
    }
    double s1 = 0.0;
#pragma unroll
    for (int j = 0; j < 16; ++j) s1 += (double)fabsf(q[j]);   // dead lanes hold zeros
    // a bucket that is the whole tile: sums over the work-group without lane shuffles
    s1 = own_scales ? segment_sum(s1, seg, lds_d) : block_sum_f64(s1, lds_d);
    const float Delta = n > 0 ? threshold_from_sum(s1, a.thr_coef, n) : 0.0f;
    double s2 = 0.0;
    uint32_t cnt = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float av = fabsf(q[j]);
      if (av > Delta) { s2 += (double)av; ++cnt; }
    }
    if (own_scales) {
      s2 = segment_sum(s2, seg, lds_d);
      cnt = segment_sum_u32(cnt, seg, lds_u);
    } else {
      s2 = wave_sum_f64(s2);
      cnt = wave_sum_u32(cnt);
      if ((t % kWave) == 0) { lds_d2[t / kWave] = s2; lds_u[t / kWave] = cnt; }
      __syncthreads();                                    // (lds_d of the first sum is not touched)
      s2 = (lds_d2[0] + lds_d2[1]) + (lds_d2[2] + lds_d2[3]);
      cnt = (lds_u[0] + lds_u[1]) + (lds_u[2] + lds_u[3]);
    }
    const float s = scale_from_sum(s2, cnt);
    if (MODE == kAggregate) {
      // the server's output: q_t = Q(SynQ_t) as a message (the thread's 16 coordinates are
      // code word t of the tile), one scale per bucket written by the bucket's first thread
      uint32_t word = 0;
#pragma unroll
      for (int j = 0; j < 16; ++j) word |= ternary_field(q[j], Delta) << (2 * j);
      if ((int64_t)t < words_here) a.q_codes[tile * kTileWords + t] = word;
      const bool leader = own_scales ? (t & (seg - 1)) == 0 : t == 0;
      if (leader && n > 0) {
        const int64_t kq = own_scales ? ((tile_base + 16 * (int64_t)t) >> a.log2b) : k;
        a.q_scales[kq] = s;
        if (a.q_thresholds) a.q_thresholds[kq] = Delta;
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) q[j] = q[j] > Delta ? s : (q[j] < -Delta ? -s : 0.0f);
  }

  if (REQUANT && MODE == kQcmd && TRACK_Z) load_state(a.z, tile_base, lo, hi, full_tile, sz);

  // ---- hand q over through LDS to the float4 mapping of the state loads ----
  float* qt = reinterpret_cast<float*>(tab);
  __syncthreads();
#pragma unroll
  for (int v = 0; v < 4; ++v)
    *reinterpret_cast<float4*>(qt + 16 * t + 4 * v) =
        make_float4(q[4 * v], q[4 * v + 1], q[4 * v + 2], q[4 * v + 3]);
  __syncthreads();
  if (full_tile && MODE != kAggregate) {
    // whole tile: each float4 group is updated and stored as soon as its q is read back.
    // Tiles whose scales lie in the safe exponent range try the short sqrt / division first;
    // a group in which any lane of the wave leaves the safe range is redone in full.
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 qv = *reinterpret_cast<const float4*>(qt + 4 * (j * kThreads + t));
      const float qq[4] = {qv.x, qv.y, qv.z, qv.w};
      float G[4] = {sG.v[j].x, sG.v[j].y, sG.v[j].z, sG.v[j].w};
      float x0[4] = {0.f, 0.f, 0.f, 0.f}, z[4] = {0.f, 0.f, 0.f, 0.f}, x[4];
      if (MODE == kQcmd) { x0[0] = sx.v[j].x; x0[1] = sx.v[j].y; x0[2] = sx.v[j].z; x0[3] = sx.v[j].w; }
      if (MODE == kQrda || TRACK_Z) { z[0] = sz.v[j].x; z[1] = sz.v[j].y; z[2] = sz.v[j].z; z[3] = sz.v[j].w; }
#pragma unroll
      for (int e = 0; e < 4; ++e) accumulate<MODE, TRACK_Z>(qq[e], G[e], z[e]);
      bool done = false;
      if (try_core) {
        bool bad = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = solve_x_core<MODE>(a, qq[e], x0[e], G[e], z[e], bad);
        done = !__any(bad);                               // uniform over the wave
      }
      if (!done) {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = solve_x<MODE>(a, qq[e], x0[e], G[e], z[e]);
      }
      const int64_t i = tile_base + (int64_t)(j * kThreads + t) * 4;
      stream_store4(a.G + i, make_float4(G[0], G[1], G[2], G[3]));
      stream_store4(a.x + i, make_float4(x[0], x[1], x[2], x[3]));
      if (MODE == kQrda || TRACK_Z) stream_store4(a.z + i, make_float4(z[0], z[1], z[2], z[3]));
    }
    return;
  }
  State4 sq;
#pragma unroll
  for (int j = 0; j < 4; ++j) sq.v[j] = *reinterpret_cast<const float4*>(qt + 4 * (j * kThreads + t));

  if (MODE == kAggregate) {
    store_state(a.gbar, tile_base, lo, hi, full_tile, sq);
    return;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float qq[4] = {sq.v[j].x, sq.v[j].y, sq.v[j].z, sq.v[j].w};
    float G[4] = {sG.v[j].x, sG.v[j].y, sG.v[j].z, sG.v[j].w};
    float x[4] = {0.f, 0.f, 0.f, 0.f}, z[4] = {0.f, 0.f, 0.f, 0.f};
    if (MODE == kQcmd) { x[0] = sx.v[j].x; x[1] = sx.v[j].y; x[2] = sx.v[j].z; x[3] = sx.v[j].w; }
    if (MODE == kQrda || TRACK_Z) { z[0] = sz.v[j].x; z[1] = sz.v[j].y; z[2] = sz.v[j].z; z[3] = sz.v[j].w; }
#pragma unroll
    for (int e = 0; e < 4; ++e) update_coordinate<MODE, TRACK_Z>(a, qq[e], x[e], G[e], z[e]);
    sG.v[j] = make_float4(G[0], G[1], G[2], G[3]);
    sx.v[j] = make_float4(x[0], x[1], x[2], x[3]);
    sz.v[j] = make_float4(z[0], z[1], z[2], z[3]);
  }
  store_state(a.G, tile_base, lo, hi, full_tile, sG);
  store_state(a.x, tile_base, lo, hi, full_tile, sx);
  if (MODE == kQrda || TRACK_Z) store_state(a.z, tile_base, lo, hi, full_tile, sz);
}

// ---- the two sums behind Q(SynQ) with one scale, from messages with one scale each -------------
//
// One scale per message (the paper's message) and at most 8 workers: the tables of partial sums
// are the same for every tile, so a work-group builds them once (no exponent-span test per tile, no
// barrier per chunk) and walks several tiles, keeping its sums in registers; per tile that leaves
// the loads, the gather, two look-ups per coordinate and the conversion.  PASS 0: sum of |gbar|;
// PASS 1: sum and count of the |gbar| above the threshold (one partial per work-group each);
// PASS 2: the codes of Q(SynQ) for that threshold, for the server's call.
struct SumArgs {
  const uint32_t* codes;
  const float* scales;
  int64_t code_stride, scale_stride;
  int64_t d, W, ntiles;
  int M, tiles_per_group, M_pow2, span_limit;
  double inv_M;
  const float* thr;                     // PASS 1, 2: the threshold
  double* part_sum;
  uint32_t* part_cnt;
  uint32_t* q_codes;                    // PASS 2
};

template <int PASS>
__global__ __launch_bounds__(kThreads) void requant_sums_kernel(SumArgs a) {
  __shared__ double tab[2 * 256];
  __shared__ double lds_d[kWaves];
  __shared__ uint32_t lds_u[kWaves];
  const int t = threadIdx.x;
  // the workers' scales, the same for every thread; may the sum over workers be reordered?
  float sc[8];
  int emax = 0, emin = 255, bad = 0;
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    sc[m] = m < a.M ? a.scales[(int64_t)m * a.scale_stride] : 0.0f;
    const uint32_t u = __float_as_uint(sc[m]);
    if ((u << 1) == 0u) continue;
    int f = (int)((u >> 23) & 0xFFu);
    if (f == 255) bad = 1;
    f = f < 1 ? 1 : f;
    emax = f > emax ? f : emax;
    emin = f < emin ? f : emin;
  }
  const bool reorder_ok = !bad && (emax - emin) <= a.span_limit;
  if (reorder_ok) {
    double dj[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) dj[j] = ((t >> j) & 1) ? (((t >> (4 + j)) & 1) ? -1.0 : 1.0) : 0.0;
#pragma unroll
    for (int g = 0; g < 2; ++g)
      tab[g * 256 + t] = fma(dj[3], (double)sc[4 * g + 3],
                             fma(dj[2], (double)sc[4 * g + 2],
                                 fma(dj[1], (double)sc[4 * g + 1], dj[0] * (double)sc[4 * g])));
    __syncthreads();
  }
  const float Delta = PASS >= 1 ? a.thr[0] : 0.0f;
  double s = 0.0;
  uint32_t cnt = 0;
  const int64_t tile0 = (int64_t)blockIdx.x * a.tiles_per_group;
  for (int u = 0; u < a.tiles_per_group && tile0 + u < a.ntiles; ++u) {
    const int64_t tile = tile0 + u;
    const int64_t words_here = a.W - tile * kTileWords;
    const uint32_t row_bytes = 4u * (uint32_t)(words_here >= kTileWords ? kTileWords : words_here);
    const uint32_t* ctile = a.codes + tile * kTileWords;
    uint32_t w[8];
#pragma unroll
    for (int m = 0; m < 8; ++m)                           // words beyond the row read as 0
      w[m] = m < a.M ? stream_load(ctile + (int64_t)m * a.code_stride, 4u * (uint32_t)t, row_bytes) : 0u;
    double acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0;
    if (reorder_ok) {
      uint32_t zq[8];
      gather_group(w[0], w[1], w[2], w[3], zq);
      gather_group(w[4], w[5], w[6], w[7], zq + 4);
      lookup_indices(zq, tab, acc);
      if (a.M > 4) lookup_indices(zq + 4, tab + 256, acc);
    } else {                                              // as the sum is written: worker 0, 1, ...
      for (int m = 0; m < a.M; ++m) {
        uint32_t wv = 0u;
        double sv = 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k)                       // (selects: w[] and sc[] stay in registers)
          if (k == m) { wv = sanitize(w[k]); sv = (double)sc[k]; }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int c = ((int)(wv << (30 - 2 * j))) >> 30;
          acc[j] = fma((double)c, sv, acc[j]);
        }
      }
    }
    float q[16];
    if (a.M_pow2) {
#pragma unroll
      for (int j = 0; j < 16; ++j) q[j] = (float)(acc[j] * a.inv_M);
    } else {
      const double Md = (double)a.M;
#pragma unroll
      for (int j = 0; j < 16; ++j) q[j] = (float)(acc[j] / Md);
    }
    const int64_t live = a.d - (tile * kTile + 16 * (int64_t)t);   // fields at or beyond d are no components
    if (live < 16) {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j >= live) q[j] = 0.0f;
    }
    if (PASS == 2) {
      uint32_t word = 0;
#pragma unroll
      for (int j = 0; j < 16; ++j) word |= ternary_field(q[j], Delta) << (2 * j);
      if ((int64_t)t < words_here) a.q_codes[tile * kTileWords + t] = word;
      continue;
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float av = fabsf(q[j]);
      if (PASS == 0) s += (double)av;
      else if (av > Delta) { s += (double)av; ++cnt; }
    }
  }
  if (PASS == 2) return;
  s = block_sum_f64(s, lds_d);
  if (PASS == 1) {
    cnt = wave_sum_u32(cnt);
    if ((t % kWave) == 0) lds_u[t / kWave] = cnt;
    __syncthreads();
    cnt = (lds_u[0] + lds_u[1]) + (lds_u[2] + lds_u[3]);
  }
  if (t == 0) {
    a.part_sum[blockIdx.x] = s;
    if (PASS == 1) a.part_cnt[blockIdx.x] = cnt;
  }
}

// ---- host side -------------------------------------------------------------------------------

static inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t select_workspace_bytes(const qa_layout* L);
bool sparse_messages_fused(const qa_layout* L);
int check_sparse_layout(const qa_layout* L);
int decode_selected_launch(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                           const uint32_t* sel_codes, uint32_t* codes_out, int64_t out_stride,
                           void* ws, size_t ws_bytes, hipStream_t stream);
void indicator_or_launch(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                         uint32_t* ind_syn_out, hipStream_t stream);
size_t quantize_workspace_bytes(const qa_layout* L);
int quantize_launch(const qa_layout* L, const float* g, int64_t g_stride, uint32_t* codes,
                    float* scales, float* thresholds, uint32_t flags, void* ws, size_t ws_bytes,
                    hipStream_t stream);
void quantize_workspace_parts(const qa_layout* L, void* ws, double** part_sum, uint32_t** part_cnt,
                              float** thr);
int quantize_finalize_launch(const qa_layout* L, int which, int64_t n_partials, float* scales,
                             float* thresholds, void* ws, size_t ws_bytes, hipStream_t stream);

// Layout of the one-message vector that carries Q(SynQ) when it is formed in separate passes.
static qa_layout requant_layout(const qa_layout* L, int requant) {
  qa_layout R = *L;
  R.M = 1;
  R.bucket = requant == QA_REQUANT_GLOBAL ? 0 : L->bucket;
  R.code_stride = words_of(L->d);
  R.scale_stride = buckets_of(L->d, R.bucket);
  return R;
}

// Can Q(SynQ) be formed inside the step kernel?  Buckets that fit a tile; also one scale for a
// vector that is a single tile (table-driven kernel only).
static bool requant_in_tile(const qa_layout* L, int requant) {
  if (requant == QA_REQUANT_BUCKET) return L->bucket != 0 && L->bucket <= kTile;
  if (requant == QA_REQUANT_GLOBAL)
    return tiles_of(L->d) == 1 && (L->bucket == 0 || L->bucket >= kTile);
  return false;
}

static size_t requant_need(const qa_layout* L, const qa_layout* R) {
  return align256((size_t)L->d * sizeof(float)) + align256((size_t)R->code_stride * 4) +
         2 * align256((size_t)R->scale_stride * 4) + quantize_workspace_bytes(R);
}

// Worst case over the second-quantization modes that need separate passes.
size_t step_workspace_bytes(const qa_layout* L) {
  qa_layout R = requant_layout(L, QA_REQUANT_GLOBAL);
  size_t need = requant_need(L, &R);
  if (L->bucket > kTile) {
    qa_layout B = requant_layout(L, QA_REQUANT_BUCKET);
    const size_t nb = requant_need(L, &B);
    if (nb > need) need = nb;
  }
  return need;
}

// Sparse messages whose buckets are not one tile each are first decoded into dense code words
// (in the workspace) and then take the dense path: the definition of the steps on sparse messages.
// Workspace: [dense codes, M rows of a 256-byte multiple][decoder's workspace][step's workspace].
static int64_t decoded_stride(const qa_layout* L) { return (words_of(L->d) + 63) & ~int64_t(63); }
size_t step_selected_workspace_bytes(const qa_layout* L) {
  if (sparse_messages_fused(L)) return step_workspace_bytes(L);
  return align256((size_t)L->M * (size_t)decoded_stride(L) * 4) + align256(select_workspace_bytes(L)) +
         step_workspace_bytes(L);
}
// Decodes into the workspace; on return *dense / *D describe the dense messages and *ws / *ws_bytes
// what is left of the workspace.
static int decode_into_workspace(const qa_layout* L, const uint32_t* ind, int64_t ind_stride,
                                 const uint32_t* sel_codes, qa_layout* D, const uint32_t** dense,
                                 void** ws, size_t* ws_bytes, hipStream_t stream) {
  const size_t codes_bytes = align256((size_t)L->M * (size_t)decoded_stride(L) * 4);
  const size_t sel_bytes = align256(select_workspace_bytes(L));
  if (!*ws || *ws_bytes < codes_bytes + sel_bytes) return QA_ERR_WORKSPACE;
  if (!aligned(*ws, 256)) return QA_ERR_ALIGNMENT;
  char* p = static_cast<char*>(*ws);
  *D = *L;
  D->code_stride = decoded_stride(L);
  uint32_t* out = reinterpret_cast<uint32_t*>(p);
  int rc = decode_selected_launch(L, ind, ind_stride, sel_codes, out, D->code_stride,
                                  sel_bytes ? p + codes_bytes : nullptr, sel_bytes, stream);
  if (rc != QA_OK) return rc;
  *dense = out;
  *ws = p + codes_bytes + sel_bytes;
  *ws_bytes -= codes_bytes + sel_bytes;
  if (*ws_bytes == 0) *ws = nullptr;
  return QA_OK;
}

static StepArgs make_args(const qa_layout* L, const uint32_t* codes, const float* scales) {
  StepArgs a{};
  a.codes = codes; a.scales = scales;
  a.code_stride = L->code_stride; a.scale_stride = L->scale_stride;
  a.d = L->d; a.W = words_of(L->d); a.M = L->M;
  a.log2b = L->bucket ? ilog2(L->bucket) : -1;
  a.M_pow2 = is_pow2(L->M) ? 1 : 0;
  a.inv_M = 1.0 / (double)L->M;
  a.thr_coef = L->thr_coef;
  // partial sums are multiples of 2^(e_min-23) and below M*2^(e_max+1): exact in binary64 iff
  // log2(M) + span + 24 <= 53
  a.span_limit = 29 - ilog2(L->M);
  a.tile_uniform = (L->bucket == 0 || L->bucket >= kTile) ? 1 : 0;
  return a;
}

// Which tiles may use the short sqrt / division of the update (see sqrt_core / div_core): the
// numerators eta*q and lambda*eta (QCMD) or eta*r (QRDA) and the denominator H = delta + sqrt(G)
// must lie where the full division does no rescaling.  With |q| between 2^(emin-150)/M and
// 2^(emax-126) for a tile whose non-zero scales have biased exponents emin..emax, that becomes a
// window on (emin, emax), and for QRDA a window on the positive r, checked per lane.
static void set_fast_limits(StepArgs& a, int mode, float eta, float lam_eta, float delta) {
  a.fast_emin = 1 << 20; a.fast_emax = -1;               // no tile qualifies
  if (!(delta >= 0x1p-64f && delta <= 0x1p63f)) return;
  if (!(eta >= 0x1p-40f && eta <= 0x1p40f)) return;
  const int le = ilogbf(eta), ld = ilogbf(delta);
  const int hi = 93 + ld < 59 ? 93 + ld : 59;            // numerators stay below 2^hi
  if (mode == kQcmd && lam_eta != 0.0f && !(lam_eta >= 0x1p-61f && lam_eta < ldexpf(1.0f, hi))) return;
  a.fast_emin = -61 - le + 150 + ilog2(a.M);
  a.fast_emax = hi - le - 2 + 126;
  const float r_lo = ldexpf(1.0f, -61 - le), r_hi = ldexpf(1.0f, hi - le - 1);
  uint32_t lo_bits, hi_bits;
  memcpy(&lo_bits, &r_lo, 4); memcpy(&hi_bits, &r_hi, 4);
  a.fast_r_lo = lo_bits; a.fast_r_span = hi_bits - lo_bits;
}

template <int MODE, bool TRACK_Z, int RQ, int NGT, bool SPARSE = false>
static void launch_lut(const StepArgs& a, dim3 grid, dim3 block, hipStream_t stream) {
  hipLaunchKernelGGL((step_lut_kernel<MODE, TRACK_Z, RQ, NGT, SPARSE>), grid, block, 0, stream, a);
}

// ngt: the NGT of the kernel variant
template <int MODE, bool TRACK_Z, int RQ>
static void launch_one(const StepArgs& a, int ngt, hipStream_t stream) {
  const dim3 grid((unsigned)(a.seg.piece_tile ? a.seg.n_pieces : tiles_of(a.d))), block(kThreads);
  if constexpr (RQ != kRqGiven) {                        // (never asked for with sparse messages)
    if (a.ind) {                                         // sparse-encoded messages
      launch_lut<MODE, TRACK_Z, RQ, 0, true>(a, grid, block, stream);
      return;
    }
  }
  switch (ngt) {
    case 4: launch_lut<MODE, TRACK_Z, RQ, 4>(a, grid, block, stream); break;
    case 2: launch_lut<MODE, TRACK_Z, RQ, 2>(a, grid, block, stream); break;
    case 1: launch_lut<MODE, TRACK_Z, RQ, 1>(a, grid, block, stream); break;
    default: launch_lut<MODE, TRACK_Z, RQ, 0>(a, grid, block, stream); break;
  }
}

template <int MODE, int RQ>
static void launch_mode_rq(const StepArgs& a, bool track_z, hipStream_t stream) {
  // buckets smaller than the tile take the ordered sum: the variant with the fewest registers
  const int which = !a.tile_uniform ? 1 : a.M % 16 == 0 ? 4 : a.M % 8 == 0 ? 2 : a.M <= 4 ? 1 : 0;
  if constexpr (MODE == kQcmd) {
    if (track_z) { launch_one<MODE, true, RQ>(a, which, stream); return; }
  }
  launch_one<MODE, false, RQ>(a, which, stream);
}
template <int MODE>
static void launch_mode(const StepArgs& a, bool track_z, bool requant, hipStream_t stream) {
  if (requant) launch_mode_rq<MODE, kRqInTile>(a, track_z, stream);
  else launch_mode_rq<MODE, kRqNone>(a, track_z, stream);
}

// A second quantization in separate passes needs the average three times (sums of |gbar|, sums of
// the kept |gbar|, the update).  With few workers the steps form it from the messages each time
// (M/4 bytes per coordinate and pass) instead of writing it out once and reading it back twice
// (4 bytes each).  The sum passes are bound by instructions, not bytes, so the gain ends early:
// measured at d = 1e8, one scale per vector, QCMD step 0.440 -> 0.400 ms at M = 2,
// 0.446 -> 0.409 at M = 4, 0.464 -> 0.450 at M = 8, but 0.515 -> 0.600 at M = 12; the server's
// call, which has no state to read, is faster with the average written out at every M (unless
// every message has one scale: see requant_sums_kernel).
constexpr int kRecomputeMaxM = 8;

// The first two of those passes and the two finalize kernels between and after them: leaves the
// thresholds and scales of Q(SynQ) in thr[] and scales[] (one per bucket of R).
// Does the kernel above serve these messages and this second quantization?
static bool one_scale_everywhere(const StepArgs& messages, const qa_layout* R) {
  return messages.log2b < 0 && R->bucket == 0 && messages.M <= 8;
}
static SumArgs sum_args(const StepArgs& messages) {
  SumArgs sa{};
  sa.codes = messages.codes; sa.scales = messages.scales;
  sa.code_stride = messages.code_stride; sa.scale_stride = messages.scale_stride;
  sa.d = messages.d; sa.W = messages.W; sa.ntiles = tiles_of(messages.d);
  sa.M = messages.M; sa.M_pow2 = messages.M_pow2; sa.inv_M = messages.inv_M;
  sa.span_limit = messages.span_limit;
  // several tiles per work-group only while that leaves a few thousand work-groups
  sa.tiles_per_group = sa.ntiles >= 16384 ? 8 : sa.ntiles >= 8192 ? 4 : sa.ntiles >= 4096 ? 2 : 1;
  return sa;
}

static int requant_sums_from_messages(const StepArgs& messages, const qa_layout* R, float* scales,
                                      float* thresholds, void* qws, size_t qws_bytes,
                                      const float** thr_out, hipStream_t stream) {
  if (!qws || qws_bytes == 0 || qws_bytes < quantize_workspace_bytes(R)) return QA_ERR_WORKSPACE;
  double* part_sum; uint32_t* part_cnt; float* thr;
  quantize_workspace_parts(R, qws, &part_sum, &part_cnt, &thr);
  *thr_out = thr;
  if (one_scale_everywhere(messages, R)) {
    // one scale per message and one for Q(SynQ): the lean kernel, one partial per work-group
    SumArgs sa = sum_args(messages);
    sa.thr = thr; sa.part_sum = part_sum; sa.part_cnt = part_cnt;
    const int64_t groups = (sa.ntiles + sa.tiles_per_group - 1) / sa.tiles_per_group;
    const dim3 grid((unsigned)groups), block(kThreads);
    hipLaunchKernelGGL(requant_sums_kernel<0>, grid, block, 0, stream, sa);
    int rc = quantize_finalize_launch(R, 0, groups, scales, thresholds, qws, qws_bytes, stream);
    if (rc != QA_OK) return rc;
    hipLaunchKernelGGL(requant_sums_kernel<1>, grid, block, 0, stream, sa);
    return quantize_finalize_launch(R, 1, groups, scales, thresholds, qws, qws_bytes, stream);
  }
  StepArgs ag = messages;
  ag.abs_partials = part_sum;
  launch_mode<kAggregate>(ag, false, false, stream);
  int rc = quantize_finalize_launch(R, 0, 0, scales, thresholds, qws, qws_bytes, stream);
  if (rc != QA_OK) return rc;
  ag.abs_partials = nullptr;
  ag.kept_sum = part_sum; ag.kept_cnt = part_cnt; ag.rq_thr = thr;
  ag.rq_tiles = R->bucket ? R->bucket / kTile : tiles_of(R->d);
  launch_mode<kAggregate>(ag, false, false, stream);
  return quantize_finalize_launch(R, 1, 0, scales, thresholds, qws, qws_bytes, stream);
}

// sparse: `codes` are compact per-bucket streams to be expanded through the indicators `ind`
static int step_common(int mode, const qa_layout* L, const uint32_t* codes, const float* scales,
                       float* x, float* G, float* z, bool track_z, int64_t t, float eta,
                       float lambda, float delta, int requant, void* ws, size_t ws_bytes,
                       hipStream_t stream, bool sparse = false, const uint32_t* ind = nullptr,
                       int64_t ind_stride = 0) {
  int rc = check_layout(L);
  if (rc != QA_OK) return rc;
  if (!codes || !scales || !x || !G) return QA_ERR_INVALID_ARG;
  if (sparse) {
    if (!ind) return QA_ERR_INVALID_ARG;
    if (ind_stride != 0 && ind_stride < (L->d + 31) / 32) return QA_ERR_INVALID_ARG;
    if (!aligned(ind, 4)) return QA_ERR_ALIGNMENT;
    rc = check_sparse_layout(L);
    if (rc != QA_OK) return rc;
  }
  if (mode == kQrda && !z) return QA_ERR_INVALID_ARG;
  if (!(eta > 0.0f) || !(lambda >= 0.0f) || !(delta > 0.0f)) return QA_ERR_INVALID_ARG;
  if (mode == kQrda && t < 1) return QA_ERR_INVALID_ARG;
  if (requant != QA_REQUANT_NONE && requant != QA_REQUANT_BUCKET && requant != QA_REQUANT_GLOBAL)
    return QA_ERR_INVALID_ARG;
  if (requant == QA_REQUANT_BUCKET && L->bucket == 0) return QA_ERR_INVALID_ARG;
  if (!aligned(x, 16) || !aligned(G, 16) || !aligned(z, 16) || !aligned(codes, 4) ||
      !aligned(scales, 4))
    return QA_ERR_ALIGNMENT;
  if (tiles_of(L->d) > 0x7fffffffLL) return QA_ERR_INVALID_ARG;

  qa_layout D;
  if (sparse && !sparse_messages_fused(L)) {
    // decode first, then the dense step on what the decoder wrote
    rc = decode_into_workspace(L, ind, ind_stride, codes, &D, &codes, &ws, &ws_bytes, stream);
    if (rc != QA_OK) return rc;
    L = &D;
    sparse = false;
  }

  qa_layout R;
  const qa_layout* use = L;
  const uint32_t* use_codes = codes;
  const float* use_scales = scales;
  bool fused_requant = false;
  const float* given_thr = nullptr;
  const float* given_scale = nullptr;
  if (requant != QA_REQUANT_NONE) {
    R = requant_layout(L, requant);
    if (requant_in_tile(L, requant)) {
      fused_requant = true;
    } else if (!sparse && L->M <= kRecomputeMaxM && quantize_workspace_bytes(&R) != 0) {
      // separate passes, each forming gbar from the messages: sums of |gbar| -> thresholds, sums
      // of the kept |gbar| -> scales, then the update with both handed in.  (Not when Q(SynQ) is
      // a one-pass quantization, i.e. one scale for a vector that is a single tile while the
      // messages' buckets are smaller: that quantizer keeps no sums in a workspace.)
      if (!ws || ws_bytes < requant_need(L, &R)) return QA_ERR_WORKSPACE;
      if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
      char* p = static_cast<char*>(ws);
      float* s1 = reinterpret_cast<float*>(p);            p += align256((size_t)R.scale_stride * 4);
      const size_t qws = quantize_workspace_bytes(&R);
      rc = requant_sums_from_messages(make_args(L, codes, scales), &R, s1, nullptr, p, qws, &given_thr,
                                      stream);
      if (rc != QA_OK) return rc;
      given_scale = s1;
    } else {
      // separate passes: gbar -> workspace, quantize it as a one-worker message, then run the
      // update on that message (its decoded value s*c is q exactly)
      if (!ws || ws_bytes < requant_need(L, &R)) return QA_ERR_WORKSPACE;
      if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
      char* p = static_cast<char*>(ws);
      float* gbar = reinterpret_cast<float*>(p);        p += align256((size_t)L->d * sizeof(float));
      uint32_t* c1 = reinterpret_cast<uint32_t*>(p);    p += align256((size_t)R.code_stride * 4);
      float* s1 = reinterpret_cast<float*>(p);          p += align256((size_t)R.scale_stride * 4);
      float* th1 = reinterpret_cast<float*>(p);         p += align256((size_t)R.scale_stride * 4);
      const size_t qws = quantize_workspace_bytes(&R);
      StepArgs ag = make_args(L, codes, scales);
      ag.gbar = gbar;
      if (sparse) { ag.ind = ind; ag.ind_stride = ind_stride; }
      // the table-driven kernel also leaves the quantizer's first pass (tile sums of |gbar|) in
      // the quantizer's workspace
      const bool fuse_abs = qws != 0;
      if (fuse_abs) ag.abs_partials = reinterpret_cast<double*>(p);
      launch_mode<kAggregate>(ag, false, false, stream);
      const int64_t gs = (L->d + 3) & ~int64_t(3);
      rc = quantize_launch(&R, gbar, gs, c1, s1, th1, fuse_abs ? kQuantAbsPartialsGiven : 0u,
                           qws ? p : nullptr, qws, stream);
      if (rc != QA_OK) return rc;
      use = &R; use_codes = c1; use_scales = s1;
    }
  }

  StepArgs a = make_args(use, use_codes, use_scales);
  if (sparse && use == L) { a.ind = ind; a.ind_stride = ind_stride; }   // else: dense Q(SynQ) message
  a.x = x; a.G = G; a.z = z;
  a.eta = eta; a.lam_eta = lambda * eta; a.delta = delta;
  a.t_lam = (float)t * lambda;
  set_fast_limits(a, mode, eta, a.lam_eta, delta);
  if (given_thr) {
    a.rq_thr = given_thr; a.rq_scale = given_scale;
    a.rq_tiles = R.bucket ? R.bucket / kTile : tiles_of(L->d);
    if (mode == kQcmd) launch_mode_rq<kQcmd, kRqGiven>(a, track_z, stream);
    else launch_mode_rq<kQrda, kRqGiven>(a, false, stream);
    return launch_status();
  }
  if (mode == kQcmd) launch_mode<kQcmd>(a, track_z, fused_requant, stream);
  else launch_mode<kQrda>(a, false, fused_requant, stream);
  return launch_status();
}

// The server's part of Algorithm 1 as one call: messages in, q_t = Q(SynQ_t) out as a one-worker
// message.  One pass when the second quantization fits a tile; otherwise the average goes to the
// workspace (with the quantizer's tile sums) and the quantizer finishes.
static int aggregate_quantize_common(const qa_layout* L, const uint32_t* codes, const float* scales,
                                     int requant, uint32_t* q_codes, float* q_scales,
                                     float* q_thresholds, void* ws, size_t ws_bytes,
                                     hipStream_t stream, bool sparse, const uint32_t* ind,
                                     int64_t ind_stride, uint32_t* ind_syn) {
  int rc = check_layout(L);
  if (rc != QA_OK) return rc;
  if (!codes || !scales || !q_codes || !q_scales) return QA_ERR_INVALID_ARG;
  if (!aligned(ind_syn, 4)) return QA_ERR_ALIGNMENT;
  if (requant != QA_REQUANT_BUCKET && requant != QA_REQUANT_GLOBAL) return QA_ERR_INVALID_ARG;
  if (requant == QA_REQUANT_BUCKET && L->bucket == 0) return QA_ERR_INVALID_ARG;
  if (sparse) {
    if (!ind) return QA_ERR_INVALID_ARG;
    if (ind_stride != 0 && ind_stride < (L->d + 31) / 32) return QA_ERR_INVALID_ARG;
    if (!aligned(ind, 4)) return QA_ERR_ALIGNMENT;
    rc = check_sparse_layout(L);
    if (rc != QA_OK) return rc;
  }
  if (!aligned(codes, 4) || !aligned(scales, 4) || !aligned(q_codes, 4) || !aligned(q_scales, 4) ||
      !aligned(q_thresholds, 4))
    return QA_ERR_ALIGNMENT;
  if (tiles_of(L->d) > 0x7fffffffLL) return QA_ERR_INVALID_ARG;

  qa_layout D;
  if (sparse && !sparse_messages_fused(L)) {
    // decode first (and OR the indicators), then the dense call on what the decoder wrote
    rc = decode_into_workspace(L, ind, ind_stride, codes, &D, &codes, &ws, &ws_bytes, stream);
    if (rc != QA_OK) return rc;
    if (ind_syn) indicator_or_launch(L, ind, ind_stride, ind_syn, stream);
    L = &D;
    sparse = false;
  }

  StepArgs ag = make_args(L, codes, scales);
  if (sparse) { ag.ind = ind; ag.ind_stride = ind_stride; ag.ind_syn = ind_syn; }
  if (requant_in_tile(L, requant)) {
    ag.q_codes = q_codes; ag.q_scales = q_scales; ag.q_thresholds = q_thresholds;
    launch_mode<kAggregate>(ag, false, true, stream);
    return launch_status();
  }
  qa_layout R = requant_layout(L, requant);
  const size_t qws = quantize_workspace_bytes(&R);
  if (!ws || ws_bytes < align256((size_t)L->d * sizeof(float)) + qws) return QA_ERR_WORKSPACE;
  if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
  char* p = static_cast<char*>(ws);
  if (!sparse && qws != 0 && one_scale_everywhere(ag, &R) && tiles_of(L->d) >= 16384) {
    // three passes over the messages (sums, kept sums, codes) instead of writing the average out
    // (long vectors only: five launches against four, d = 2^24 and M = 8: 0.044 against 0.039 ms)
    const float* thr = nullptr;
    rc = requant_sums_from_messages(ag, &R, q_scales, q_thresholds, p, qws, &thr, stream);
    if (rc != QA_OK) return rc;
    SumArgs sa = sum_args(ag);
    sa.thr = thr; sa.q_codes = q_codes;
    const int64_t groups = (sa.ntiles + sa.tiles_per_group - 1) / sa.tiles_per_group;
    hipLaunchKernelGGL(requant_sums_kernel<2>, dim3((unsigned)groups), dim3(kThreads), 0, stream, sa);
    return launch_status();
  }
  float* gbar = reinterpret_cast<float*>(p);            p += align256((size_t)L->d * sizeof(float));
  ag.gbar = gbar;
  const bool fuse_abs = qws != 0;
  if (fuse_abs) ag.abs_partials = reinterpret_cast<double*>(p);
  launch_mode<kAggregate>(ag, false, false, stream);
  const int64_t gs = (L->d + 3) & ~int64_t(3);
  return quantize_launch(&R, gbar, gs, q_codes, q_scales, q_thresholds,
                         fuse_abs ? kQuantAbsPartialsGiven : 0u, qws ? p : nullptr, qws, stream);
}

// Tensor-list steps: the table-driven kernel with one work-group per piece.  The second
// quantization runs as separate passes: average -> workspace, quantize it per tensor as a
// one-worker message, update from that message.
size_t step_segments_workspace_bytes(const qa_segment_plan* P) {
  return align256((size_t)P->d * sizeof(float)) + align256((size_t)words_of(P->d) * 4) +
         2 * align256((size_t)P->n_seg * 4) + quantize_segments_workspace_bytes(P, 1);
}

static int step_segments_common(int mode, const qa_layout* L, const qa_segment_plan* P,
                                const uint32_t* codes, const float* scales, float* x, float* G,
                                float* z, bool track_z, int64_t t, float eta, float lambda,
                                float delta, int requant, void* ws, size_t ws_bytes,
                                hipStream_t stream) {
  int rc = check_layout(L);
  if (rc != QA_OK) return rc;
  rc = check_plan(P, L);
  if (rc != QA_OK) return rc;
  if (!codes || !scales || !x || !G) return QA_ERR_INVALID_ARG;
  if (mode == kQrda && !z) return QA_ERR_INVALID_ARG;
  if (!(eta > 0.0f) || !(lambda >= 0.0f) || !(delta > 0.0f)) return QA_ERR_INVALID_ARG;
  if (mode == kQrda && t < 1) return QA_ERR_INVALID_ARG;
  if (requant == QA_REQUANT_GLOBAL) return QA_ERR_UNSUPPORTED;
  if (requant != QA_REQUANT_NONE && requant != QA_REQUANT_BUCKET) return QA_ERR_INVALID_ARG;
  if (!aligned(x, 16) || !aligned(G, 16) || !aligned(z, 16) || !aligned(codes, 4) ||
      !aligned(scales, 4))
    return QA_ERR_ALIGNMENT;
  if (P->n_pieces == 0) return QA_OK;                    // every tensor is empty

  qa_layout R = *L;
  const uint32_t* use_codes = codes;
  const float* use_scales = scales;
  if (requant != QA_REQUANT_NONE) {
    if (!ws || ws_bytes < step_segments_workspace_bytes(P)) return QA_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
    R.M = 1; R.code_stride = words_of(L->d); R.scale_stride = P->n_seg;
    char* p = static_cast<char*>(ws);
    float* gbar = reinterpret_cast<float*>(p);        p += align256((size_t)L->d * sizeof(float));
    uint32_t* c1 = reinterpret_cast<uint32_t*>(p);    p += align256((size_t)R.code_stride * 4);
    float* s1 = reinterpret_cast<float*>(p);          p += align256((size_t)P->n_seg * 4);
    float* th1 = reinterpret_cast<float*>(p);         p += align256((size_t)P->n_seg * 4);
    StepArgs ag = make_args(L, codes, scales);
    ag.seg = seg_table_of(P);
    ag.gbar = gbar;
    launch_mode<kAggregate>(ag, false, false, stream);
    const int64_t gs = (L->d + 3) & ~int64_t(3);
    rc = quantize_segments_launch(&R, P, gbar, gs, c1, s1, th1, p,
                                  quantize_segments_workspace_bytes(P, 1), stream);
    if (rc != QA_OK) return rc;
    use_codes = c1; use_scales = s1;
  }
  StepArgs a = make_args(&R, use_codes, use_scales);
  a.seg = seg_table_of(P);
  a.x = x; a.G = G; a.z = z;
  a.eta = eta; a.lam_eta = lambda * eta; a.delta = delta;
  a.t_lam = (float)t * lambda;
  set_fast_limits(a, mode, eta, a.lam_eta, delta);
  if (mode == kQcmd) launch_mode<kQcmd>(a, track_z, false, stream);
  else launch_mode<kQrda>(a, false, false, stream);
  return launch_status();
}

}  // namespace qa

extern "C" size_t qa_segment_workspace_bytes(const qa_segment_plan* plan, int32_t M, int op) {
  using namespace qa;
  if (!plan || plan->d < 1 || plan->n_seg < 1 || plan->n_pieces < 0 || M < 1 || M > 4096) return 0;
  if (op == QA_OP_QUANTIZE) return quantize_segments_workspace_bytes(plan, M);
  if (op == QA_OP_STEP) return step_segments_workspace_bytes(plan);
  return 0;
}

extern "C" int qa_step_qcmd_segments(const qa_layout* layout, const qa_segment_plan* plan,
                                     const uint32_t* codes, const float* scales, float* x, float* G,
                                     float* z_or_null, float eta, float lambda, float delta,
                                     int requant, void* ws, size_t ws_bytes, void* stream) {
  return qa::step_segments_common(qa::kQcmd, layout, plan, codes, scales, x, G, z_or_null,
                                  z_or_null != nullptr, 1, eta, lambda, delta, requant, ws,
                                  ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int qa_step_qrda_segments(const qa_layout* layout, const qa_segment_plan* plan,
                                     const uint32_t* codes, const float* scales, float* x, float* G,
                                     float* z, int64_t t, float eta, float lambda, float delta,
                                     int requant, void* ws, size_t ws_bytes, void* stream) {
  return qa::step_segments_common(qa::kQrda, layout, plan, codes, scales, x, G, z, false, t, eta,
                                  lambda, delta, requant, ws, ws_bytes,
                                  static_cast<hipStream_t>(stream));
}

extern "C" int qa_aggregate_unpack(const qa_layout* layout, const uint32_t* codes,
                                   const float* scales, float* gbar_out, void* stream) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  if (!codes || !scales || !gbar_out) return QA_ERR_INVALID_ARG;
  if (!aligned(gbar_out, 16) || !aligned(codes, 4) || !aligned(scales, 4)) return QA_ERR_ALIGNMENT;
  if (tiles_of(layout->d) > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  StepArgs a = make_args(layout, codes, scales);
  a.gbar = gbar_out;
  launch_mode<kAggregate>(a, false, false, static_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int qa_step_qcmd(const qa_layout* layout, const uint32_t* codes, const float* scales,
                            float* x, float* G, float* z_or_null, float eta, float lambda,
                            float delta, int requant, void* ws, size_t ws_bytes, void* stream) {
  return qa::step_common(qa::kQcmd, layout, codes, scales, x, G, z_or_null, z_or_null != nullptr, 1,
                         eta, lambda, delta, requant, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

extern "C" int qa_step_qrda(const qa_layout* layout, const uint32_t* codes, const float* scales,
                            float* x, float* G, float* z, int64_t t, float eta, float lambda,
                            float delta, int requant, void* ws, size_t ws_bytes, void* stream) {
  return qa::step_common(qa::kQrda, layout, codes, scales, x, G, z, false, t, eta, lambda, delta,
                         requant, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int qa_step_qcmd_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                                     const uint32_t* sel_codes, const float* scales, float* x,
                                     float* G, float* z_or_null, float eta, float lambda, float delta,
                                     int requant, void* ws, size_t ws_bytes, void* stream) {
  return qa::step_common(qa::kQcmd, layout, sel_codes, scales, x, G, z_or_null, z_or_null != nullptr,
                         1, eta, lambda, delta, requant, ws, ws_bytes,
                         static_cast<hipStream_t>(stream), true, ind, ind_stride);
}

extern "C" int qa_step_qrda_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                                     const uint32_t* sel_codes, const float* scales, float* x,
                                     float* G, float* z, int64_t t, float eta, float lambda,
                                     float delta, int requant, void* ws, size_t ws_bytes,
                                     void* stream) {
  return qa::step_common(qa::kQrda, layout, sel_codes, scales, x, G, z, false, t, eta, lambda, delta,
                         requant, ws, ws_bytes, static_cast<hipStream_t>(stream), true, ind,
                         ind_stride);
}

extern "C" int qa_aggregate_quantize(const qa_layout* layout, const uint32_t* codes,
                                     const float* scales, int requant, uint32_t* q_codes,
                                     float* q_scales, float* q_thresholds, void* ws, size_t ws_bytes,
                                     void* stream) {
  return qa::aggregate_quantize_common(layout, codes, scales, requant, q_codes, q_scales,
                                       q_thresholds, ws, ws_bytes, static_cast<hipStream_t>(stream),
                                       false, nullptr, 0, nullptr);
}

extern "C" int qa_aggregate_quantize_selected(const qa_layout* layout, const uint32_t* ind,
                                              int64_t ind_stride, const uint32_t* sel_codes,
                                              const float* scales, int requant, uint32_t* q_codes,
                                              float* q_scales, float* q_thresholds,
                                              uint32_t* ind_syn_out, void* ws, size_t ws_bytes,
                                              void* stream) {
  return qa::aggregate_quantize_common(layout, sel_codes, scales, requant, q_codes, q_scales,
                                       q_thresholds, ws, ws_bytes, static_cast<hipStream_t>(stream),
                                       true, ind, ind_stride, ind_syn_out);
}

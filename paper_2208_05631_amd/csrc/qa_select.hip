// Indicator, selection and sparse encoding (Section 3.2, equations "select" and "ind";
// Algorithm 1 worker block and server decode; Encode paragraph: 32 + d + 2k bits) for gfx950.
//
//   indicator_kernel          : I_i = (x_i != 0) or (x^_i != 0), x^ being the worker's own QCMD/QRDA
//                               update from its full-precision gradient; one bit per coordinate,
//                               formed with wave ballots (64 consecutive coordinates per ballot).
//   quantize_selected_kernel  : per 4096-tile, threshold/scale over the marked components only and
//                               their 2-bit codes compacted in index order (block prefix sum of
//                               the per-thread popcounts, LDS bit stream).
//   decode_selected_kernel    : S^{-1}: spreads the compact codes back to the dense 2-bit layout
//                               that the fused steps read.
//   select_codes_kernel       : S applied to a coded message (the server's push): the inverse.
// (The steps that read sparse messages directly live with the step kernel.)
#include "qa_common.h"
#include "qa_sparse.h"

namespace qa {

struct SelArgs {
  const float* g; int64_t g_stride;
  const float* x; const float* G; const float* z;
  uint32_t* ind; const uint32_t* ind_in; int64_t ind_stride;
  uint32_t* sel_codes; const uint32_t* sel_in; uint32_t* dense; int64_t code_stride;
  int64_t dense_stride;        // words between workers in `dense` (the decoder's output)
  uint32_t* counts; float* scales; float* thresholds; int64_t scale_stride;
  int64_t d, W, NW;            // coordinates, dense code words, indicator words
  int M, method;
  float eta, lam_eta, delta, t_lam, thr_coef;
  // buckets other than one 4096-tile (the general kernels below)
  int seg;                     // threads per bucket inside a tile: bucket/16 for 64 <= bucket <= 4096
  int64_t nb, ntiles, tiles_per_bucket, area_words;   // buckets spanning several tiles
  uint32_t* ws_count; double* ws_s1; double* ws_s2; uint32_t* ws_c2; int64_t* ws_start; float* ws_thr;
};

// Granularity of a sparse message's buckets: one 4096-tile each; 64 .. 2048 coordinates, inside a
// tile (bucket j of a tile = the segment of seg = bucket/16 consecutive code words, its compact
// stream starts at word j*seg of the tile's 256 words); or spanning several tiles.
enum SelKind { kSelTile, kSelLocal, kSelMulti };

// The worker's own would-be parameter from gradient component g (same operation order as the
// update of the fused steps).
__device__ __forceinline__ float local_update(const SelArgs& a, float g, float x, float G, float z) {
  const float g2 = g * g;
  const float Gh = G + g2;
  const float H = a.delta + sqrtf(Gh);
  if (a.method == 0) {
    const float step = (a.eta * g) / H;
    const float u = x - step;
    const float tau = a.lam_eta / H;
    const float r = fabsf(u) - tau;
    return r > 0.0f ? copysignf(r, u) : 0.0f;
  }
  const float zh = z + g;
  const float r = fabsf(zh) - a.t_lam;
  const float mag = (a.eta * r) / H;
  return r > 0.0f ? -copysignf(mag, zh) : 0.0f;
}

// Whether the worker's own update is non-zero, decided without square root or division whenever
// that is provably the same as evaluating local_update():
//   QCMD with x == 0:  x^ != 0  <=>  fl(a/H) > fl(b/H),  a = |fl(eta*g)|, b = fl(lambda*eta).
//     Correctly rounded division by the same H > 0 is monotone, so a <= b gives "zero"; and if
//     a > b*(1+2^-21) while b/H is a normal number, the two quotients differ by more than their
//     rounding errors (2^-24 relative each), which gives "non-zero".
//   QRDA:  r = fl(|fl(z+g)| - t*lambda) is formed exactly as in the update; r <= 0 gives "zero",
//     and r > 0 gives "non-zero" unless (eta*r)/H underflows to 0.
//   H <= delta + max(1, G + g*g) bounds the quotients away from the subnormal range.
// Everything else (ties within the margin, possible underflow, NaN/Inf) is left undecided and
// the caller evaluates the closed form itself.
// Written without branches: every lane runs the same straight-line code.
template <int METHOD>
__device__ __forceinline__ bool quick_indicator(const SelArgs& a, float g, float x, float G, float z,
                                                bool* mark) {
  const bool xnz = x != 0.0f;
  const float s2 = G + g * g;
  const bool valid = s2 >= 0.0f;                         // false for NaN or an invalid accumulator
  const float tiny = (a.delta + (s2 > 1.0f ? s2 : 1.0f)) * 0x1p-100f;
  bool m, decided;
  if (METHOD == 0) {
    const float av = fabsf(a.eta * g), b = a.lam_eta;
    m = av > b;
    decided = (av <= b) | ((av > b * 1.0000005f) & (b >= tiny));
  } else {
    const float zh = z + g;
    const float r = fabsf(zh) - a.t_lam;
    m = r > 0.0f;
    decided = !m | (a.eta * r >= tiny);
  }
  *mark = xnz | m;
  return xnz | (valid & decided);
}

// Rare path: the 1024 coordinates of one wave for worker m, all through the closed form.
__device__ __forceinline__ void indicator_slab_exact(const SelArgs& a, int m, int64_t base, int lane) {
  const float* g = a.g + (int64_t)m * a.g_stride;
  uint32_t* out = a.ind + (int64_t)m * a.ind_stride;
#pragma unroll 1
  for (int j = 0; j < 16; ++j) {
    const int64_t c = base + j * 64 + lane;
    bool mark = false;
    if (c < a.d) {
      const float x = a.x[c];
      const float xh = local_update(a, g[c], x, a.G[c], a.method == 1 ? a.z[c] : 0.0f);
      mark = x != 0.0f || xh != 0.0f;
    }
    const uint64_t bits = __ballot(mark);
    const int64_t w0 = (base + j * 64) / 32;
    if (lane < 2 && w0 + lane < a.NW) out[w0 + lane] = (uint32_t)(bits >> (32 * lane));
  }
}

// wave w of the work-group owns coordinates [w*1024, (w+1)*1024) of the tile, lane l the
// coordinates j*64 + l (j = 0..15): each ballot is 64 consecutive indicator bits.
// Slab that lies wholly below d: no clamps or masks; the next worker's gradient is requested
// before the current one is examined; ballot j (64 indicator bits) is kept by lane j, and lanes
// 0..15 store the slab's 128 bytes.
template <int METHOD>
__device__ __forceinline__ void indicator_wave_full(const SelArgs& a, int64_t base, int lane) {
  const float* px = a.x + base + lane;
  const float* pG = a.G + base + lane;
  const float* pz = METHOD == 1 ? a.z + base + lane : px;  // z may be null for QCMD
  float x[16], G[16], z[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    x[j] = px[j * 64];
    G[j] = pG[j * 64];
    z[j] = METHOD == 1 ? pz[j * 64] : 0.0f;
  }
  const float* pg = a.g + base + lane;
  uint32_t* out = a.ind + base / 32 + 2 * lane;
  float gn[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) gn[j] = pg[j * 64];
  for (int m = 0; m < a.M; ++m) {
    float gv[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) gv[j] = gn[j];
    if (m + 1 < a.M) {                                   // the next worker's gradient, ahead of use
      const float* pn = pg + (int64_t)(m + 1) * a.g_stride;
#pragma unroll
      for (int j = 0; j < 16; ++j) gn[j] = pn[j * 64];
    }
    bool undecided = false;
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      bool mark = false;
      undecided |= !quick_indicator<METHOD>(a, gv[j], x[j], G[j], z[j], &mark);
      const uint64_t bits = __ballot(mark);
      lo = lane == j ? (uint32_t)bits : lo;
      hi = lane == j ? (uint32_t)(bits >> 32) : hi;
    }
    if (__any(undecided)) {
      indicator_slab_exact(a, m, base, lane);
    } else if (lane < 16) {
      out[(int64_t)m * a.ind_stride] = lo;
      out[(int64_t)m * a.ind_stride + 1] = hi;
    }
  }
}

// Three waves per SIMD: measured best for this access pattern (2: 2.15 ms, 3: 1.91, 4: 1.98,
// 6-8: 2.00 at d = 2^28, M = 8); the kernel needs only 58-77 registers and would otherwise run 6-8.
template <int METHOD>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
void indicator_kernel(SelArgs a) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t base = (int64_t)blockIdx.x * kTile + wave * 1024;
  if (base + 1024 <= a.d) indicator_wave_full<METHOD>(a, base, lane);
  else if (base < a.d)                                   // the vector ends inside this slab: closed form
    for (int m = 0; m < a.M; ++m) indicator_slab_exact(a, m, base, lane);
}

__global__ __launch_bounds__(kThreads) void indicator_or_kernel(SelArgs a) {
  const int64_t w = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (w >= a.NW) return;
  uint32_t v = 0u;
  for (int m = 0; m < a.M; ++m) v |= a.ind_in[(int64_t)m * a.ind_stride + w];
  a.ind[w] = v;
}

// Exclusive prefix sum of `v` over the 256 threads and the total; two barriers.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* lds_w, uint32_t* total) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint32_t incl = wave_inclusive_scan_u32(v);
  __syncthreads();
  if (lane == kWave - 1) lds_w[wave] = incl;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t s = lds_w[w];
    if (w < wave) before += s;
    tot += s;
  }
  *total = tot;
  return before + incl - v;
}

// the 16 indicator bits of coordinates [16t, 16t+16) of tile `tile`
__device__ __forceinline__ uint32_t mask16_of(const uint32_t* ind, int64_t NW, int64_t tile, int t) {
  const int64_t w = tile * (kTile / 32) + t / 2;
  const uint32_t word = w < NW ? ind[w] : 0u;
  return (word >> (16 * (t & 1))) & 0xFFFFu;
}

__global__ __launch_bounds__(kThreads) void quantize_selected_kernel(SelArgs a) {
  __shared__ uint32_t stream[kTileWords + 1];
  __shared__ uint32_t lds_w[kWaves];
  __shared__ double lds_s1[kWaves];
  __shared__ double lds_s2[kWaves];
  __shared__ uint32_t lds_c[kWaves];
  const int t = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const float* g = a.g + (int64_t)m * a.g_stride;
  const uint32_t mask = mask16_of(a.ind_in + (int64_t)m * a.ind_stride, a.NW, tile, t);
  const int64_t i0 = tile * kTile + 16 * (int64_t)t;

  float v[16];
  if (i0 + 16 <= a.d) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 f = *reinterpret_cast<const float4*>(g + i0 + 4 * q);
      v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = (i0 + j < a.d) ? g[i0 + j] : 0.0f;
  }
  stream[t] = 0u;
  if (t == 0) stream[kTileWords] = 0u;

  double s1 = 0.0;
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((mask >> j) & 1u) s1 += (double)fabsf(v[j]);
  const uint32_t cnt = (uint32_t)__popc(mask);
  uint32_t K;
  const uint32_t before = block_exclusive_scan(cnt, lds_w, &K);
  const double S1 = block_sum_f64(s1, lds_s1);
  const float Delta = K ? threshold_from_sum(S1, a.thr_coef, (int64_t)K) : 0.0f;

  double s2 = 0.0;
  uint32_t c2 = 0, bits = 0, pos = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    if ((mask >> j) & 1u) {
      const float av = fabsf(v[j]);
      if (av > Delta) { s2 += (double)av; ++c2; }
      bits |= ternary_field(v[j], Delta) << (2 * pos);
      ++pos;
    }
  }
  // append this thread's 2*cnt bits at bit 2*before of the tile's compact stream
  if (cnt) {
    const uint32_t word = before / 16, sh = 2 * (before % 16);
    atomicOr(&stream[word], bits << sh);
    if (sh && (2 * cnt + sh > 32)) atomicOr(&stream[word + 1], bits >> (32 - sh));
  }
  s2 = wave_sum_f64(s2);
  c2 = wave_sum_u32(c2);
  if ((t % kWave) == 0) { lds_s2[t / kWave] = s2; lds_c[t / kWave] = c2; }
  __syncthreads();
  const uint32_t nwords = (K + 15) / 16;
  if ((uint32_t)t < nwords) (a.sel_codes + (int64_t)m * a.code_stride)[tile * kTileWords + t] = stream[t];
  if (t == 0) {
    const double S2 = (lds_s2[0] + lds_s2[1]) + (lds_s2[2] + lds_s2[3]);
    const uint32_t C = lds_c[0] + lds_c[1] + lds_c[2] + lds_c[3];
    a.counts[(int64_t)m * a.scale_stride + tile] = K;
    a.scales[(int64_t)m * a.scale_stride + tile] = scale_from_sum(S2, C);
    if (a.thresholds) a.thresholds[(int64_t)m * a.scale_stride + tile] = Delta;
  }
}

// A wave decodes kDecodeTiles consecutive 4096-tiles, phase by phase for all of them (their loads
// are independent and overlap).  Within a tile lane l holds code words j*64 + l (j = 0..3), so
// that each store instruction of the wave writes 256 consecutive bytes.  The position of a
// word's first marked component in the tile's compact stream is the number of marked components
// before it: a wave scan per j plus the totals of the earlier j.  The codes are spread to their
// fields four components at a time through the deposit table (copied to LDS once per block).
constexpr int kDecodeTiles = 2;

// kSelMulti: buckets that span tiles (and one scale per message of a long vector): a tile's codes
// start at code `start` of its bucket's stream, start being the tile's entry of the scan in the
// workspace: word start/16 of the bucket's area, code start%16 of that word.
// kSelLocal: a word's codes are counted from the start of its own bucket's stream, i.e. its
// position in the tile minus the position of the bucket's first word (same j and a lane of the
// wave for buckets up to 1024 coordinates, lane 0 of an even j for 2048).
template <int KIND>
__global__ __launch_bounds__(kThreads) void decode_selected_kernel(SelArgs a) {
  __shared__ uint8_t lut[16 * 256];
  reinterpret_cast<uint4*>(lut)[threadIdx.x] = reinterpret_cast<const uint4*>(kDepositLut.v)[threadIdx.x];
  const int lane = threadIdx.x % kWave;
  const int64_t tile0 = ((int64_t)blockIdx.x * kWaves + threadIdx.x / kWave) * kDecodeTiles;
  const int m = blockIdx.y;
  const uint32_t* ind = a.ind_in + (int64_t)m * a.ind_stride;
  uint32_t mask[kDecodeTiles][4], incl[kDecodeTiles][4];
#pragma unroll
  for (int u = 0; u < kDecodeTiles; ++u)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int wl = j * 64 + lane;                        // code word within the tile
      const int64_t iw = (tile0 + u) * (kTile / 32) + wl / 2;
      const uint32_t word = iw < a.NW ? ind[iw] : 0u;
      mask[u][j] = (word >> (16 * (wl & 1))) & 0xFFFFu;
    }
#pragma unroll
  for (int u = 0; u < kDecodeTiles; ++u)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // bits at or beyond d are not components: ignoring them keeps every read of the compact
      // stream inside the words that exist for this tile
      const int64_t left = a.d - ((tile0 + u) * kTile + (int64_t)(j * 64 + lane) * 16);
      if (left < 16) mask[u][j] = left > 0 ? (mask[u][j] & ((1u << left) - 1u)) : 0u;
      incl[u][j] = wave_inclusive_scan_u32((uint32_t)__popc(mask[u][j]));
    }
  uint32_t win_lo[kDecodeTiles][4], win_hi[kDecodeTiles][4], sh[kDecodeTiles][4];
#pragma unroll
  for (int u = 0; u < kDecodeTiles; ++u) {
    // clamped for tiles beyond the vector: their masks are 0, so nothing is read through it
    const int64_t tile = (tile0 + u) * kTile < a.d ? tile0 + u : 0;
    const uint32_t* sel = a.sel_in + (int64_t)m * a.code_stride;
    uint32_t start = 0;                                  // marked components in earlier j
    if (KIND == kSelMulti) {
      const int64_t first = a.ws_start[(int64_t)m * a.ntiles + tile];
      sel += (tile / a.tiles_per_bucket) * a.area_words + (first >> 4);
      start = (uint32_t)(first & 15);
    } else {
      sel += tile * kTileWords;
    }
    uint32_t ex[4];                                      // marked components of the tile before the word
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ex[j] = start + incl[u][j] - (uint32_t)__popc(mask[u][j]);
      start += (uint32_t)__builtin_amdgcn_readlane((int)incl[u][j], kWave - 1);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // the word's n <= 16 codes are codes before .. before+n-1 of the compact stream `src`:
      // word before/16 and, only if they cross a word boundary, the next one; both lie below
      // ceil(K/16) <= the words that exist for the stream (K = its marked components)
      const uint32_t n = (uint32_t)__popc(mask[u][j]);
      uint32_t before = ex[j];
      const uint32_t* src = sel;
      if (KIND == kSelLocal) {
        const int s0 = (j * 64 + lane) & ~(a.seg - 1);     // first code word of the bucket
        const uint32_t e0 = a.seg <= kWave ? (uint32_t)__shfl((int)ex[j], lane & ~(a.seg - 1), kWave)
                                           : (uint32_t)__builtin_amdgcn_readlane((int)ex[j & ~1], 0);
        before = ex[j] - e0;
        src = sel + s0;
      }
      const uint32_t w0 = before / 16;
      sh[u][j] = 2 * (before % 16);
      win_lo[u][j] = n != 0u ? src[w0] : 0u;
      win_hi[u][j] = (before % 16) + n > 16u ? src[w0 + 1] : 0u;
    }
  }
  __syncthreads();                                       // the table is in LDS
#pragma unroll
  for (int u = 0; u < kDecodeTiles; ++u)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t win = win_lo[u][j] >> sh[u][j];
      if (sh[u][j]) win |= win_hi[u][j] << (32 - sh[u][j]);
      uint32_t out = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t nib = (mask[u][j] >> (4 * q)) & 15u;
        out |= (uint32_t)lut[nib * 256 + (win & 0xFFu)] << (8 * q);
        win >>= 2 * __popc(nib);
      }
      const int64_t w = (tile0 + u) * kTileWords + j * 64 + lane;
      if (w < a.W) (a.dense + (int64_t)m * a.dense_stride)[w] = out;
    }
}

// Extract table, the inverse of the deposit table: entry [nib][s] packs the 2-bit fields of byte s
// at the set bits of nib towards bit 0 (lowest set bit first).
constexpr DepositLut make_extract_lut() {
  DepositLut t{};
  for (int nib = 0; nib < 16; ++nib)
    for (int s = 0; s < 256; ++s) {
      uint32_t out = 0;
      int n = 0;
      for (int b = 0; b < 4; ++b)
        if ((nib >> b) & 1) { out |= (((uint32_t)s >> (2 * b)) & 3u) << (2 * n); ++n; }
      t.v[nib * 256 + s] = (uint8_t)out;
    }
  return t;
}
__device__ const DepositLut kExtractLut = make_extract_lut();

// S applied to a coded message: one wave per 4096-tile, lane l holds code words j*64 + l of the
// tile (as in the decoder).  Each word's marked codes are packed through the extract table and
// appended at their position in the tile's compact stream, which is assembled in LDS (one area
// per wave) and written out in whole words.
// kSelMulti (buckets that span tiles): the tile's codes start at code start%16 of word start/16
// of the bucket's area (start from the scan in the workspace); words that a neighbouring tile may
// also touch are OR-ed into memory that was zeroed before, the others stored.
// kSelLocal (buckets inside a tile): bucket j's stream starts at word j*seg; its first
// ceil(K_j/16) words are written, and K_j by the bucket's first lane.
template <int KIND>
__global__ __launch_bounds__(kThreads) void select_codes_kernel(SelArgs a) {
  __shared__ uint8_t lut[16 * 256];
  __shared__ uint32_t stream_all[kWaves][kTileWords + 2];
  reinterpret_cast<uint4*>(lut)[threadIdx.x] = reinterpret_cast<const uint4*>(kExtractLut.v)[threadIdx.x];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  uint32_t* stream = stream_all[wave];
  const int64_t tile_raw = (int64_t)blockIdx.x * kWaves + wave;
  const bool exists = tile_raw * kTile < a.d;
  const int64_t tile = exists ? tile_raw : 0;            // clamped: every wave runs the same code
  const int m = blockIdx.y;
  const uint32_t* ind = a.ind_in + (int64_t)m * a.ind_stride;
  const uint32_t* dense = a.sel_in + (int64_t)m * a.code_stride + tile * kTileWords;
  uint32_t mask[4], word[4], incl[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int wl = j * 64 + lane;
    const int64_t iw = tile * (kTile / 32) + wl / 2;
    const uint32_t iv = iw < a.NW ? ind[iw] : 0u;
    mask[j] = (iv >> (16 * (wl & 1))) & 0xFFFFu;
    const int64_t left = a.d - (tile * kTile + (int64_t)wl * 16);
    if (left < 16) mask[j] = left > 0 ? (mask[j] & ((1u << left) - 1u)) : 0u;
    const int64_t w = tile * kTileWords + wl;
    const uint32_t raw = w < a.W ? dense[wl] : 0u;
    const uint32_t lo = raw & 0x55555555u;
    word[j] = lo | (raw & (lo << 1));                    // reserved pattern 10 reads as 0
    stream[wl] = 0u;
  }
  if (lane < 2) stream[kTileWords + lane] = 0u;
#pragma unroll
  for (int j = 0; j < 4; ++j) incl[j] = wave_inclusive_scan_u32((uint32_t)__popc(mask[j]));
  __syncthreads();                                       // table and zeroed streams are in LDS
  int64_t base = tile * kTileWords;
  uint32_t first = 0;
  if (KIND == kSelMulti) {
    const int64_t st = a.ws_start[(int64_t)m * a.ntiles + tile];
    base = (tile / a.tiles_per_bucket) * a.area_words + (st >> 4);
    first = (uint32_t)(st & 15);
  }
  uint32_t start = first, ex[4], total[4], in_bucket[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    total[j] = (uint32_t)__builtin_amdgcn_readlane((int)incl[j], kWave - 1);
    ex[j] = start + incl[j] - (uint32_t)__popc(mask[j]);
    start += total[j];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t n = (uint32_t)__popc(mask[j]);
    uint32_t before = ex[j];
    if (KIND == kSelLocal) {
      const int s0 = (j * 64 + lane) & ~(a.seg - 1);       // first code word of the bucket
      uint32_t e0, Kb = n;
      if (a.seg <= kWave) {
        e0 = (uint32_t)__shfl((int)ex[j], lane & ~(a.seg - 1), kWave);
        for (int off = 1; off < a.seg; off <<= 1) Kb += (uint32_t)__shfl_xor((int)Kb, off, kWave);
      } else {
        e0 = (uint32_t)__builtin_amdgcn_readlane((int)ex[j & ~1], 0);
        Kb = total[j] + total[j ^ 1];
      }
      in_bucket[j] = Kb;
      before = 16u * (uint32_t)s0 + (ex[j] - e0);
    }
    uint32_t bits = 0, filled = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t nib = (mask[j] >> (4 * q)) & 15u;
      bits |= (uint32_t)lut[nib * 256 + ((word[j] >> (8 * q)) & 0xFFu)] << filled;
      filled += 2 * __popc(nib);
    }
    if (n) {
      const uint32_t w0 = before / 16, sh = 2 * (before % 16);
      atomicOr(&stream[w0], bits << sh);
      if (sh && 2 * n + sh > 32) atomicOr(&stream[w0 + 1], bits >> (32 - sh));
    }
  }
  __syncthreads();
  if (exists) {
    const uint32_t end = start, nwords = (end + 15) / 16;  // one past the tile's last code
    uint32_t* out = a.sel_codes + (int64_t)m * a.code_stride + base;
    if (KIND == kSelMulti) {
      if (end != first)
        for (uint32_t w = lane; w < nwords; w += kWave) {  // at most 257 words
          const bool shared = (w == 0 && first != 0) || (w == nwords - 1 && (end % 16) != 0);
          if (shared) atomicOr(&out[w], stream[w]);
          else out[w] = stream[w];
        }
    } else if (KIND == kSelLocal) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int wl = j * 64 + lane, s0 = wl & ~(a.seg - 1);
        if ((uint32_t)(wl - s0) < (in_bucket[j] + 15) / 16) out[wl] = stream[wl];
        const int64_t kb = (tile * kTile + 16 * (int64_t)wl) / (16 * (int64_t)a.seg);
        if (wl == s0 && kb < a.nb) a.counts[(int64_t)m * a.scale_stride + kb] = in_bucket[j];
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((uint32_t)(j * 64 + lane) < nwords) out[j * 64 + lane] = stream[j * 64 + lane];
      if (lane == 0) a.counts[(int64_t)m * a.scale_stride + tile] = end;
    }
  }
}

// ---- any bucket size -------------------------------------------------------------------------
//
// The decoder and S above take every granularity (their KIND parameter); the quantizer above is
// the one for one threshold/scale per 4096-tile.  Below: the quantizers of the other
// granularities and the passes that buckets spanning tiles need.
//   * buckets of 64 .. 2048 coordinates lie inside a tile: bucket j of a tile is the segment of
//     seg = bucket/16 consecutive code words, its compact stream starts at word j*seg of the
//     tile's 256 words, and a word's codes start at (selected components of its bucket before it);
//   * buckets above 4096, and one scale for a vector of several tiles (the 32 + d + 2k bit
//     message of the Encode paragraph), span tiles: a first pass counts every tile's selected
//     components, a scan per bucket turns the counts into each tile's first position in the
//     bucket's stream (kept in the workspace), and the tiles then place or fetch their codes
//     there.  Neighbouring tiles share stream words, so producers OR their part into words that
//     a small kernel has zeroed first.

// the 16 indicator bits of the thread's coordinates, without those at or beyond d
__device__ __forceinline__ uint32_t live_mask16(const SelArgs& a, const uint32_t* ind, int64_t tile, int t) {
  const int64_t left = a.d - (tile * kTile + 16 * (int64_t)t);
  const uint32_t m = mask16_of(ind, a.NW, tile, t);
  return left >= 16 ? m : (left > 0 ? (m & ((1u << left) - 1u)) : 0u);
}

// the thread's 16 gradient components (coordinates 16t .. 16t+15 of the tile), 0 beyond d
__device__ __forceinline__ void load16(const float* __restrict__ g, int64_t d, int64_t i0, float v[16]) {
  if (i0 + 16 <= d) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 f = *reinterpret_cast<const float4*>(g + i0 + 4 * q);
      v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = (i0 + j < d) ? g[i0 + j] : 0.0f;
  }
}

// Where the thread's selected codes sit inside a tile whose buckets are segments of a.seg threads.
struct StreamPos {
  uint32_t pos;        // this thread's first selected code, counted from the tile's word 0
  uint32_t in_bucket;  // selected components of the thread's bucket
};

// n = number of selected components of this thread.  Contains barriers.
__device__ __forceinline__ StreamPos stream_position(const SelArgs& a, uint32_t n, uint32_t* lds_w,
                                                     uint32_t* lds_ex) {
  StreamPos p;
  const int t = threadIdx.x;
  uint32_t in_tile;
  const uint32_t ex = block_exclusive_scan(n, lds_w, &in_tile);
  lds_ex[t] = ex;
  if (t == 0) lds_ex[kThreads] = in_tile;
  __syncthreads();
  const int s0 = t & ~(a.seg - 1);
  p.in_bucket = lds_ex[s0 + a.seg] - lds_ex[s0];
  p.pos = 16u * (uint32_t)s0 + (ex - lds_ex[s0]);
  return p;
}

// OR `bits` (2*n bits) into the LDS stream at code position pos.
__device__ __forceinline__ void stream_append(uint32_t* stream, uint32_t pos, uint32_t n, uint32_t bits) {
  if (n == 0) return;
  const uint32_t word = pos / 16, sh = 2 * (pos % 16);
  atomicOr(&stream[word], bits << sh);
  if (sh && (2 * n + sh > 32)) atomicOr(&stream[word + 1], bits >> (32 - sh));
}

// pass 1 of the multi-tile quantizer: selected components of every tile and the sum of their
// magnitudes
__global__ __launch_bounds__(kThreads) void gsel_count_kernel(SelArgs a) {
  __shared__ uint32_t lds_w[kWaves];
  __shared__ double lds_d[kWaves];
  const int t = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const uint32_t mask = live_mask16(a, a.ind_in + (int64_t)m * a.ind_stride, tile, t);
  uint32_t K;
  block_exclusive_scan((uint32_t)__popc(mask), lds_w, &K);
  float v[16];
  load16(a.g + (int64_t)m * a.g_stride, a.d, tile * kTile + 16 * (int64_t)t, v);
  double s1 = 0.0;
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((mask >> j) & 1u) s1 += (double)fabsf(v[j]);
  const double S1 = block_sum_f64(s1, lds_d);
  if (t == 0) {
    a.ws_s1[(int64_t)m * a.ntiles + tile] = S1;
    a.ws_count[(int64_t)m * a.ntiles + tile] = K;
  }
}

// pass 1 without a gradient (decoder, S of a coded message): a wave counts kCountTiles
// consecutive tiles, lane l the indicator words 2l and 2l+1 of each tile (bits at or beyond d
// are not components).
constexpr int kCountTiles = 8;
__global__ __launch_bounds__(kThreads) void gsel_count_ind_kernel(SelArgs a) {
  const int lane = threadIdx.x % kWave;
  const int64_t tile0 = ((int64_t)blockIdx.x * kWaves + threadIdx.x / kWave) * kCountTiles;
  const int m = blockIdx.y;
  const uint32_t* ind = a.ind_in + (int64_t)m * a.ind_stride;
  uint32_t c[kCountTiles];
#pragma unroll
  for (int u = 0; u < kCountTiles; ++u) {
    c[u] = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int64_t iw = (tile0 + u) * (kTile / 32) + 2 * lane + h;
      uint32_t v = iw < a.NW ? ind[iw] : 0u;
      const int64_t left = a.d - 32 * iw;
      if (left < 32) v = left > 0 ? (v & ((1u << left) - 1u)) : 0u;
      c[u] += (uint32_t)__popc(v);
    }
  }
#pragma unroll
  for (int u = 0; u < kCountTiles; ++u) {
    const uint32_t K = wave_sum_u32(c[u]);
    if (lane == 0 && tile0 + u < a.ntiles) a.ws_count[(int64_t)m * a.ntiles + tile0 + u] = K;
  }
}

// pass 2: per (bucket, worker), in tile order: each tile's first position in the bucket's stream,
// the bucket's count and (with a gradient) its threshold.  One work-group per bucket; a round takes
// 256 x 16 consecutive tiles (thread t the 16 from t*16 on) with a running offset, so the order
// of the binary64 additions is fixed.
constexpr int kScanRun = 16;
template <bool HAS_G>
__global__ __launch_bounds__(kThreads) void gsel_scan_kernel(SelArgs a) {
  __shared__ uint32_t lds_w[kWaves];
  __shared__ double lds_d[kWaves];
  const int t = threadIdx.x;
  const int64_t k = blockIdx.x;
  const int m = blockIdx.y;
  const int64_t t0 = k * a.tiles_per_bucket;
  const int64_t t1 = t0 + a.tiles_per_bucket < a.ntiles ? t0 + a.tiles_per_bucket : a.ntiles;
  const uint32_t* cnt = a.ws_count + (int64_t)m * a.ntiles;
  const double* s1p = a.ws_s1 + (int64_t)m * a.ntiles;
  int64_t* start = a.ws_start + (int64_t)m * a.ntiles;
  int64_t running = 0;
  double s1 = 0.0;
  for (int64_t i = t0; i < t1; i += (int64_t)kThreads * kScanRun) {
    const int64_t j0 = i + (int64_t)t * kScanRun;
    uint32_t c[kScanRun], mine = 0;
#pragma unroll
    for (int u = 0; u < kScanRun; ++u) {
      c[u] = j0 + u < t1 ? cnt[j0 + u] : 0u;
      mine += c[u];
      if (HAS_G && j0 + u < t1) s1 += s1p[j0 + u];
    }
    uint32_t total;
    uint32_t ex = block_exclusive_scan(mine, lds_w, &total);   // at most 256 x 16 x 4096 = 2^24
#pragma unroll
    for (int u = 0; u < kScanRun; ++u) {
      if (j0 + u < t1) start[j0 + u] = running + ex;
      ex += c[u];
    }
    running += total;
  }
  if (HAS_G) s1 = block_sum_f64(s1, lds_d);
  if (t == 0) {
    a.counts[(int64_t)m * a.scale_stride + k] = (uint32_t)running;   // a bucket holds < 2^32 here
    if (HAS_G) {
      const float Delta = running ? threshold_from_sum(s1, a.thr_coef, running) : 0.0f;
      a.ws_thr[(int64_t)m * a.nb + k] = Delta;
      if (a.thresholds) a.thresholds[(int64_t)m * a.scale_stride + k] = Delta;
    }
  }
}

// zero the first ceil(K/16) words of every bucket's area (a tile covers 256 of them, a work-group
// kZeroTiles consecutive tiles)
constexpr int kZeroTiles = 8;
__global__ __launch_bounds__(kThreads) void gsel_zero_kernel(SelArgs a) {
  const int m = blockIdx.y;
#pragma unroll
  for (int u = 0; u < kZeroTiles; ++u) {
    const int64_t tile = (int64_t)blockIdx.x * kZeroTiles + u;
    if (tile >= a.ntiles) break;
    const int64_t k = tile / a.tiles_per_bucket;
    const int64_t w = (tile - k * a.tiles_per_bucket) * kTileWords + threadIdx.x;   // word of the area
    const int64_t K = a.counts[(int64_t)m * a.scale_stride + k];
    if (w < (K + 15) / 16) a.sel_codes[(int64_t)m * a.code_stride + k * a.area_words + w] = 0u;
  }
}

// Q(S(g, I)) for buckets of 64 .. 2048 coordinates: thread t = code word t of the tile, a bucket =
// a.seg consecutive threads.
__global__ __launch_bounds__(kThreads) void gsel_quantize_local_kernel(SelArgs a) {
  __shared__ uint32_t stream[kTileWords + 2];
  __shared__ uint32_t lds_w[kWaves];
  __shared__ uint32_t lds_ex[kThreads + 1];
  __shared__ double lds_d[kWaves];
  __shared__ uint32_t lds_u[kWaves];
  const int t = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int m = blockIdx.y;
  const float* g = a.g + (int64_t)m * a.g_stride;
  const uint32_t mask = live_mask16(a, a.ind_in + (int64_t)m * a.ind_stride, tile, t);
  float v[16];
  load16(g, a.d, tile * kTile + 16 * (int64_t)t, v);
  stream[t] = 0u;
  if (t < 2) stream[kTileWords + t] = 0u;
  const uint32_t n = (uint32_t)__popc(mask);
  const StreamPos p = stream_position(a, n, lds_w, lds_ex);   // barriers: stream is zero

  double s1 = 0.0;
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((mask >> j) & 1u) s1 += (double)fabsf(v[j]);
  const double S1 = segment_sum(s1, a.seg, lds_d);
  const float Delta = p.in_bucket ? threshold_from_sum(S1, a.thr_coef, (int64_t)p.in_bucket) : 0.0f;
  double s2 = 0.0;
  uint32_t c2 = 0, bits = 0, k = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    if ((mask >> j) & 1u) {
      const float av = fabsf(v[j]);
      if (av > Delta) { s2 += (double)av; ++c2; }
      bits |= ternary_field(v[j], Delta) << (2 * k);
      ++k;
    }
  }
  stream_append(stream, p.pos, n, bits);
  __syncthreads();                                       // lds_d of the first sum has been read
  const double S2 = segment_sum(s2, a.seg, lds_d);
  const uint32_t C2 = segment_sum_u32(c2, a.seg, lds_u);
  __syncthreads();                                       // the stream is complete
  // the first ceil(K/16) words of each bucket's area, nothing else
  const int s0 = t & ~(a.seg - 1);
  uint32_t* row = a.sel_codes + (int64_t)m * a.code_stride + tile * kTileWords;
  if ((uint32_t)(t - s0) < (p.in_bucket + 15) / 16) row[t] = stream[t];
  if (t == s0) {
    const int64_t kb = (tile * kTile + 16 * (int64_t)t) / (16 * (int64_t)a.seg);
    if (kb < a.nb) {
      a.counts[(int64_t)m * a.scale_stride + kb] = p.in_bucket;
      a.scales[(int64_t)m * a.scale_stride + kb] = scale_from_sum(S2, C2);
      if (a.thresholds) a.thresholds[(int64_t)m * a.scale_stride + kb] = Delta;
    }
  }
}

// Q(S(g, I)) for buckets that span tiles, one wave per tile and no work-group barrier on the way
// (lane l holds code words j*64 + l of the tile, j = 0..3, as in the decoder): the threshold comes
// from pass 2, the tile's codes go to their place in the bucket's stream (words that a
// neighbouring tile may also touch are OR-ed into memory zeroed before), the tile's kept sum and
// count to the workspace for gsel_scale_kernel.
__global__ __launch_bounds__(kThreads) void gsel_quantize_multi_kernel(SelArgs a) {
  __shared__ uint32_t stream_all[kWaves][kTileWords + 2];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  uint32_t* stream = stream_all[wave];
  const int64_t tile_raw = (int64_t)blockIdx.x * kWaves + wave;
  const bool exists = tile_raw < a.ntiles;
  const int64_t tile = exists ? tile_raw : 0;            // clamped: every wave runs the same code
  const int m = blockIdx.y;
  const uint32_t* ind = a.ind_in + (int64_t)m * a.ind_stride;
  const float* g = a.g + (int64_t)m * a.g_stride;
  uint32_t mask[4], incl[4];
  float v[4][16];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int wl = j * 64 + lane;
    const int64_t iw = tile * (kTile / 32) + wl / 2;
    const uint32_t iv = iw < a.NW ? ind[iw] : 0u;
    mask[j] = (iv >> (16 * (wl & 1))) & 0xFFFFu;
    const int64_t left = a.d - (tile * kTile + (int64_t)wl * 16);
    if (left < 16) mask[j] = left > 0 ? (mask[j] & ((1u << left) - 1u)) : 0u;
    load16(g, a.d, tile * kTile + (int64_t)wl * 16, v[j]);
    stream[wl] = 0u;
  }
  if (lane < 2) stream[kTileWords + lane] = 0u;
#pragma unroll
  for (int j = 0; j < 4; ++j) incl[j] = wave_inclusive_scan_u32((uint32_t)__popc(mask[j]));
  const int64_t st = a.ws_start[(int64_t)m * a.ntiles + tile];
  const int64_t k = tile / a.tiles_per_bucket;
  const uint32_t first = (uint32_t)(st & 15);
  const float Delta = a.ws_thr[(int64_t)m * a.nb + k];
  __syncthreads();                                       // the zeroed streams are in LDS
  double s2 = 0.0;
  uint32_t c2 = 0, start = first;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t n = (uint32_t)__popc(mask[j]);
    const uint32_t before = start + incl[j] - n;
    start += (uint32_t)__builtin_amdgcn_readlane((int)incl[j], kWave - 1);
    uint32_t bits = 0, filled = 0;
#pragma unroll
    for (int c = 0; c < 16; ++c)
      if ((mask[j] >> c) & 1u) {
        const float av = fabsf(v[j][c]);
        if (av > Delta) { s2 += (double)av; ++c2; }
        bits |= ternary_field(v[j][c], Delta) << filled;
        filled += 2;
      }
    if (n) {
      const uint32_t w0 = before / 16, sh = 2 * (before % 16);
      atomicOr(&stream[w0], bits << sh);
      if (sh && 2 * n + sh > 32) atomicOr(&stream[w0 + 1], bits >> (32 - sh));
    }
  }
  const double S2 = wave_sum_f64(s2);
  const uint32_t C2 = wave_sum_u32(c2);
  __syncthreads();                                       // the streams are complete
  if (exists) {
    const uint32_t end = start, nwords = (end + 15) / 16;  // one past the tile's last code
    uint32_t* out = a.sel_codes + (int64_t)m * a.code_stride + k * a.area_words + (st >> 4);
    if (end != first)
      for (uint32_t w = lane; w < nwords; w += kWave) {    // at most 257 words
        const bool shared = (w == 0 && first != 0) || (w == nwords - 1 && (end % 16) != 0);
        if (shared) atomicOr(&out[w], stream[w]);
        else out[w] = stream[w];
      }
    if (lane == 0) {
      a.ws_s2[(int64_t)m * a.ntiles + tile] = S2;
      a.ws_c2[(int64_t)m * a.ntiles + tile] = C2;
    }
  }
}

// last pass of the multi-tile quantizer: scale of each (bucket, worker)
__global__ __launch_bounds__(kThreads) QA_FEW_WAVES void gsel_scale_kernel(SelArgs a) {
  __shared__ double lds_d[kWaves];
  __shared__ double lds_c[kWaves];
  const int64_t k = blockIdx.x;
  const int m = blockIdx.y;
  const int64_t t0 = k * a.tiles_per_bucket;
  const int64_t t1 = t0 + a.tiles_per_bucket < a.ntiles ? t0 + a.tiles_per_bucket : a.ntiles;
  double s, c;
  strided_partial_sums(a.ws_s2 + (int64_t)m * a.ntiles, a.ws_c2 + (int64_t)m * a.ntiles, t0, t1, &s, &c);
  s = segment_sum(s, kThreads, lds_d);
  c = segment_sum(c, kThreads, lds_c);
  if (threadIdx.x == 0) a.scales[(int64_t)m * a.scale_stride + k] = scale_from_sum(s, (uint64_t)c);
}

// Which kernels serve a layout's sparse messages.
static SelKind sel_kind(const qa_layout* L) {
  if (L->bucket == kTile || (L->bucket == 0 && L->d <= kTile)) return kSelTile;   // the tuned kernels
  if (L->bucket != 0 && L->bucket < kTile) return kSelLocal;                        // buckets inside a tile
  return kSelMulti;                                                                 // buckets over several tiles
}

static inline size_t sel_align(size_t v) { return (v + 255) & ~size_t(255); }
static inline dim3 zero_grid(const qa_layout* L) {
  return dim3((unsigned)((tiles_of(L->d) + kZeroTiles - 1) / kZeroTiles), (unsigned)L->M);
}
static inline dim3 count_grid(const qa_layout* L) {
  return dim3((unsigned)((tiles_of(L->d) + kWaves * kCountTiles - 1) / (kWaves * kCountTiles)), (unsigned)L->M);
}

// Workspace of the multi-tile path: per (worker, tile) a count, two binary64 sums, a kept count and
// the tile's first position in its bucket's stream; per (worker, bucket) a threshold.
size_t select_workspace_bytes(const qa_layout* L) {
  if (sel_kind(L) != kSelMulti) return 0;
  const size_t mt = (size_t)L->M * (size_t)tiles_of(L->d);
  return sel_align(mt * 4) + 2 * sel_align(mt * 8) + sel_align(mt * 4) + sel_align(mt * 8) +
         sel_align((size_t)L->M * (size_t)buckets_of(L->d, L->bucket) * 4);
}

static int check_select_layout(const qa_layout* L) {
  int rc = check_layout(L);
  if (rc != QA_OK) return rc;
  // a bucket's selected count is kept in 32 bits
  const int64_t blen = L->bucket ? L->bucket : L->d;
  if (blen >= (int64_t(1) << 32)) return QA_ERR_UNSUPPORTED;
  return QA_OK;
}

// Geometry of the general kernels and, for multi-tile buckets, the workspace pointers.
static int general_args(const qa_layout* L, SelArgs& a, void* ws, size_t ws_bytes) {
  const SelKind kind = sel_kind(L);
  a.nb = buckets_of(L->d, L->bucket);
  a.ntiles = tiles_of(L->d);
  a.seg = kind == kSelLocal ? L->bucket / 16 : kThreads;
  if (kind != kSelMulti) return QA_OK;
  const size_t need = select_workspace_bytes(L);
  if (!ws || ws_bytes < need) return QA_ERR_WORKSPACE;
  if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
  a.tiles_per_bucket = L->bucket ? L->bucket / kTile : a.ntiles;
  a.area_words = L->bucket ? L->bucket / 16 : words_of(L->d);
  const size_t mt = (size_t)L->M * (size_t)a.ntiles;
  char* p = static_cast<char*>(ws);
  a.ws_count = reinterpret_cast<uint32_t*>(p); p += sel_align(mt * 4);
  a.ws_s1 = reinterpret_cast<double*>(p);      p += sel_align(mt * 8);
  a.ws_s2 = reinterpret_cast<double*>(p);      p += sel_align(mt * 8);
  a.ws_c2 = reinterpret_cast<uint32_t*>(p);    p += sel_align(mt * 4);
  a.ws_start = reinterpret_cast<int64_t*>(p);  p += sel_align(mt * 8);
  a.ws_thr = reinterpret_cast<float*>(p);
  return QA_OK;
}

static SelArgs base_args(const qa_layout* L) {
  SelArgs a{};
  a.d = L->d; a.W = words_of(L->d); a.NW = (L->d + 31) / 32; a.M = L->M;
  a.code_stride = L->code_stride; a.scale_stride = L->scale_stride; a.thr_coef = L->thr_coef;
  return a;
}

}  // namespace qa

extern "C" int qa_indicator(const qa_layout* layout, int method, const float* g, int64_t g_stride,
                            const float* x, const float* G, const float* z, int64_t t, float eta,
                            float lambda, float delta, uint32_t* ind_out, int64_t ind_stride,
                            void* stream) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  if (method != 0 && method != 1) return QA_ERR_INVALID_ARG;
  if (!g || !x || !G || !ind_out || (method == 1 && !z)) return QA_ERR_INVALID_ARG;
  if (g_stride < layout->d || ind_stride < (layout->d + 31) / 32) return QA_ERR_INVALID_ARG;
  if (!(eta > 0.0f) || !(lambda >= 0.0f) || !(delta > 0.0f) || (method == 1 && t < 1))
    return QA_ERR_INVALID_ARG;
  if (!aligned(g, 4) || !aligned(x, 4) || !aligned(G, 4) || !aligned(z, 4) || !aligned(ind_out, 4))
    return QA_ERR_ALIGNMENT;
  SelArgs a = base_args(layout);
  a.method = method; a.g = g; a.g_stride = g_stride; a.x = x; a.G = G; a.z = z;
  a.ind = ind_out; a.ind_stride = ind_stride;
  a.eta = eta; a.lam_eta = lambda * eta; a.delta = delta; a.t_lam = (float)t * lambda;
  const dim3 grid((unsigned)tiles_of(layout->d)), block(kThreads);
  if (method == 0) hipLaunchKernelGGL(indicator_kernel<0>, grid, block, 0, static_cast<hipStream_t>(stream), a);
  else hipLaunchKernelGGL(indicator_kernel<1>, grid, block, 0, static_cast<hipStream_t>(stream), a);
  return launch_status();
}

namespace qa {
// does the fused step read this layout's sparse messages itself (one threshold/scale per tile)?
bool sparse_messages_fused(const qa_layout* L) { return sel_kind(L) == kSelTile; }
int check_sparse_layout(const qa_layout* L) { return check_select_layout(L); }

void indicator_or_launch(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                         uint32_t* ind_syn_out, hipStream_t stream) {
  SelArgs a = base_args(layout);
  a.ind_in = ind; a.ind_stride = ind_stride; a.ind = ind_syn_out;
  hipLaunchKernelGGL(indicator_or_kernel, dim3((unsigned)((a.NW + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, stream, a);
}
}  // namespace qa

extern "C" int qa_indicator_or(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                               uint32_t* ind_syn_out, void* stream) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  if (!ind || !ind_syn_out || ind_stride < (layout->d + 31) / 32) return QA_ERR_INVALID_ARG;
  if (!aligned(ind, 4) || !aligned(ind_syn_out, 4)) return QA_ERR_ALIGNMENT;
  indicator_or_launch(layout, ind, ind_stride, ind_syn_out, static_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int qa_quantize_pack_selected(const qa_layout* layout, const float* g, int64_t g_stride,
                                         const uint32_t* ind, int64_t ind_stride, uint32_t* sel_codes,
                                         uint32_t* counts, float* scales, float* thresholds,
                                         void* ws, size_t ws_bytes, void* stream_) {
  using namespace qa;
  int rc = check_select_layout(layout);
  if (rc != QA_OK) return rc;
  if (!g || !ind || !sel_codes || !counts || !scales) return QA_ERR_INVALID_ARG;
  if (g_stride < layout->d || (g_stride % 4) != 0 || ind_stride < (layout->d + 31) / 32)
    return QA_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(ind, 4) || !aligned(sel_codes, 4) || !aligned(counts, 4) ||
      !aligned(scales, 4) || !aligned(thresholds, 4))
    return QA_ERR_ALIGNMENT;
  if (tiles_of(layout->d) > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  SelArgs a = base_args(layout);
  a.g = g; a.g_stride = g_stride; a.ind_in = ind; a.ind_stride = ind_stride;
  a.sel_codes = sel_codes; a.counts = counts; a.scales = scales; a.thresholds = thresholds;
  const dim3 block(kThreads), tiles((unsigned)tiles_of(layout->d), (unsigned)layout->M);
  const SelKind kind = sel_kind(layout);
  if (kind == kSelTile) {
    hipLaunchKernelGGL(quantize_selected_kernel, tiles, block, 0, stream, a);
    return launch_status();
  }
  rc = general_args(layout, a, ws, ws_bytes);
  if (rc != QA_OK) return rc;
  if (kind == kSelLocal) {
    hipLaunchKernelGGL(gsel_quantize_local_kernel, tiles, block, 0, stream, a);
    return launch_status();
  }
  const dim3 buckets((unsigned)a.nb, (unsigned)layout->M);
  hipLaunchKernelGGL(gsel_count_kernel, tiles, block, 0, stream, a);
  hipLaunchKernelGGL(gsel_scan_kernel<true>, buckets, block, 0, stream, a);
  hipLaunchKernelGGL(gsel_zero_kernel, zero_grid(layout), block, 0, stream, a);
  hipLaunchKernelGGL(gsel_quantize_multi_kernel,
                     dim3((unsigned)((tiles_of(layout->d) + kWaves - 1) / kWaves), (unsigned)layout->M),
                     block, 0, stream, a);
  hipLaunchKernelGGL(gsel_scale_kernel, buckets, block, 0, stream, a);
  return launch_status();
}

namespace qa {
// S^{-1} for all M messages into dense code words; shared with the steps that take sparse
// messages of other bucket sizes than 4096.  `counts_scratch` (multi-tile buckets only) receives
// the per-bucket counts that the scan produces on the way; it may be the workspace's own.
int decode_selected_launch(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                           const uint32_t* sel_codes, uint32_t* codes_out, int64_t out_stride,
                           void* ws, size_t ws_bytes, hipStream_t stream) {
  SelArgs a = base_args(layout);
  a.ind_in = ind; a.ind_stride = ind_stride; a.sel_in = sel_codes; a.dense = codes_out;
  a.dense_stride = out_stride;
  const dim3 block(kThreads), tiles((unsigned)tiles_of(layout->d), (unsigned)layout->M);
  const SelKind kind = sel_kind(layout);
  const dim3 wave_tiles((unsigned)((tiles_of(layout->d) + kWaves * kDecodeTiles - 1) / (kWaves * kDecodeTiles)),
                        (unsigned)layout->M);
  if (kind == kSelTile) {
    hipLaunchKernelGGL(decode_selected_kernel<kSelTile>, wave_tiles, block, 0, stream, a);
    return launch_status();
  }
  int rc = general_args(layout, a, ws, ws_bytes);
  if (rc != QA_OK) return rc;
  if (kind == kSelLocal) {
    hipLaunchKernelGGL(decode_selected_kernel<kSelLocal>, wave_tiles, block, 0, stream, a);
    return launch_status();
  }
  // the scan also leaves each bucket's count; nobody asked for it here: the kept-count slots of
  // the workspace (unused by a decode) take it, M*nb <= M*ntiles words
  a.counts = a.ws_c2; a.scale_stride = a.nb;
  hipLaunchKernelGGL(gsel_count_ind_kernel, count_grid(layout), block, 0, stream, a);
  hipLaunchKernelGGL(gsel_scan_kernel<false>, dim3((unsigned)a.nb, (unsigned)layout->M), block, 0, stream, a);
  hipLaunchKernelGGL(decode_selected_kernel<kSelMulti>, wave_tiles, block, 0, stream, a);
  return launch_status();
}
}  // namespace qa

extern "C" int qa_decode_selected(const qa_layout* layout, const uint32_t* ind, int64_t ind_stride,
                                  const uint32_t* sel_codes, uint32_t* codes_out, void* ws,
                                  size_t ws_bytes, void* stream) {
  using namespace qa;
  int rc = check_select_layout(layout);
  if (rc != QA_OK) return rc;
  if (!ind || !sel_codes || !codes_out) return QA_ERR_INVALID_ARG;
  if (ind_stride != 0 && ind_stride < (layout->d + 31) / 32) return QA_ERR_INVALID_ARG;
  if (!aligned(ind, 4) || !aligned(sel_codes, 4) || !aligned(codes_out, 4)) return QA_ERR_ALIGNMENT;
  if (tiles_of(layout->d) > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  return decode_selected_launch(layout, ind, ind_stride, sel_codes, codes_out, layout->code_stride, ws,
                                ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int qa_select_codes(const qa_layout* layout, const uint32_t* codes, const uint32_t* ind,
                               int64_t ind_stride, uint32_t* sel_codes, uint32_t* counts, void* ws,
                               size_t ws_bytes, void* stream_) {
  using namespace qa;
  int rc = check_select_layout(layout);
  if (rc != QA_OK) return rc;
  if (!codes || !ind || !sel_codes || !counts) return QA_ERR_INVALID_ARG;
  if (ind_stride != 0 && ind_stride < (layout->d + 31) / 32) return QA_ERR_INVALID_ARG;
  if (!aligned(codes, 4) || !aligned(ind, 4) || !aligned(sel_codes, 4) || !aligned(counts, 4))
    return QA_ERR_ALIGNMENT;
  if (codes == sel_codes) return QA_ERR_INVALID_ARG;       // not in place
  if (tiles_of(layout->d) > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  SelArgs a = base_args(layout);
  a.ind_in = ind; a.ind_stride = ind_stride; a.sel_in = codes; a.sel_codes = sel_codes; a.counts = counts;
  const dim3 block(kThreads), tiles((unsigned)tiles_of(layout->d), (unsigned)layout->M);
  const SelKind kind = sel_kind(layout);
  const dim3 wave_tiles((unsigned)((tiles_of(layout->d) + kWaves - 1) / kWaves), (unsigned)layout->M);
  if (kind == kSelTile) {
    hipLaunchKernelGGL(select_codes_kernel<kSelTile>, wave_tiles, block, 0, stream, a);
    return launch_status();
  }
  rc = general_args(layout, a, ws, ws_bytes);
  if (rc != QA_OK) return rc;
  if (kind == kSelLocal) {
    hipLaunchKernelGGL(select_codes_kernel<kSelLocal>, wave_tiles, block, 0, stream, a);
    return launch_status();
  }
  hipLaunchKernelGGL(gsel_count_ind_kernel, count_grid(layout), block, 0, stream, a);
  hipLaunchKernelGGL(gsel_scan_kernel<false>, dim3((unsigned)a.nb, (unsigned)layout->M), block, 0, stream, a);
  hipLaunchKernelGGL(gsel_zero_kernel, zero_grid(layout), block, 0, stream, a);
  hipLaunchKernelGGL(select_codes_kernel<kSelMulti>, wave_tiles, block, 0, stream, a);
  return launch_status();
}

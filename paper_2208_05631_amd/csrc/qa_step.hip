// Server average and fused QCMD / QRDA adagrad steps (Section 3.2 and Algorithm 1 of
// arXiv 2208.05631) for gfx950.
//
// Tile = 4096 coordinates = 256 code words per 256-thread work-group; thread t owns code
// word t of the tile, i.e. 16 consecutive coordinates, for every worker.  A wave therefore
// reads 256 consecutive bytes of each worker's code stream per load instruction.
// Per coordinate the kernel forms  acc = sum_m s_m * c_m  in binary64 (each product is exact),
// gbar = (float)(acc / M), optionally re-quantizes gbar per bucket inside the tile, and applies
// the accumulator + closed-form update, touching x, G (and z) exactly once.
#include "qa_common.h"

namespace qa {

enum StepMode { kAggregate = 0, kQcmd = 1, kQrda = 2 };

struct StepArgs {
  const uint32_t* codes;
  const float* scales;
  int64_t code_stride, scale_stride;
  int64_t d, W;
  int M;
  int log2b;          // log2(bucket), or -1 for one scale per vector
  double inv_M;       // exact 1/M when M is a power of two, unused otherwise
  int M_pow2;
  float* x; float* G; float* z; float* gbar;
  float eta, lam_eta, delta, t_lam, thr_coef;
};

// 10 -> 00 so that the reserved pattern reads as zero; 01 and 11 are unchanged.
__device__ __forceinline__ uint32_t sanitize(uint32_t w) {
  const uint32_t lo = w & 0x55555555u;
  return lo | ((w & (lo << 1)));
}

__device__ __forceinline__ void load16(const float* __restrict__ p, int64_t i0, int64_t d,
                                       float out[16]) {
  if (i0 + 16 <= d) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(p + i0 + 4 * q);
      out[4 * q] = v.x; out[4 * q + 1] = v.y; out[4 * q + 2] = v.z; out[4 * q + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j) out[j] = (i0 + j < d) ? p[i0 + j] : 0.0f;
  }
}

__device__ __forceinline__ void store16(float* __restrict__ p, int64_t i0, int64_t d,
                                        const float v[16]) {
  if (i0 + 16 <= d) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<float4*>(p + i0 + 4 * q) =
          make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (i0 + j < d) p[i0 + j] = v[j];
  }
}

template <int MODE, bool TRACK_Z, bool REQUANT>
__global__ __launch_bounds__(kThreads) void step_kernel(StepArgs a) {
  __shared__ double lds_d[kWaves];
  __shared__ uint32_t lds_u[kWaves];
  const int t = threadIdx.x;
  const int64_t wi = (int64_t)blockIdx.x * kTileWords + t;   // code word of this thread
  const int64_t i0 = wi * 16;                                // its first coordinate
  const bool live = wi < a.W;
  const int64_t k = a.log2b >= 0 ? (i0 >> a.log2b) : 0;      // its bucket

  // ---- unpack + sum over workers (binary64; every product s*c is exact) ----
  double acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.0;
  if (live) {
    const uint32_t* cw = a.codes + wi;
    const float* sc = a.scales + k;
    for (int m = 0; m < a.M; ++m) {
      const uint32_t w = sanitize(cw[(int64_t)m * a.code_stride]);
      const double s = (double)sc[(int64_t)m * a.scale_stride];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int c = ((int)(w << (30 - 2 * j))) >> 30;      // sign-extended 2-bit field
        acc[j] = fma((double)c, s, acc[j]);
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

  if (i0 + 16 > a.d) {                                       // last word: ignore tail bits
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (i0 + j >= a.d) q[j] = 0.0f;
  }

  // ---- second quantization inside the tile (bucket <= 4096) ----
  if (REQUANT) {
    const int b = 1 << a.log2b;
    const int seg = b / 16;                                  // threads per bucket: 4..256
    double s1 = 0.0;
#pragma unroll
    for (int j = 0; j < 16; ++j) s1 += (double)fabsf(q[j]);  // dead lanes hold zeros
    s1 = segment_sum(s1, seg, lds_d);
    const int64_t lo = k << a.log2b;
    const int64_t n = (a.d - lo) < (int64_t)b ? (a.d - lo) : (int64_t)b;
    const float Delta = n > 0 ? threshold_from_sum(s1, a.thr_coef, n) : 0.0f;
    double s2 = 0.0;
    uint32_t cnt = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float av = fabsf(q[j]);
      if (av > Delta) { s2 += (double)av; ++cnt; }
    }
    s2 = segment_sum(s2, seg, lds_d);
    cnt = segment_sum_u32(cnt, seg, lds_u);
    const float s = scale_from_sum(s2, cnt);
#pragma unroll
    for (int j = 0; j < 16; ++j) q[j] = q[j] > Delta ? s : (q[j] < -Delta ? -s : 0.0f);
  }

  if (!live) return;

  if (MODE == kAggregate) {
    store16(a.gbar, i0, a.d, q);
    return;
  }

  // ---- accumulator and closed-form update (binary32, one rounding per operation) ----
  float G[16], x[16], z[16];
  load16(a.G, i0, a.d, G);
  if (MODE == kQcmd) load16(a.x, i0, a.d, x);
  if (MODE == kQrda || TRACK_Z) load16(a.z, i0, a.d, z);
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const float q2 = q[j] * q[j];
    G[j] = G[j] + q2;
    const float H = a.delta + sqrtf(G[j]);
    if (MODE == kQcmd) {
      const float step = (a.eta * q[j]) / H;
      const float u = x[j] - step;
      const float tau = a.lam_eta / H;
      const float r = fabsf(u) - tau;
      x[j] = r > 0.0f ? copysignf(r, u) : 0.0f;
      if (TRACK_Z) z[j] = z[j] + q[j];
    } else {
      z[j] = z[j] + q[j];
      const float r = fabsf(z[j]) - a.t_lam;
      const float mag = (a.eta * r) / H;
      x[j] = r > 0.0f ? -copysignf(mag, z[j]) : 0.0f;
    }
  }
  store16(a.G, i0, a.d, G);
  store16(a.x, i0, a.d, x);
  if (MODE == kQrda || TRACK_Z) store16(a.z, i0, a.d, z);
}

// ---- host side -------------------------------------------------------------------------------

static inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t quantize_workspace_bytes(const qa_layout* L);
int quantize_launch(const qa_layout* L, const float* g, int64_t g_stride, uint32_t* codes,
                    float* scales, float* thresholds, uint32_t flags, void* ws, size_t ws_bytes,
                    hipStream_t stream);

// Layout of the one-message vector that carries Q(SynQ) when it is formed in separate passes.
static qa_layout requant_layout(const qa_layout* L, int requant) {
  qa_layout R = *L;
  R.M = 1;
  R.bucket = requant == QA_REQUANT_GLOBAL ? 0 : L->bucket;
  R.code_stride = words_of(L->d);
  R.scale_stride = buckets_of(L->d, R.bucket);
  return R;
}

static bool requant_in_tile(const qa_layout* L, int requant) {
  return requant == QA_REQUANT_BUCKET && L->bucket != 0 && L->bucket <= kTile;
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

static StepArgs make_args(const qa_layout* L, const uint32_t* codes, const float* scales) {
  StepArgs a{};
  a.codes = codes; a.scales = scales;
  a.code_stride = L->code_stride; a.scale_stride = L->scale_stride;
  a.d = L->d; a.W = words_of(L->d); a.M = L->M;
  a.log2b = L->bucket ? ilog2(L->bucket) : -1;
  a.M_pow2 = is_pow2(L->M) ? 1 : 0;
  a.inv_M = 1.0 / (double)L->M;
  a.thr_coef = L->thr_coef;
  return a;
}

template <int MODE>
static void launch_mode(const StepArgs& a, bool track_z, bool requant, hipStream_t stream) {
  const dim3 grid((unsigned)tiles_of(a.d)), block(kThreads);
  if (requant) {
    if (track_z) hipLaunchKernelGGL((step_kernel<MODE, true, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((step_kernel<MODE, false, true>), grid, block, 0, stream, a);
  } else {
    if (track_z) hipLaunchKernelGGL((step_kernel<MODE, true, false>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((step_kernel<MODE, false, false>), grid, block, 0, stream, a);
  }
}

static int step_common(int mode, const qa_layout* L, const uint32_t* codes, const float* scales,
                       float* x, float* G, float* z, bool track_z, int64_t t, float eta,
                       float lambda, float delta, int requant, void* ws, size_t ws_bytes,
                       hipStream_t stream) {
  int rc = check_layout(L);
  if (rc != QA_OK) return rc;
  if (!codes || !scales || !x || !G) return QA_ERR_INVALID_ARG;
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

  qa_layout R;
  const qa_layout* use = L;
  const uint32_t* use_codes = codes;
  const float* use_scales = scales;
  bool fused_requant = false;
  if (requant != QA_REQUANT_NONE) {
    if (requant_in_tile(L, requant)) {
      fused_requant = true;
    } else {
      // separate passes: gbar -> workspace, quantize it as a one-worker message, then run the
      // update on that message (its decoded value s*c is q exactly)
      R = requant_layout(L, requant);
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
      launch_mode<kAggregate>(ag, false, false, stream);
      const int64_t gs = (L->d + 3) & ~int64_t(3);
      rc = quantize_launch(&R, gbar, gs, c1, s1, th1, 0, qws ? p : nullptr, qws, stream);
      if (rc != QA_OK) return rc;
      use = &R; use_codes = c1; use_scales = s1;
    }
  }

  StepArgs a = make_args(use, use_codes, use_scales);
  a.x = x; a.G = G; a.z = z;
  a.eta = eta; a.lam_eta = lambda * eta; a.delta = delta;
  a.t_lam = (float)t * lambda;
  if (mode == kQcmd) launch_mode<kQcmd>(a, track_z, fused_requant, stream);
  else launch_mode<kQrda>(a, false, fused_requant, stream);
  return launch_status();
}

}  // namespace qa

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

// qa_oracle.cpp -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, single-threaded CPU statement of what one step of QCMD adagrad /
// QRDA adagrad (arXiv 2208.05631) computes on the data-parallel path:
//   local logistic gradient -> threshold quantizer -> 2-bit pack -> unpack + average
//   -> (optional second quantization) -> diagonal AdaGrad accumulator -> QCMD or QRDA update.
// It exists so that the GPU library can be compared with something written straight
// from the paper.  It shares no code with the GPU library and nothing outside tests/,
// the smoke check and the benchmark's cpu_baseline leg may call it.
//
// Arithmetic contract (the paper gives real-number formulas, not arithmetic):
//   * state (x, G, z), gradients, scales, thresholds are IEEE binary32;
//   * every element-wise formula is evaluated one correctly rounded binary32
//     operation at a time, in the order written here, with no fused multiply-add
//     (build with -ffp-contract=off);
//   * every sum over many terms (over a row, a minibatch, a bucket, the workers) is
//     accumulated in binary64 over exactly representable terms, in index order, and
//     the expression that uses it is rounded once to binary32.
//
// Pin status: every function here is pinned by tests/test_oracle_*.py against hand-worked
// values, closed forms, brute-force minimisation, a library optimiser or Monte Carlo,
// except the paper's undefined "Error" column (Table 3), which is not computed at all.
//
// Build: g++ -std=c++17 -O2 -ffp-contract=off -fPIC -shared qa_oracle.cpp -o liboracle.so

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// ---------------------------------------------------------------------------------
// Threshold quantizer, Section 3.4 ("Threshold Quantization") and Section 3.5
// ("Threshold Approximation").
// ---------------------------------------------------------------------------------

// Threshold of Section 3.5: Delta = (thr_coef / n) * sum_i |v_i|, thr_coef = 0.75 in the paper.
// n is the number of elements handed to the quantizer, zeros included.
float approx_threshold(const float* v, int64_t n, float thr_coef) {
  double S1 = 0.0;
  for (int64_t i = 0; i < n; ++i) S1 += (double)std::fabs(v[i]);
  return (float)(((double)thr_coef * S1) / (double)n);
}

// Optimal scale for a given threshold (the equation for s*_Delta in Section 3.4):
// the mean of |v_i| over I_Delta = { i : |v_i| > Delta }.  An empty I_Delta (only
// possible for an all-zero or NaN-poisoned vector) gives s = 0.
float optimal_scale(const float* v, int64_t n, float Delta, int64_t* cnt_out) {
  double S2 = 0.0;
  int64_t cnt = 0;
  for (int64_t i = 0; i < n; ++i) {
    float a = std::fabs(v[i]);
    if (a > Delta) { S2 += (double)a; ++cnt; }
  }
  if (cnt_out) *cnt_out = cnt;
  return cnt ? (float)(S2 / (double)cnt) : 0.0f;
}

// Ternary code of one component (the piecewise definition of v_i in Section 3.4).
// Comparisons are strict, so |v_i| == Delta gives 0.
inline int8_t ternary(float v, float Delta) {
  if (v > Delta) return 1;
  if (v < -Delta) return -1;
  return 0;
}

// Length of bucket k when a vector of length d is cut into contiguous pieces of
// `bucket` elements (bucket == 0: the whole vector is one piece, as in the paper's
// "one floating-point number" per message in the Encode paragraph).
inline int64_t bucket_len(int64_t d, int64_t bucket) { return bucket > 0 ? bucket : d; }
inline int64_t n_buckets(int64_t d, int64_t bucket) {
  int64_t b = bucket_len(d, bucket);
  return (d + b - 1) / b;
}

// Quantize one vector piece by piece: thresholds, scales and ternary codes.
void quantize_vector(const float* v, int64_t d, int64_t bucket, float thr_coef,
                     int8_t* code, float* scale, float* thresh, const float* thresh_in) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  for (int64_t k = 0; k < nb; ++k) {
    const int64_t lo = k * b, n = std::min(b, d - lo);
    const float Delta = thresh_in ? thresh_in[k] : approx_threshold(v + lo, n, thr_coef);
    const float s = optimal_scale(v + lo, n, Delta, nullptr);
    for (int64_t i = 0; i < n; ++i) code[lo + i] = ternary(v[lo + i], Delta);
    scale[k] = s;
    if (thresh) thresh[k] = Delta;
  }
}

// ---------------------------------------------------------------------------------
// Encoding ("Encode" paragraph of Section 3.5): 2 bits per component plus one float
// scale.  Bit patterns (the paper fixes only the width): 00 = 0, 01 = +1, 11 = -1,
// i.e. the 2-bit two's-complement value; 10 is never written and reads as 0.
// Component i sits in bits [2*(i mod 16), 2*(i mod 16)+1] of 32-bit word i/16.
// ---------------------------------------------------------------------------------
void pack_codes(const int8_t* code, int64_t d, uint32_t* words) {
  const int64_t W = (d + 15) / 16;
  for (int64_t w = 0; w < W; ++w) words[w] = 0u;
  for (int64_t i = 0; i < d; ++i) {
    uint32_t f = code[i] == 1 ? 1u : (code[i] == -1 ? 3u : 0u);
    words[i / 16] |= f << (2 * (i % 16));
  }
}

inline int decode_field(uint32_t word, int pos) {
  uint32_t f = (word >> (2 * pos)) & 3u;
  return f == 1u ? 1 : (f == 3u ? -1 : 0);
}

// ---------------------------------------------------------------------------------
// Server side: SynQ_t = (1/M) sum_m Q(g^(m))  (the equation labelled SynQ_t, and the
// "Average the quantized gradients" line of Algorithm 1).
// ---------------------------------------------------------------------------------
float averaged_component(const uint32_t* codes, int64_t code_stride, const float* scales,
                         int64_t scale_stride, int M, int64_t bucket_b, int64_t i) {
  double acc = 0.0;
  const int64_t k = i / bucket_b;
  for (int m = 0; m < M; ++m) {
    int c = decode_field(codes[(int64_t)m * code_stride + i / 16], (int)(i % 16));
    acc += (double)scales[(int64_t)m * scale_stride + k] * (double)c;
  }
  return (float)(acc / (double)M);
}

// ---------------------------------------------------------------------------------
// Worker side: H_t = delta*I + diag(||q_{1:t,i}||_2)  (the equation labelled Hq), kept
// as the running sum of squares G, then the closed-form updates.
// ---------------------------------------------------------------------------------
inline float accumulate_H(float* G, float q, float delta) {
  const float g2 = q * q;
  *G = *G + g2;
  return delta + std::sqrt(*G);
}

// QCMD update (the equation labelled QCMD): soft threshold of x - eta*q/H by lambda*eta/H.
inline float qcmd_component(float x, float q, float H, float eta, float lambda) {
  const float step = (eta * q) / H;
  const float u = x - step;
  const float tau = (lambda * eta) / H;
  const float r = std::fabs(u) - tau;
  return r > 0.0f ? std::copysign(r, u) : 0.0f;
}

// QRDA update (the equation labelled QRDA) with z = sum_{tau<=t} q_tau:
//   x = sign(-z) * (t*eta/H) * [ |z/t| - lambda ]_+  =  -sign(z) * eta * [ |z| - t*lambda ]_+ / H,
// the second form being the first multiplied through by t (one rounding fewer).
inline float qrda_component(float z, float H, int64_t t, float eta, float lambda) {
  const float tl = (float)t * lambda;
  const float r = std::fabs(z) - tl;
  if (!(r > 0.0f)) return 0.0f;
  const float mag = (eta * r) / H;
  return -std::copysign(mag, z);
}

}  // namespace

extern "C" {

// ---- quantizer ------------------------------------------------------------------

// Delta and s of one piece of n elements (Sections 3.4-3.5).  cnt_out = |I_Delta|.
void orc_threshold_scale(const float* v, int64_t n, float thr_coef, float* Delta_out,
                         float* s_out, int64_t* cnt_out) {
  const float Delta = approx_threshold(v, n, thr_coef);
  *Delta_out = Delta;
  *s_out = optimal_scale(v, n, Delta, cnt_out);
}

// Scale and count for a caller-chosen threshold.
void orc_scale_for_threshold(const float* v, int64_t n, float Delta, float* s_out,
                             int64_t* cnt_out) {
  *s_out = optimal_scale(v, n, Delta, cnt_out);
}

// Ternary codes (int8 in {-1,0,1}), scales and thresholds of one vector.
// thresh_in may be NULL (thresholds computed by the Section 3.5 rule) or hold one
// threshold per bucket to use instead.  thresh_out may be NULL.
void orc_quantize(const float* v, int64_t d, int64_t bucket, float thr_coef, int8_t* code_out,
                  float* scale_out, float* thresh_out, const float* thresh_in) {
  quantize_vector(v, d, bucket, thr_coef, code_out, scale_out, thresh_out, thresh_in);
}

// Exact optimal threshold of Section 3.4 by ranking: every component magnitude is tried
// as "keep everything at least this large"; the kept set of size k maximises
// (sum of the k largest |v|)^2 / k.  Returns the smallest kept magnitude (kept set is
// {|v_i| >= that}), the matching scale and the objective value.
void orc_exact_threshold(const float* v, int64_t n, double* kept_min_out, double* s_out,
                         double* objective_out, int64_t* kept_out) {
  std::vector<double> a(n);
  for (int64_t i = 0; i < n; ++i) a[i] = std::fabs((double)v[i]);
  std::sort(a.begin(), a.end(), [](double p, double q) { return p > q; });
  double best = -1.0, best_s = 0.0, best_min = 0.0, run = 0.0;
  int64_t best_k = 0;
  for (int64_t k = 1; k <= n; ++k) {
    run += a[k - 1];
    if (k < n && a[k] == a[k - 1]) continue;  // a threshold cannot split equal magnitudes
    if (a[k - 1] == 0.0) break;
    double obj = run * run / (double)k;
    if (obj > best) { best = obj; best_s = run / (double)k; best_min = a[k - 1]; best_k = k; }
  }
  *kept_min_out = best_min; *s_out = best_s; *objective_out = best < 0 ? 0.0 : best;
  *kept_out = best_k;
}

// The optimal threshold as a number to compare with strictly: per bucket, the largest magnitude
// that is NOT kept by the optimum above (the (k*+1)-th largest; 0 if everything non-zero is
// kept or the bucket is all zero), so that {|v_i| > Delta} is exactly the optimal kept set.
void orc_exact_thresholds(const float* v, int64_t d, int64_t bucket, float* thresh_out) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  for (int64_t k = 0; k < nb; ++k) {
    const int64_t lo = k * b, n = std::min(b, d - lo);
    double kept_min, s, obj;
    int64_t kept;
    orc_exact_threshold(v + lo, n, &kept_min, &s, &obj, &kept);
    float Delta = 0.0f;
    for (int64_t i = 0; i < n; ++i) {           // largest magnitude below the kept ones
      const float a = std::fabs(v[lo + i]);
      if ((double)a < kept_min && a > Delta) Delta = a;
    }
    thresh_out[k] = Delta;
  }
}

// ---- encoding -------------------------------------------------------------------

void orc_pack(const int8_t* code, int64_t d, uint32_t* words) { pack_codes(code, d, words); }

void orc_unpack(const uint32_t* words, int64_t d, int8_t* code_out) {
  for (int64_t i = 0; i < d; ++i) code_out[i] = (int8_t)decode_field(words[i / 16], (int)(i % 16));
}

// Quantize and pack M gradients g[m*g_stride + i] (worker side of Algorithm 1).
void orc_quantize_pack(const float* g, int64_t g_stride, int64_t d, int M, int64_t bucket,
                       float thr_coef, uint32_t* codes, int64_t code_stride, float* scales,
                       float* thresholds, int64_t scale_stride, int thresholds_given) {
  std::vector<int8_t> code(d);
  const int64_t nb = n_buckets(d, bucket);
  std::vector<float> th(nb);
  for (int m = 0; m < M; ++m) {
    const float* tin = thresholds_given ? thresholds + (int64_t)m * scale_stride : nullptr;
    quantize_vector(g + (int64_t)m * g_stride, d, bucket, thr_coef, code.data(),
                    scales + (int64_t)m * scale_stride, th.data(), tin);
    if (thresholds && !thresholds_given)
      std::memcpy(thresholds + (int64_t)m * scale_stride, th.data(), nb * sizeof(float));
    pack_codes(code.data(), d, codes + (int64_t)m * code_stride);
  }
}

// ---- server ---------------------------------------------------------------------

// gbar_i = (1/M) sum_m s_{m,bucket(i)} * c_{m,i}
void orc_aggregate(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float* gbar_out) {
  const int64_t b = bucket_len(d, bucket);
  for (int64_t i = 0; i < d; ++i)
    gbar_out[i] = averaged_component(codes, code_stride, scales, scale_stride, M, b, i);
}

// Second quantization q_t = Q(SynQ_t) (the equation labelled Qt; Algorithm 1, server):
// the same quantizer applied to the averaged vector, decoded again: q_i = s * code_i.
void orc_requantize(const float* gbar, int64_t d, int64_t bucket, float thr_coef, float* q_out) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  std::vector<int8_t> code(d);
  std::vector<float> sc(nb);
  quantize_vector(gbar, d, bucket, thr_coef, code.data(), sc.data(), nullptr, nullptr);
  for (int64_t i = 0; i < d; ++i) q_out[i] = sc[i / b] * (float)code[i];
}

// ---- worker updates from a given q_t ---------------------------------------------

// G += q^2 ; H = delta + sqrt(G) ; QCMD update of x.  If z != NULL also z += q.
void orc_update_qcmd(const float* q, int64_t d, float* x, float* G, float* z, float eta,
                     float lambda, float delta) {
  for (int64_t i = 0; i < d; ++i) {
    const float H = accumulate_H(&G[i], q[i], delta);
    x[i] = qcmd_component(x[i], q[i], H, eta, lambda);
    if (z) z[i] = z[i] + q[i];
  }
}

// G += q^2 ; H = delta + sqrt(G) ; z += q ; QRDA update of x (x is overwritten).
void orc_update_qrda(const float* q, int64_t d, float* x, float* G, float* z, int64_t t,
                     float eta, float lambda, float delta) {
  for (int64_t i = 0; i < d; ++i) {
    const float H = accumulate_H(&G[i], q[i], delta);
    z[i] = z[i] + q[i];
    x[i] = qrda_component(z[i], H, t, eta, lambda);
  }
}

// QRDA exactly as printed: sign(-z) * (t*eta/H) * [ |z/t| - lambda ]_+ , in binary64.
void orc_qrda_literal_f64(const double* z, const double* H, int64_t d, int64_t t, double eta,
                          double lambda, double* x_out) {
  for (int64_t i = 0; i < d; ++i) {
    double r = std::fabs(z[i] / (double)t) - lambda;
    double sgn = z[i] > 0 ? -1.0 : (z[i] < 0 ? 1.0 : 0.0);
    x_out[i] = r > 0 ? sgn * ((double)t * eta / H[i]) * r : 0.0;
  }
}

// ---- whole server+worker step from packed codes ------------------------------------

// requant: 0 = q is the average itself (the paper's dagger variants), 1 = second
// quantization per bucket of the same length as the first, 2 = second quantization
// with one threshold/scale for the whole vector (the paper's single float per message).
static void form_q(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float thr_coef,
                   int requant, std::vector<float>& q) {
  q.resize(d);
  orc_aggregate(codes, code_stride, scales, scale_stride, d, M, bucket, q.data());
  if (requant == 1 || requant == 2) {
    std::vector<float> gbar(q);
    orc_requantize(gbar.data(), d, requant == 1 ? bucket : 0, thr_coef, q.data());
  }
}

void orc_step_qcmd(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float thr_coef,
                   float* x, float* G, float* z_or_null, float eta, float lambda, float delta,
                   int requant) {
  std::vector<float> q;
  form_q(codes, code_stride, scales, scale_stride, d, M, bucket, thr_coef, requant, q);
  orc_update_qcmd(q.data(), d, x, G, z_or_null, eta, lambda, delta);
}

void orc_step_qrda(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float thr_coef,
                   float* x, float* G, float* z, int64_t t, float eta, float lambda, float delta,
                   int requant) {
  std::vector<float> q;
  form_q(codes, code_stride, scales, scale_stride, d, M, bucket, thr_coef, requant, q);
  orc_update_qrda(q.data(), d, x, G, z, t, eta, lambda, delta);
}

// ---- a list of parameter tensors in one flat vector (models such as the CNNs of Section 5,
//      whose parameters are many tensors of very different sizes) --------------------------------
//
// Reading: the quantizer is applied to each tensor's gradient on its own (own threshold, own
// scale), exactly as to a vector of that length.  Tensor s occupies coordinates
// [begin[s], begin[s] + length[s]) of the flat vector; begin[s] is a multiple of 16 so that no
// code word is shared; coordinates between tensors belong to no tensor: their code fields are 0
// and the step leaves their state alone.  scales[m*scale_stride + s] is worker m's scale of
// tensor s.  Every function below is the single-vector function applied slice by slice.
void orc_quantize_pack_segments(const float* g, int64_t g_stride, int64_t d, int M, int64_t n_seg,
                                const int64_t* begin, const int64_t* length, float thr_coef,
                                uint32_t* codes, int64_t code_stride, float* scales,
                                float* thresholds, int64_t scale_stride) {
  (void)d;
  for (int m = 0; m < M; ++m)
    for (int64_t s = 0; s < n_seg; ++s) {
      float* sc = scales + (int64_t)m * scale_stride + s;
      float* th = thresholds ? thresholds + (int64_t)m * scale_stride + s : nullptr;
      if (length[s] == 0) { *sc = 0.0f; if (th) *th = 0.0f; continue; }
      orc_quantize_pack(g + (int64_t)m * g_stride + begin[s], 0, length[s], 1, 0, thr_coef,
                        codes + (int64_t)m * code_stride + begin[s] / 16, 0, sc, th, 0, 0);
    }
}

// requant: 0 = none, otherwise the averaged gradient of each tensor is quantized again as a
// vector of that tensor's length.
void orc_step_segments(int method, const uint32_t* codes, int64_t code_stride, const float* scales,
                       int64_t scale_stride, int64_t d, int M, int64_t n_seg, const int64_t* begin,
                       const int64_t* length, float thr_coef, float* x, float* G, float* z_or_null,
                       int64_t t, float eta, float lambda, float delta, int requant) {
  (void)d;
  for (int64_t s = 0; s < n_seg; ++s) {
    if (length[s] == 0) continue;
    const int64_t b = begin[s];
    float* zs = z_or_null ? z_or_null + b : nullptr;
    if (method == 0)
      orc_step_qcmd(codes + b / 16, code_stride, scales + s, scale_stride, length[s], M, 0,
                    thr_coef, x + b, G + b, zs, eta, lambda, delta, requant ? 2 : 0);
    else
      orc_step_qrda(codes + b / 16, code_stride, scales + s, scale_stride, length[s], M, 0,
                    thr_coef, x + b, G + b, zs, t, eta, lambda, delta, requant ? 2 : 0);
  }
}

// ---- indicator, selection and sparse encoding (Section 3.2: equations "select" and "ind";
//      Algorithm 1, worker block; "Encode" paragraph: (32 + d + 2k) bits) ----------------------
//
// Worker m forms the parameter it WOULD get from its own full-precision gradient g,
//   H^ = delta + sqrt(G + g^2)   (c^ = ||[q_{1:t-1}, g]||_2, G being the sum of the q^2 so far),
//   x^ = the QCMD or QRDA update with g in place of q_t,
// and marks coordinate i iff x_i != 0 or x^_i != 0.  Only marked components are quantized
// (the quantizer sees the k marked components as a vector of length k) and sent together with
// the d-bit indicator.  method: 0 = QCMD, 1 = QRDA.  Indicator bit i = bit (i%32) of word i/32.
void orc_indicator(int method, const float* g, int64_t d, const float* x, const float* G,
                   const float* z, int64_t t, float eta, float lambda, float delta,
                   uint32_t* ind_out) {
  const int64_t nw = (d + 31) / 32;
  for (int64_t w = 0; w < nw; ++w) ind_out[w] = 0u;
  for (int64_t i = 0; i < d; ++i) {
    float Gh = G[i];
    const float Hh = accumulate_H(&Gh, g[i], delta);
    float xh;
    if (method == 0) {
      xh = qcmd_component(x[i], g[i], Hh, eta, lambda);
    } else {
      const float zh = z[i] + g[i];
      xh = qrda_component(zh, Hh, t, eta, lambda);
    }
    if (x[i] != 0.0f || xh != 0.0f) ind_out[i / 32] |= 1u << (i % 32);
  }
}

// Synchronous indicator: bitwise OR of the M indicators (Algorithm 1, server).
void orc_indicator_or(const uint32_t* ind, int64_t ind_stride, int M, int64_t d, uint32_t* out) {
  const int64_t nw = (d + 31) / 32;
  for (int64_t w = 0; w < nw; ++w) {
    uint32_t v = 0u;
    for (int m = 0; m < M; ++m) v |= ind[(int64_t)m * ind_stride + w];
    out[w] = v;
  }
}

// Q(S(g, I)) bucket by bucket: the marked components of bucket k, in index order, form a vector
// of length count[k]; it is quantized by the threshold quantizer (threshold uses count[k] as
// its length) and its codes are packed from bit 0 of word k*area_words of `sel_codes`
// (area_words = ceil(bucket_len/16)).  count[k] == 0: scale 0, threshold 0, nothing written.
void orc_quantize_selected(const float* g, const uint32_t* ind, int64_t d, int64_t bucket,
                           float thr_coef, uint32_t* sel_codes, uint32_t* count, float* scale,
                           float* thresh) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  const int64_t area = (b + 15) / 16;
  std::vector<float> sel;
  std::vector<int8_t> code;
  for (int64_t k = 0; k < nb; ++k) {
    const int64_t lo = k * b, hi = std::min(lo + b, d);
    sel.clear();
    for (int64_t i = lo; i < hi; ++i)
      if ((ind[i / 32] >> (i % 32)) & 1u) sel.push_back(g[i]);
    count[k] = (uint32_t)sel.size();
    scale[k] = 0.0f;
    if (thresh) thresh[k] = 0.0f;
    if (sel.empty()) continue;
    code.resize(sel.size());
    float s, D;
    quantize_vector(sel.data(), (int64_t)sel.size(), 0, thr_coef, code.data(), &s, &D, nullptr);
    scale[k] = s;
    if (thresh) thresh[k] = D;
    pack_codes(code.data(), (int64_t)sel.size(), sel_codes + k * area);
  }
}

// S applied to codes (Algorithm 1, server: "Push S(q_t, I^Syn) and I^Syn to every worker"): the
// 2-bit codes of the marked components of one dense message, in index order, packed per bucket
// exactly like the output of orc_quantize_selected; count[k] = marked components of bucket k.
void orc_select_codes(const uint32_t* dense_words, const uint32_t* ind, int64_t d, int64_t bucket,
                      uint32_t* sel_codes, uint32_t* count) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  const int64_t area = (b + 15) / 16;
  std::vector<int8_t> code;
  for (int64_t k = 0; k < nb; ++k) {
    const int64_t lo = k * b, hi = std::min(lo + b, d);
    code.clear();
    for (int64_t i = lo; i < hi; ++i)
      if ((ind[i / 32] >> (i % 32)) & 1u)
        code.push_back((int8_t)decode_field(dense_words[i / 16], (int)(i % 16)));
    count[k] = (uint32_t)code.size();
    if (!code.empty()) pack_codes(code.data(), (int64_t)code.size(), sel_codes + k * area);
  }
}

// S^{-1}: put the codes of the marked components back at their coordinates (unmarked -> 0) in
// the dense 2-bit layout of one worker.
void orc_decode_selected(const uint32_t* ind, const uint32_t* sel_codes, int64_t d, int64_t bucket,
                         uint32_t* dense_words) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  const int64_t area = (b + 15) / 16;
  std::vector<int8_t> code(d, 0);
  for (int64_t k = 0; k < nb; ++k) {
    const int64_t lo = k * b, hi = std::min(lo + b, d);
    int64_t j = 0;
    for (int64_t i = lo; i < hi; ++i)
      if ((ind[i / 32] >> (i % 32)) & 1u) {
        code[i] = (int8_t)decode_field(sel_codes[k * area + j / 16], (int)(j % 16));
        ++j;
      }
  }
  pack_codes(code.data(), d, dense_words);
}

// ---- stochastic ternary quantizer (the "ternary" baseline of Section 5.1: TernGrad, Wen et
//      al. 2017, which the paper cites and does not restate) with a counter-based generator ----
//
// Per bucket: s = max_i |v_i|;  component i is kept with probability |v_i| / s and then coded
// as sign(v_i), so that E[s * code_i] = v_i.  The uniform numbers come from Philox4x32-10
// (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11), keyed by
// the 64-bit seed, counter = (i/4 low, i/4 high, worker, step); component i takes output word
// i%4.  u = (r >> 8) * 2^-24 in [0,1); keep iff u < |v_i|/s with the division in binary32.
void orc_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
  uint32_t c[4] = {ctr_in[0], ctr_in[1], ctr_in[2], ctr_in[3]};
  uint32_t k0 = key_in[0], k1 = key_in[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
  }
  for (int j = 0; j < 4; ++j) out[j] = c[j];
}

// The uniform number of component i of worker m at step `step`.
float orc_uniform(uint64_t seed, uint32_t step, uint32_t m, int64_t i) {
  const uint64_t j = (uint64_t)i / 4;
  const uint32_t ctr[4] = {(uint32_t)j, (uint32_t)(j >> 32), m, step};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t r[4];
  orc_philox4x32_10(ctr, key, r);
  return (float)(r[i % 4] >> 8) * 0x1p-24f;
}

void orc_quantize_stochastic(const float* v, int64_t d, int64_t bucket, uint64_t seed, uint32_t step,
                             uint32_t m, int8_t* code_out, float* scale_out) {
  const int64_t b = bucket_len(d, bucket), nb = n_buckets(d, bucket);
  for (int64_t k = 0; k < nb; ++k) {
    const int64_t lo = k * b, hi = std::min(lo + b, d);
    float s = 0.0f;
    for (int64_t i = lo; i < hi; ++i) {
      const float a = std::fabs(v[i]);
      if (a > s) s = a;                        // NaN never wins
    }
    scale_out[k] = s;
    for (int64_t i = lo; i < hi; ++i) {
      const float p = std::fabs(v[i]) / s;     // 0/0 = NaN when the bucket is all zero: never kept
      const bool keep = orc_uniform(seed, step, m, i) < p;
      code_out[i] = keep ? (v[i] < 0.0f ? -1 : 1) : 0;
    }
  }
}

// ---- local gradient: L1-regularised logistic regression (Section 5.1) ----------------
//
// Loss of one sample (a, y), y in {-1,+1}:  log(1 + exp(-y * a.x)); the minibatch
// gradient is the mean over the batch (the stochastic-gradient equation of Section 3.1).
// Row i of the data is given either densely (A[row*d + j]) or in CSR form
// (indptr/indices/vals).  Batch rows may repeat.

static void logistic_from_margin(float p, float y, int B, float* coef_out, double* loss_out) {
  const double m = (double)y * (double)p;           // margin y * a.x
  const double e = std::exp(-std::fabs(m));
  *loss_out = std::log1p(e) + (m < 0 ? -m : 0.0);   // log(1 + exp(-m)), overflow-free
  const double sig = m >= 0 ? e / (1.0 + e) : 1.0 / (1.0 + e);   // 1 / (1 + exp(m))
  *coef_out = (float)((-(double)y * sig) / (double)B);
}

void orc_local_grad_dense(const float* A, int64_t n_rows, int64_t d, const float* y,
                          const int32_t* batch_rows, int B, const float* x, float* g_out,
                          float* loss_out) {
  (void)n_rows;
  std::vector<float> coef(B);
  double loss_sum = 0.0;
  for (int b = 0; b < B; ++b) {
    const float* a = A + (int64_t)batch_rows[b] * d;
    double dot = 0.0;
    for (int64_t j = 0; j < d; ++j) dot += (double)a[j] * (double)x[j];
    double l;
    logistic_from_margin((float)dot, y[batch_rows[b]], B, &coef[b], &l);
    loss_sum += l;
  }
  for (int64_t j = 0; j < d; ++j) {
    double acc = 0.0;
    for (int b = 0; b < B; ++b)
      acc += (double)coef[b] * (double)A[(int64_t)batch_rows[b] * d + j];
    g_out[j] = (float)acc;
  }
  if (loss_out) *loss_out = (float)(loss_sum / (double)B);
}

void orc_local_grad_csr(const float* vals, const int64_t* indptr, const int32_t* indices,
                        int64_t n_rows, int64_t d, const float* y, const int32_t* batch_rows,
                        int B, const float* x, float* g_out, float* loss_out) {
  (void)n_rows;
  std::vector<float> coef(B);
  std::vector<double> acc(d, 0.0);
  double loss_sum = 0.0;
  for (int b = 0; b < B; ++b) {
    const int64_t r = batch_rows[b];
    double dot = 0.0;
    for (int64_t k = indptr[r]; k < indptr[r + 1]; ++k)
      dot += (double)vals[k] * (double)x[indices[k]];
    double l;
    logistic_from_margin((float)dot, y[r], B, &coef[b], &l);
    loss_sum += l;
  }
  for (int b = 0; b < B; ++b) {
    const int64_t r = batch_rows[b];
    for (int64_t k = indptr[r]; k < indptr[r + 1]; ++k)
      acc[indices[k]] += (double)coef[b] * (double)vals[k];
  }
  for (int64_t j = 0; j < d; ++j) g_out[j] = (float)acc[j];
  if (loss_out) *loss_out = (float)(loss_sum / (double)B);
}

}  // extern "C"

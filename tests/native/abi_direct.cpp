// Calls libqadagrad through its C ABI from a plain C++ host program: no Python, no torch, device
// memory from hipMalloc.  One worker-side quantize+pack and T fused QCMD and QRDA steps are
// compared bit for bit with the CPU checker (oracle/liboracle.so), which this TEST links as well;
// then the materialised average, the entry point that allocates nothing, and a dense minibatch
// gradient.  Exit status 0 = all as expected.  Built by __graft_entry__.build(); run by
// tests/test_gpu_native.py.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "qadagrad.h"

extern "C" {
void orc_quantize_pack(const float* g, int64_t g_stride, int64_t d, int M, int64_t bucket,
                       float thr_coef, uint32_t* codes, int64_t code_stride, float* scales,
                       float* thresholds, int64_t scale_stride, int thresholds_given);
void orc_step_qcmd(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float thr_coef, float* x,
                   float* G, float* z_or_null, float eta, float lambda, float delta, int requant);
void orc_step_qrda(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float thr_coef, float* x,
                   float* G, float* z, int64_t t, float eta, float lambda, float delta, int requant);
void orc_aggregate(const uint32_t* codes, int64_t code_stride, const float* scales,
                   int64_t scale_stride, int64_t d, int M, int64_t bucket, float* gbar_out);
void orc_local_grad_dense(const float* A, int64_t n_rows, int64_t d, const float* y,
                          const int32_t* batch_rows, int B, const float* x, float* g_out,
                          float* loss_out);
}

#define HIP_OK(call)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) {                                                            \
      std::fprintf(stderr, "%s:%d %s\n", __FILE__, __LINE__, hipGetErrorString(e_));   \
      return 2;                                                                        \
    }                                                                                  \
  } while (0)
#define QA_CALL(call)                                                                  \
  do {                                                                                 \
    int rc_ = (call);                                                                  \
    if (rc_ != QA_OK) {                                                                \
      std::fprintf(stderr, "%s:%d %s\n", __FILE__, __LINE__, qa_strerror(rc_));        \
      return 3;                                                                        \
    }                                                                                  \
  } while (0)

// seeded, synthetic: a sparse heavy-tailed gradient from a 64-bit LCG
static void fill_gradient(std::vector<float>& g, uint64_t seed) {
  uint64_t s = seed * 0x9E3779B97F4A7C15ull + 1;
  for (auto& v : g) {
    s = s * 6364136223846793005ull + 1442695040888963407ull;
    const uint32_t r = (uint32_t)(s >> 33);
    const float u = (float)(r & 0xFFFF) / 65536.0f - 0.5f;
    v = (r >> 16) % 10 < 3 ? u * u * u * 0.08f : 0.0f;
  }
}

template <typename T>
static bool same(const std::vector<T>& a, const std::vector<T>& b, const char* what) {
  if (a.size() == b.size() && std::memcmp(a.data(), b.data(), a.size() * sizeof(T)) == 0) return true;
  std::fprintf(stderr, "MISMATCH in %s\n", what);
  return false;
}

int main() {
  const int64_t d = 70001;
  const int M = 8, bucket = 4096, T = 4;
  const float eta = 0.1f, lambda = 2e-4f, delta = 1e-8f;
  qa_layout L;
  L.d = d; L.M = M; L.bucket = bucket; L.thr_coef = 0.75f;
  L.code_stride = (d + 15) / 16 + 5;                       // padded rows on purpose
  L.scale_stride = (d + bucket - 1) / bucket + 3;
  const int64_t gs = (d + 3) / 4 * 4;

  float *dg, *dx, *dG, *dz, *dscales;
  uint32_t* dcodes;
  HIP_OK(hipMalloc(&dg, sizeof(float) * M * gs));
  HIP_OK(hipMalloc(&dcodes, sizeof(uint32_t) * M * L.code_stride));
  HIP_OK(hipMalloc(&dscales, sizeof(float) * M * L.scale_stride));
  HIP_OK(hipMalloc(&dx, sizeof(float) * d));
  HIP_OK(hipMalloc(&dG, sizeof(float) * d));
  HIP_OK(hipMalloc(&dz, sizeof(float) * d));
  HIP_OK(hipMemset(dx, 0, sizeof(float) * d));
  HIP_OK(hipMemset(dG, 0, sizeof(float) * d));
  HIP_OK(hipMemset(dz, 0, sizeof(float) * d));
  HIP_OK(hipMemset(dcodes, 0, sizeof(uint32_t) * M * L.code_stride));
  HIP_OK(hipMemset(dscales, 0, sizeof(float) * M * L.scale_stride));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  if (qa_version() != QA_VERSION) { std::fprintf(stderr, "version\n"); return 4; }
  if (qa_workspace_bytes(&L, QA_OP_QUANTIZE) != 0) { std::fprintf(stderr, "workspace\n"); return 4; }

  std::vector<float> g((size_t)M * gs), ox(d, 0.f), oG(d, 0.f), oz(d, 0.f);
  std::vector<uint32_t> oc((size_t)M * L.code_stride, 0u), hc(oc.size());
  std::vector<float> os((size_t)M * L.scale_stride, 0.f), hs(os.size()), hx(d), hG(d), hz(d);
  bool ok = true;
  for (int t = 1; t <= T && ok; ++t) {
    fill_gradient(g, (uint64_t)t);
    HIP_OK(hipMemcpyAsync(dg, g.data(), sizeof(float) * g.size(), hipMemcpyHostToDevice, stream));
    QA_CALL(qa_quantize_pack(&L, dg, gs, dcodes, dscales, nullptr, 0, nullptr, 0, stream));
    if (t % 2)
      QA_CALL(qa_step_qcmd(&L, dcodes, dscales, dx, dG, dz, eta, lambda, delta, QA_REQUANT_BUCKET,
                           nullptr, 0, stream));
    else
      QA_CALL(qa_step_qrda(&L, dcodes, dscales, dx, dG, dz, t, eta, lambda, delta, QA_REQUANT_NONE,
                           nullptr, 0, stream));
    HIP_OK(hipMemcpyAsync(hc.data(), dcodes, sizeof(uint32_t) * hc.size(), hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(hs.data(), dscales, sizeof(float) * hs.size(), hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(hx.data(), dx, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(hG.data(), dG, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(hz.data(), dz, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));

    orc_quantize_pack(g.data(), gs, d, M, bucket, 0.75f, oc.data(), L.code_stride, os.data(), nullptr,
                      L.scale_stride, 0);
    if (t % 2)
      orc_step_qcmd(oc.data(), L.code_stride, os.data(), L.scale_stride, d, M, bucket, 0.75f, ox.data(),
                    oG.data(), oz.data(), eta, lambda, delta, 1);
    else
      orc_step_qrda(oc.data(), L.code_stride, os.data(), L.scale_stride, d, M, bucket, 0.75f, ox.data(),
                    oG.data(), oz.data(), t, eta, lambda, delta, 0);
    // rows are padded: compare what the layout defines
    for (int m = 0; m < M && ok; ++m) {
      const size_t W = (size_t)((d + 15) / 16), nb = (size_t)((d + bucket - 1) / bucket);
      ok = ok && std::memcmp(&hc[m * L.code_stride], &oc[m * L.code_stride], W * 4) == 0 &&
           std::memcmp(&hs[m * L.scale_stride], &os[m * L.scale_stride], nb * 4) == 0;
      if (!ok) std::fprintf(stderr, "MISMATCH in codes/scales of worker %d, step %d\n", m, t);
    }
    ok = ok && same(hx, ox, "x") && same(hG, oG, "G") && same(hz, oz, "z");
    size_t nz = 0;
    for (float v : hx) nz += v != 0.0f;
    std::printf("step %d: %s, %zu non-zero parameters\n", t, ok ? "identical" : "DIFFERENT", nz);
  }
  // the average as fp32 (the codes and scales of the last step are still on both sides)
  {
    std::vector<float> hq(d), oq(d);
    float* dq;
    HIP_OK(hipMalloc(&dq, sizeof(float) * d));
    QA_CALL(qa_aggregate_unpack(&L, dcodes, dscales, dq, stream));
    HIP_OK(hipMemcpyAsync(hq.data(), dq, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    orc_aggregate(oc.data(), L.code_stride, os.data(), L.scale_stride, d, M, bucket, oq.data());
    ok = ok && same(hq, oq, "the average");
    std::printf("qa_aggregate_unpack: %s\n", ok ? "identical" : "DIFFERENT");
    (void)hipFree(dq);
  }
  // one scale per vector: the multi-pass quantizer with a workspace, and the entry point that
  // keeps its partial sums in the library's own array, must write the same message
  {
    qa_layout L0 = L;
    L0.bucket = 0; L0.scale_stride = 1;
    const size_t wsb = qa_workspace_bytes(&L0, QA_OP_QUANTIZE);
    void* dws;
    uint32_t* dc2;
    float *ds1, *ds2;
    HIP_OK(hipMalloc(&dws, wsb));
    HIP_OK(hipMalloc(&dc2, sizeof(uint32_t) * M * L.code_stride));
    HIP_OK(hipMalloc(&ds1, sizeof(float) * M));
    HIP_OK(hipMalloc(&ds2, sizeof(float) * M));
    QA_CALL(qa_quantize_pack(&L0, dg, gs, dcodes, ds1, nullptr, 0, dws, wsb, stream));
    QA_CALL(qa_quantize_pack_static(&L0, dg, gs, dc2, ds2, nullptr, 0, stream));
    std::vector<uint32_t> c1(hc.size()), c2(hc.size());
    std::vector<float> s1(M), s2(M), os0(M);
    HIP_OK(hipMemcpyAsync(c1.data(), dcodes, sizeof(uint32_t) * c1.size(), hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(c2.data(), dc2, sizeof(uint32_t) * c2.size(), hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(s1.data(), ds1, sizeof(float) * M, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(s2.data(), ds2, sizeof(float) * M, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    orc_quantize_pack(g.data(), gs, d, M, 0, 0.75f, oc.data(), L.code_stride, os0.data(), nullptr, 1, 0);
    bool q_ok = same(s1, s2, "scales of the two quantizer entry points") && same(s1, os0, "scales, one per vector");
    const size_t W = (size_t)((d + 15) / 16);
    for (int m = 0; m < M && q_ok; ++m)
      q_ok = std::memcmp(&c1[m * L.code_stride], &c2[m * L.code_stride], W * 4) == 0 &&
             std::memcmp(&c1[m * L.code_stride], &oc[m * L.code_stride], W * 4) == 0;
    std::printf("qa_quantize_pack_static: %s\n", q_ok ? "identical" : "DIFFERENT");
    ok = ok && q_ok;
    (void)hipFree(dws); (void)hipFree(dc2); (void)hipFree(ds1); (void)hipFree(ds2);
  }
  // one scale per message and one scale for Q(SynQ): the second quantization spans the whole
  // vector, so the steps run it in separate passes over the caller's workspace
  {
    qa_layout L0 = L;
    L0.bucket = 0; L0.scale_stride = 1;
    const size_t qwsb = qa_workspace_bytes(&L0, QA_OP_QUANTIZE), wsb = qa_workspace_bytes(&L0, QA_OP_STEP);
    void *dqws, *dws;
    float* ds0;
    HIP_OK(hipMalloc(&dqws, qwsb));
    HIP_OK(hipMalloc(&dws, wsb));
    HIP_OK(hipMalloc(&ds0, sizeof(float) * M));
    QA_CALL(qa_quantize_pack(&L0, dg, gs, dcodes, ds0, nullptr, 0, dqws, qwsb, stream));
    QA_CALL(qa_step_qcmd(&L0, dcodes, ds0, dx, dG, dz, eta, lambda, delta, QA_REQUANT_GLOBAL, dws, wsb, stream));
    QA_CALL(qa_step_qrda(&L0, dcodes, ds0, dx, dG, dz, T + 2, eta, lambda, delta, QA_REQUANT_GLOBAL, dws, wsb,
                         stream));
    HIP_OK(hipMemcpyAsync(hx.data(), dx, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(hG.data(), dG, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(hz.data(), dz, sizeof(float) * d, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    std::vector<float> os0(M);
    orc_quantize_pack(g.data(), gs, d, M, 0, 0.75f, oc.data(), L.code_stride, os0.data(), nullptr, 1, 0);
    orc_step_qcmd(oc.data(), L.code_stride, os0.data(), 1, d, M, 0, 0.75f, ox.data(), oG.data(), oz.data(), eta,
                  lambda, delta, 2);
    orc_step_qrda(oc.data(), L.code_stride, os0.data(), 1, d, M, 0, 0.75f, ox.data(), oG.data(), oz.data(), T + 2,
                  eta, lambda, delta, 2);
    const bool g_ok = same(hx, ox, "x") && same(hG, oG, "G") && same(hz, oz, "z");
    std::printf("steps with one scale for Q(SynQ): %s\n", g_ok ? "identical" : "DIFFERENT");
    ok = ok && g_ok;
    (void)hipFree(dqws); (void)hipFree(dws); (void)hipFree(ds0);
  }
  // a dense minibatch gradient of the logistic loss (binary64 sums rounded once on both sides, in
  // different orders: values within 1e-6, the loss too)
  {
    const int64_t n = 256, dd = 1003;
    const int B = 50;
    std::vector<float> A((size_t)n * dd), y(n), xx(dd), og(dd), hg(dd);
    std::vector<int32_t> rows(B);
    fill_gradient(A, 99);
    for (auto& v : A) v *= 40.0f;
    fill_gradient(xx, 98);
    for (int64_t i = 0; i < n; ++i) y[i] = (i * 7 % 3) ? 1.0f : -1.0f;
    for (int b = 0; b < B; ++b) rows[b] = (int32_t)((b * 37 + 11) % n);
    float ol = 0.0f, hl = 0.0f;
    orc_local_grad_dense(A.data(), n, dd, y.data(), rows.data(), B, xx.data(), og.data(), &ol);
    qa_layout Lg = L;
    Lg.d = dd; Lg.M = 1; Lg.bucket = 0; Lg.code_stride = (dd + 15) / 16; Lg.scale_stride = 1;
    const size_t wsb = qa_workspace_bytes(&Lg, QA_OP_GRAD_DENSE);
    float *dA, *dy, *dxx, *dgg, *dl;
    int32_t* drows;
    void* dws;
    HIP_OK(hipMalloc(&dA, sizeof(float) * A.size()));
    HIP_OK(hipMalloc(&dy, sizeof(float) * n));
    HIP_OK(hipMalloc(&dxx, sizeof(float) * dd));
    HIP_OK(hipMalloc(&dgg, sizeof(float) * dd));
    HIP_OK(hipMalloc(&dl, sizeof(float)));
    HIP_OK(hipMalloc(&drows, sizeof(int32_t) * B));
    HIP_OK(hipMalloc(&dws, wsb));
    HIP_OK(hipMemcpyAsync(dA, A.data(), sizeof(float) * A.size(), hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dy, y.data(), sizeof(float) * n, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dxx, xx.data(), sizeof(float) * dd, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(drows, rows.data(), sizeof(int32_t) * B, hipMemcpyHostToDevice, stream));
    QA_CALL(qa_local_grad(QA_DENSE, dA, nullptr, nullptr, n, dd, dy, drows, B, dxx, dgg, dl, dws, wsb, stream));
    HIP_OK(hipMemcpyAsync(hg.data(), dgg, sizeof(float) * dd, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipMemcpyAsync(&hl, dl, sizeof(float), hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    bool g_ok = true;
    size_t exact = 0;
    for (int64_t i = 0; i < dd; ++i) {
      const double a = hg[i], b = og[i], diff = a > b ? a - b : b - a, mag = b < 0 ? -b : b;
      g_ok = g_ok && diff <= 1e-6 * mag + 1e-12 && ((a == 0.0) == (b == 0.0));
      exact += hg[i] == og[i];
    }
    const double ldiff = hl > ol ? hl - ol : ol - hl;
    g_ok = g_ok && ldiff <= 1e-6 * ol;
    std::printf("qa_local_grad: %s (%zu of %lld components bit-identical, loss %.7g vs %.7g)\n",
                g_ok ? "within 1e-6" : "DIFFERENT", exact, (long long)dd, hl, ol);
    ok = ok && g_ok;
    (void)hipFree(dA); (void)hipFree(dy); (void)hipFree(dxx); (void)hipFree(dgg); (void)hipFree(dl);
    (void)hipFree(drows); (void)hipFree(dws);
  }
  // error path through the same ABI: nothing is launched
  if (qa_step_qcmd(&L, dcodes, dscales, dx, dG, nullptr, -1.0f, lambda, delta, 0, nullptr, 0, stream) !=
      QA_ERR_INVALID_ARG) { std::fprintf(stderr, "error path\n"); ok = false; }
  (void)hipStreamDestroy(stream);
  (void)hipFree(dg); (void)hipFree(dcodes); (void)hipFree(dscales);
  (void)hipFree(dx); (void)hipFree(dG); (void)hipFree(dz);
  return ok ? 0 : 1;
}

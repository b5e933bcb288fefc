// Minibatch gradient of the logistic loss for one worker (stochastic gradient of Section 3.1
// for the L1-regularised logistic regression of Section 5.1, arXiv 2208.05631), dense rows or
// CSR rows, for gfx950.
//
//   margins  : p_b = a_{r_b}.x in binary64 (work-group per row for dense, wave per row for CSR),
//              then coef_b = -y/(1+exp(y p_b))/B and the row's loss, in binary64.
//   gradient : dense -- one thread per 4 columns (one column when d is not a multiple of 4 or the
//                       operands are not 16-byte aligned) walks the batch in order, binary64
//                       accumulator;
//              CSR   -- hardware binary64 atomic adds into a d-long accumulator that is cleared
//                       only at the batch's columns, then rounded into the zero-filled g.
//   Every product coef*a is exact in binary64, so only the order of the binary64 additions can
//   differ from a sequential evaluation.
#include "qa_common.h"

namespace qa {

constexpr int kMaxBatch = 65536;

struct GradArgs {
  const float* A;            // dense matrix or CSR values
  const int64_t* indptr;
  const int32_t* indices;
  int64_t n_rows, d;
  const float* y;
  const int32_t* rows;
  int B;
  const float* x;
  float* g;
  float* loss_out;
  float* coef;               // [B]   workspace
  double* loss_part;         // [B]   workspace
  double* acc;               // [d]   workspace (CSR)
  // batched calls: worker m = blockIdx.y uses rows + m*B, g + m*g_stride, loss_out + m and the
  // m-th slice of each workspace array
  int64_t g_stride;
  int64_t ws_stride_bytes;
};

// View of the arguments for the worker selected by blockIdx.y.
__device__ __forceinline__ GradArgs for_worker(GradArgs a) {
  const int64_t m = blockIdx.y;
  a.rows += m * a.B;
  a.g += m * a.g_stride;
  if (a.loss_out) a.loss_out += m;
  a.coef = reinterpret_cast<float*>(reinterpret_cast<char*>(a.coef) + m * a.ws_stride_bytes);
  a.loss_part = reinterpret_cast<double*>(reinterpret_cast<char*>(a.loss_part) + m * a.ws_stride_bytes);
  a.acc = reinterpret_cast<double*>(reinterpret_cast<char*>(a.acc) + m * a.ws_stride_bytes);
  return a;
}

// The matrix rows of a batch are read once per pass: streaming (non-temporal) 16-byte load.
typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float4* p) {
  const floatx4 t = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p));
  return make_float4(t.x, t.y, t.z, t.w);
}

// coef and loss of one sample from its binary32 margin term p = a.x
__device__ __forceinline__ void logistic_terms(float p, float y, int B, float* coef, double* loss) {
  const double m = (double)y * (double)p;
  const double e = exp(-fabs(m));
  *loss = log1p(e) + (m < 0.0 ? -m : 0.0);
  const double sig = m >= 0.0 ? e / (1.0 + e) : 1.0 / (1.0 + e);
  *coef = (float)((-(double)y * sig) / (double)B);
}

// Work-group per batch row.  VEC: d is a multiple of 4 and A, x are 16-byte aligned, so a row is
// read as float4 with four loads in flight per thread.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void dense_margin_kernel(GradArgs a_all) {
  const GradArgs a = for_worker(a_all);
  __shared__ double lds_d[kWaves];
  const int b = blockIdx.x;
  const int64_t r = a.rows[b];
  const bool ok = r >= 0 && r < a.n_rows;
  double s = 0.0;
  if (ok) {
    const float* row = a.A + r * a.d;
    if (VEC) {
      const float4* row4 = reinterpret_cast<const float4*>(row);
      const float4* x4 = reinterpret_cast<const float4*>(a.x);
      const int64_t n4 = a.d / 4;
      double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
      int64_t j = threadIdx.x;
      for (; j + 3 * kThreads < n4; j += 4 * kThreads) {
        float4 v[4], w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = stream_load4(row4 + j + u * kThreads);
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = x4[j + u * kThreads];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          s0 = fma((double)v[u].x, (double)w[u].x, s0);
          s1 = fma((double)v[u].y, (double)w[u].y, s1);
          s2 = fma((double)v[u].z, (double)w[u].z, s2);
          s3 = fma((double)v[u].w, (double)w[u].w, s3);
        }
      }
      for (; j < n4; j += kThreads) {
        const float4 v = stream_load4(row4 + j), w = x4[j];
        s0 = fma((double)v.x, (double)w.x, s0);
        s1 = fma((double)v.y, (double)w.y, s1);
        s2 = fma((double)v.z, (double)w.z, s2);
        s3 = fma((double)v.w, (double)w.w, s3);
      }
      s = (s0 + s1) + (s2 + s3);
    } else {
      for (int64_t j = threadIdx.x; j < a.d; j += kThreads)
        s = fma((double)row[j], (double)a.x[j], s);
    }
  }
  s = segment_sum(s, kThreads, lds_d);
  if (threadIdx.x == 0) {
    float c = 0.0f; double l = 0.0;
    if (ok) logistic_terms((float)s, a.y[r], a.B, &c, &l);
    a.coef[b] = c; a.loss_part[b] = l;
  }
}

// g_j = sum over the batch, in batch order, of coef_b * A[r_b][j].  VEC: thread per 4 columns,
// sixteen rows' loads in flight.  The batch's row ids and coefficients pass through LDS, 1024 at
// a time, so that the matrix loads of a thread depend on nothing but an LDS read (read one by one
// from memory they made a chain of dependent scalar loads: 13.7 us for 64 rows of 1000 columns).
template <bool VEC>
__global__ __launch_bounds__(kThreads) void dense_colsum_kernel(GradArgs a_all) {
  const GradArgs a = for_worker(a_all);
  if (VEC) {
    constexpr int kRows = 16, kStage = 1024;
    __shared__ int4 s_row[kStage / 4];                    // -1: no row or id out of range, adds nothing
    __shared__ float4 s_coef[kStage / 4];
    int32_t* s_row1 = reinterpret_cast<int32_t*>(s_row);
    float* s_coef1 = reinterpret_cast<float*>(s_coef);
    const int64_t j4 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool live = j4 < a.d / 4;
    const float4* A4 = reinterpret_cast<const float4*>(a.A);
    const int64_t pitch4 = a.d / 4;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    for (int c0 = 0; c0 < a.B; c0 += kStage) {
      const int nb = a.B - c0 < kStage ? a.B - c0 : kStage;
      const int nb_pad = (nb + kRows - 1) / kRows * kRows;
      if (c0 > 0) __syncthreads();                        // the previous ids have been used
      for (int i = threadIdx.x; i < nb_pad; i += kThreads) {
        const int32_t r = i < nb ? a.rows[c0 + i] : -1;
        const bool ok = r >= 0 && r < a.n_rows;
        s_row1[i] = ok ? r : -1;
        s_coef1[i] = ok ? a.coef[c0 + i] : 0.0f;
      }
      __syncthreads();
      if (!live) continue;
      for (int b0 = 0; b0 < nb_pad; b0 += kRows) {
        int32_t r[kRows];
        float cf32[kRows];
#pragma unroll
        for (int u = 0; u < kRows / 4; ++u) {
          const int4 rr = s_row[b0 / 4 + u];
          const float4 cc = s_coef[b0 / 4 + u];
          r[4 * u] = rr.x; r[4 * u + 1] = rr.y; r[4 * u + 2] = rr.z; r[4 * u + 3] = rr.w;
          cf32[4 * u] = cc.x; cf32[4 * u + 1] = cc.y; cf32[4 * u + 2] = cc.z; cf32[4 * u + 3] = cc.w;
        }
        float4 v[kRows];
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          v[u] = stream_load4(A4 + (int64_t)(r[u] >= 0 ? r[u] : 0) * pitch4 + j4);
          if (r[u] < 0) v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          const double cf = (double)cf32[u];
          acc0 = fma(cf, (double)v[u].x, acc0);
          acc1 = fma(cf, (double)v[u].y, acc1);
          acc2 = fma(cf, (double)v[u].z, acc2);
          acc3 = fma(cf, (double)v[u].w, acc3);
        }
      }
    }
    if (live)
      reinterpret_cast<float4*>(a.g)[j4] = make_float4((float)acc0, (float)acc1, (float)acc2, (float)acc3);
  } else {
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= a.d) return;
    double acc = 0.0;
    for (int b = 0; b < a.B; ++b) {
      const int64_t r = a.rows[b];
      if (r < 0 || r >= a.n_rows) continue;
      acc = fma((double)a.coef[b], (double)a.A[r * a.d + j], acc);
    }
    a.g[j] = (float)acc;
  }
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float* p_all, int64_t n,
                                                            int64_t stride) {
  float* p = p_all + (int64_t)blockIdx.y * stride;
  const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
  if (i + 3 < n) *reinterpret_cast<float4*>(p + i) = make_float4(0.f, 0.f, 0.f, 0.f);
  else for (int e = 0; e < 4; ++e) if (i + e < n) p[i + e] = 0.0f;
}

// one wave per batch row: margin, coef, loss; also clears the accumulator at the row's columns.
// ZERO_G: the work-groups of a worker first share out the zero-fill of its gradient vector (the
// stores drain while the latency-bound margins are computed); otherwise fill_zero_kernel ran before.
template <bool ZERO_G>
__global__ __launch_bounds__(kThreads) void csr_margin_kernel(GradArgs a_all) {
  const GradArgs a = for_worker(a_all);
  if (ZERO_G) {
    const int64_t n4 = a.d / 4;
    const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per, hi = lo + per < n4 ? lo + per : n4;
    float4* g4 = reinterpret_cast<float4*>(a.g);
    for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) g4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (blockIdx.x == 0 && threadIdx.x < (a.d & 3)) a.g[4 * n4 + threadIdx.x] = 0.0f;
  }
  const int b = blockIdx.x * kWaves + threadIdx.x / kWave;
  if (b >= a.B) return;
  const int lane = threadIdx.x % kWave;
  const int64_t r = a.rows[b];
  const bool ok = r >= 0 && r < a.n_rows;
  double s = 0.0;
  if (ok) {
    const int64_t k0 = a.indptr[r], k1 = a.indptr[r + 1];
    for (int64_t k = k0 + lane; k < k1; k += kWave) {
      const uint32_t c = (uint32_t)a.indices[k];
      if (c < (uint64_t)a.d) {
        s = fma((double)a.A[k], (double)a.x[c], s);
        a.acc[c] = 0.0;
      }
    }
  }
  for (int off = 1; off < kWave; off <<= 1) s += shfl_xor_f64(s, off);
  if (lane == 0) {
    float c = 0.0f; double l = 0.0;
    if (ok) logistic_terms((float)s, a.y[r], a.B, &c, &l);
    a.coef[b] = c; a.loss_part[b] = l;
  }
}

template <bool FINALIZE>
__global__ __launch_bounds__(kThreads) void csr_scatter_kernel(GradArgs a_all) {
  const GradArgs a = for_worker(a_all);
  const int b = blockIdx.x * kWaves + threadIdx.x / kWave;
  if (b >= a.B) return;
  const int lane = threadIdx.x % kWave;
  const int64_t r = a.rows[b];
  if (r < 0 || r >= a.n_rows) return;
  const double cf = (double)a.coef[b];
  const int64_t k0 = a.indptr[r], k1 = a.indptr[r + 1];
  for (int64_t k = k0 + lane; k < k1; k += kWave) {
    const uint32_t c = (uint32_t)a.indices[k];
    if (c >= (uint64_t)a.d) continue;
    if (FINALIZE) a.g[c] = (float)a.acc[c];
    else unsafeAtomicAdd(&a.acc[c], cf * (double)a.A[k]);
  }
}

__global__ __launch_bounds__(kThreads) void loss_finalize_kernel(GradArgs a_all) {
  const GradArgs a = for_worker(a_all);
  __shared__ double lds_d[kWaves];
  double s = 0.0;
  for (int b = threadIdx.x; b < a.B; b += kThreads) s += a.loss_part[b];
  s = segment_sum(s, kThreads, lds_d);
  if (threadIdx.x == 0) *a.loss_out = (float)(s / (double)a.B);
}

static inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t grad_workspace_bytes(int64_t d, bool csr) {
  return align256((size_t)kMaxBatch * sizeof(float)) + align256((size_t)kMaxBatch * sizeof(double)) +
         (csr ? align256((size_t)d * sizeof(double)) : 0);
}

static int grad_launch(int format, const float* A_or_vals, const int64_t* indptr,
                       const int32_t* indices, int64_t n_rows, int64_t d, const float* y,
                       const int32_t* batch_rows, int32_t B, int32_t M, const float* x, float* g_out,
                       int64_t g_stride, float* loss_out, void* ws, size_t ws_bytes,
                       hipStream_t stream) {
  if (format != QA_DENSE && format != QA_CSR) return QA_ERR_INVALID_ARG;
  if (!A_or_vals || !y || !batch_rows || !x || !g_out) return QA_ERR_INVALID_ARG;
  if (format == QA_CSR && (!indptr || !indices)) return QA_ERR_INVALID_ARG;
  if (n_rows < 1 || d < 1 || d >= (int64_t(1) << 31) || B < 1 || B > kMaxBatch || M < 1 || M > 4096)
    return QA_ERR_INVALID_ARG;
  if (M > 1 && (g_stride < d || (g_stride % 4) != 0)) return QA_ERR_INVALID_ARG;
  if (!aligned(g_out, 16) || !aligned(A_or_vals, 4) || !aligned(x, 4) || !aligned(indptr, 8) ||
      !aligned(indices, 4) || !aligned(batch_rows, 4) || !aligned(loss_out, 4))
    return QA_ERR_ALIGNMENT;
  const bool csr = format == QA_CSR;
  const size_t per_worker = grad_workspace_bytes(d, csr);
  if (!ws || ws_bytes < per_worker * (size_t)M) return QA_ERR_WORKSPACE;
  if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;

  GradArgs a{};
  a.A = A_or_vals; a.indptr = indptr; a.indices = indices; a.n_rows = n_rows; a.d = d;
  a.y = y; a.rows = batch_rows; a.B = B; a.x = x; a.g = g_out; a.loss_out = loss_out;
  a.g_stride = g_stride; a.ws_stride_bytes = (int64_t)per_worker;
  char* p = static_cast<char*>(ws);
  a.coef = reinterpret_cast<float*>(p);        p += align256((size_t)kMaxBatch * sizeof(float));
  a.loss_part = reinterpret_cast<double*>(p);  p += align256((size_t)kMaxBatch * sizeof(double));
  a.acc = reinterpret_cast<double*>(p);

  const dim3 block(kThreads);
  const unsigned Mu = (unsigned)M;
  if (!csr) {
    if ((d % 4) == 0 && aligned(A_or_vals, 16) && aligned(x, 16)) {
      hipLaunchKernelGGL((dense_margin_kernel<true>), dim3(B, Mu), block, 0, stream, a);
      hipLaunchKernelGGL((dense_colsum_kernel<true>),
                         dim3((unsigned)((d / 4 + kThreads - 1) / kThreads), Mu), block, 0, stream, a);
    } else {
      hipLaunchKernelGGL((dense_margin_kernel<false>), dim3(B, Mu), block, 0, stream, a);
      hipLaunchKernelGGL((dense_colsum_kernel<false>),
                         dim3((unsigned)((d + kThreads - 1) / kThreads), Mu), block, 0, stream, a);
    }
  } else {
    const dim3 grid_rows((B + kWaves - 1) / kWaves, Mu);
    // few rows for a long vector: the zero-fill gets a launch of its own
    const bool fused_fill = d / 4 <= (int64_t)grid_rows.x * kThreads * 32;
    if (fused_fill) {
      hipLaunchKernelGGL(csr_margin_kernel<true>, grid_rows, block, 0, stream, a);
    } else {
      hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((d + 4 * kThreads - 1) / (4 * kThreads)), Mu),
                         block, 0, stream, g_out, d, g_stride);
      hipLaunchKernelGGL(csr_margin_kernel<false>, grid_rows, block, 0, stream, a);
    }
    hipLaunchKernelGGL((csr_scatter_kernel<false>), grid_rows, block, 0, stream, a);
    hipLaunchKernelGGL((csr_scatter_kernel<true>), grid_rows, block, 0, stream, a);
  }
  if (loss_out) hipLaunchKernelGGL(loss_finalize_kernel, dim3(1, Mu), block, 0, stream, a);
  return launch_status();
}

}  // namespace qa

extern "C" int qa_local_grad(int format, const float* A_or_vals, const int64_t* indptr,
                             const int32_t* indices, int64_t n_rows, int64_t d, const float* y,
                             const int32_t* batch_rows, int32_t B, const float* x, float* g_out,
                             float* loss_out, void* ws, size_t ws_bytes, void* stream) {
  return qa::grad_launch(format, A_or_vals, indptr, indices, n_rows, d, y, batch_rows, B, 1, x, g_out,
                         0, loss_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int qa_local_grad_batched(int format, const float* A_or_vals, const int64_t* indptr,
                                     const int32_t* indices, int64_t n_rows, int64_t d,
                                     const float* y, const int32_t* batch_rows, int32_t B, int32_t M,
                                     const float* x, float* g_out, int64_t g_stride, float* loss_out,
                                     void* ws, size_t ws_bytes, void* stream) {
  return qa::grad_launch(format, A_or_vals, indptr, indices, n_rows, d, y, batch_rows, B, M, x, g_out,
                         g_stride, loss_out, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

// Tensor-list quantizer: the threshold quantizer of Sections 3.4-3.5 applied to each tensor of a
// flat vector on its own, all tensors and all workers in one launch per pass.
//
// Work-group = one piece (tile x tensor intersection) of one worker.  Four passes, as for a
// bucket larger than a tile: piece sums of |v| -> threshold per tensor -> codes and piece
// (sum, count) of the kept magnitudes -> scale per tensor.  Partial results are combined in a
// fixed order in binary64, so the result does not depend on scheduling.
#include <vector>

#include "qa_segments.h"

namespace qa {

struct SegQuantArgs {
  const float* g;
  int64_t g_stride;
  int64_t d;
  uint32_t* codes;
  int64_t code_stride;
  float* scales;
  float* thresholds;        // user array, may be null
  int64_t scale_stride;
  float thr_coef;
  double* part_sum;         // [M][n_pieces]
  uint32_t* part_cnt;       // [M][n_pieces]
  float* thr_ws;            // [M][n_seg]
  SegTable seg;
};

// The thread's 4 float4 groups f = j*256 + t of the piece's tile; elements outside [lo, hi)
// read as +0 (lo is a multiple of 16, so a group never straddles it).
__device__ __forceinline__ void load_piece_values(const float* __restrict__ g, const Piece& pc,
                                                  float v[4][4]) {
  const int64_t base = pc.tile * kTile;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t i = base + (int64_t)(j * kThreads + (int)threadIdx.x) * 4;
    if (i >= pc.lo && i + 3 < pc.hi) {
      // streaming: each of the two passes over the gradients reads an element once, a whole
      // pass apart
      typedef float floatx4 __attribute__((ext_vector_type(4)));
      const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + i));
      v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[j][e] = (i + e >= pc.lo && i + e < pc.hi) ? g[i + e] : 0.0f;
    }
  }
}

__global__ __launch_bounds__(kThreads) void seg_abs_partial_kernel(SegQuantArgs a) {
  __shared__ double lds_d[kWaves];
  const int64_t p = blockIdx.x;
  const int m = blockIdx.y;
  const Piece pc = load_piece(a.seg, p, a.d);
  float v[4][4];
  load_piece_values(a.g + (int64_t)m * a.g_stride, pc, v);
  double s = 0.0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) s += (double)fabsf(v[j][e]);
  s = block_sum_f64(s, lds_d);
  if (threadIdx.x == 0) a.part_sum[(int64_t)m * a.seg.n_pieces + p] = s;
}

// Pieces of tensor s, clamped to the table.
__device__ __forceinline__ void piece_range(const SegTable& T, int64_t s, int64_t* p0, int64_t* p1) {
  int64_t a = T.piece_first[s], b = T.piece_first[s + 1];
  a = a < 0 ? 0 : (a > T.n_pieces ? T.n_pieces : a);
  b = b < a ? a : (b > T.n_pieces ? T.n_pieces : b);
  *p0 = a; *p1 = b;
}

__global__ __launch_bounds__(kThreads) QA_FEW_WAVES void seg_threshold_finalize_kernel(SegQuantArgs a) {
  __shared__ double lds_d[kWaves];
  const int64_t s = blockIdx.x;
  const int m = blockIdx.y;
  int64_t p0, p1;
  piece_range(a.seg, s, &p0, &p1);
  double sum = strided_partial_sum(a.part_sum + (int64_t)m * a.seg.n_pieces, p0, p1);
  sum = segment_sum(sum, kThreads, lds_d);
  if (threadIdx.x == 0) {
    const int64_t n = a.seg.length[s];
    const float Delta = n > 0 ? threshold_from_sum(sum, a.thr_coef, n) : 0.0f;
    a.thr_ws[(int64_t)m * a.seg.n_seg + s] = Delta;
    if (a.thresholds) a.thresholds[(int64_t)m * a.scale_stride + s] = Delta;
  }
}

__global__ __launch_bounds__(kThreads) void seg_codes_partial_kernel(SegQuantArgs a) {
  __shared__ double lds_d[kWaves];
  __shared__ uint32_t lds_u[kWaves];
  const int t = threadIdx.x;
  const int64_t p = blockIdx.x;
  const int m = blockIdx.y;
  const Piece pc = load_piece(a.seg, p, a.d);
  const float D = a.thr_ws[(int64_t)m * a.seg.n_seg + pc.seg];
  float v[4][4];
  load_piece_values(a.g + (int64_t)m * a.g_stride, pc, v);
  double s = 0.0;
  uint32_t c = 0;
  uint32_t mine = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t b = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float av = fabsf(v[j][e]);
      if (av > D) { s += (double)av; ++c; }
      b |= ternary_field(v[j][e], D) << (2 * e);
    }
    // the four lanes of a quad hold the four bytes of code word j*64 + t/4 of the tile
    uint32_t w = b << (8 * (t & 3));
    w |= (uint32_t)dpp_i32<kDppQuadXor1>((int)w);
    w |= (uint32_t)dpp_i32<kDppQuadXor2>((int)w);
    if ((t & 3) == j) mine = w;
  }
  // words of the tile that hold coordinates of this piece
  const int64_t base = pc.tile * kTile;
  const int wlo = (int)((pc.lo - base) >> 4), whi = (int)((pc.hi - base + 15) >> 4);
  const int wl = (t & 3) * 64 + (t >> 2);
  if (wl >= wlo && wl < whi)
    a.codes[(int64_t)m * a.code_stride + pc.tile * kTileWords + wl] = mine;
  s = wave_sum_f64(s);
  c = wave_sum_u32(c);
  if ((t % kWave) == 0) { lds_d[t / kWave] = s; lds_u[t / kWave] = c; }
  __syncthreads();
  if (t == 0) {
    a.part_sum[(int64_t)m * a.seg.n_pieces + p] = (lds_d[0] + lds_d[1]) + (lds_d[2] + lds_d[3]);
    a.part_cnt[(int64_t)m * a.seg.n_pieces + p] = lds_u[0] + lds_u[1] + lds_u[2] + lds_u[3];
  }
}

__global__ __launch_bounds__(kThreads) QA_FEW_WAVES void seg_scale_finalize_kernel(SegQuantArgs a) {
  __shared__ double lds_d[kWaves];
  __shared__ double lds_c[kWaves];
  const int64_t s = blockIdx.x;
  const int m = blockIdx.y;
  int64_t p0, p1;
  piece_range(a.seg, s, &p0, &p1);
  // counts are integers < 2^53: exact in binary64
  double sum, cnt;
  strided_partial_sums(a.part_sum + (int64_t)m * a.seg.n_pieces, a.part_cnt + (int64_t)m * a.seg.n_pieces, p0, p1,
                       &sum, &cnt);
  sum = segment_sum(sum, kThreads, lds_d);
  cnt = segment_sum(cnt, kThreads, lds_c);
  if (threadIdx.x == 0)
    a.scales[(int64_t)m * a.scale_stride + s] = scale_from_sum(sum, (uint64_t)cnt);
}

static inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t quantize_segments_workspace_bytes(const qa_segment_plan* P, int M) {
  const size_t np = (size_t)(P->n_pieces > 0 ? P->n_pieces : 1);
  return align256((size_t)M * np * sizeof(double)) + align256((size_t)M * np * sizeof(uint32_t)) +
         align256((size_t)M * (size_t)P->n_seg * sizeof(float));
}

int quantize_segments_launch(const qa_layout* L, const qa_segment_plan* P, const float* g,
                             int64_t g_stride, uint32_t* codes, float* scales, float* thresholds,
                             void* ws, size_t ws_bytes, hipStream_t stream) {
  if (!ws || ws_bytes < quantize_segments_workspace_bytes(P, L->M)) return QA_ERR_WORKSPACE;
  if (!aligned(ws, 256)) return QA_ERR_ALIGNMENT;
  SegQuantArgs a{};
  a.g = g; a.g_stride = g_stride; a.d = L->d;
  a.codes = codes; a.code_stride = L->code_stride;
  a.scales = scales; a.thresholds = thresholds; a.scale_stride = L->scale_stride;
  a.thr_coef = L->thr_coef;
  a.seg = seg_table_of(P);
  const size_t np = (size_t)(P->n_pieces > 0 ? P->n_pieces : 1);
  char* p = static_cast<char*>(ws);
  a.part_sum = reinterpret_cast<double*>(p);    p += align256((size_t)L->M * np * sizeof(double));
  a.part_cnt = reinterpret_cast<uint32_t*>(p);  p += align256((size_t)L->M * np * sizeof(uint32_t));
  a.thr_ws = reinterpret_cast<float*>(p);
  const dim3 block(kThreads);
  const dim3 grid_p((unsigned)P->n_pieces, (unsigned)L->M), grid_s((unsigned)P->n_seg, (unsigned)L->M);
  if (P->n_pieces > 0) hipLaunchKernelGGL(seg_abs_partial_kernel, grid_p, block, 0, stream, a);
  hipLaunchKernelGGL(seg_threshold_finalize_kernel, grid_s, block, 0, stream, a);
  if (P->n_pieces > 0) hipLaunchKernelGGL(seg_codes_partial_kernel, grid_p, block, 0, stream, a);
  hipLaunchKernelGGL(seg_scale_finalize_kernel, grid_s, block, 0, stream, a);
  return launch_status();
}

}  // namespace qa

extern "C" size_t qa_segment_plan_bytes(int64_t d, int64_t n_seg) {
  using namespace qa;
  if (d < 1 || d >= (int64_t(1) << 40) || n_seg < 1 || n_seg > 0x7fffffffLL) return 0;
  const int64_t np_max = tiles_of(d) + n_seg;
  return (size_t)(kSegHeader + 2 * n_seg + (n_seg + 1) + 2 * np_max) * sizeof(int64_t);
}

// Validates the tensor list and writes the table (layout in qa_segments.h) into host memory.
static int build_table(int64_t d, int64_t n_seg, const int64_t* begin, const int64_t* length,
                       std::vector<int64_t>& h, int64_t* n_pieces_out) {
  using namespace qa;
  if (!begin || !length) return QA_ERR_INVALID_ARG;
  if (qa_segment_plan_bytes(d, n_seg) == 0) return QA_ERR_INVALID_ARG;
  int64_t end_prev = 0, n_pieces = 0;
  for (int64_t s = 0; s < n_seg; ++s) {
    if (begin[s] < end_prev || (begin[s] & 15) != 0 || length[s] < 0) return QA_ERR_INVALID_ARG;
    if (begin[s] > d || length[s] > d - begin[s]) return QA_ERR_INVALID_ARG;
    end_prev = begin[s] + length[s];
    if (length[s] > 0) n_pieces += (end_prev - 1) / kTile - begin[s] / kTile + 1;
  }
  if (n_pieces > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  h.assign((size_t)(kSegHeader + 2 * n_seg + (n_seg + 1) + 2 * n_pieces), 0);
  h[0] = kSegMagic; h[1] = d; h[2] = n_seg; h[3] = n_pieces;
  int64_t* hb = h.data() + kSegHeader;
  int64_t* hl = hb + n_seg;
  int64_t* hf = hl + n_seg;
  int64_t* ht = hf + n_seg + 1;
  int64_t* hs = ht + n_pieces;
  int64_t p = 0;
  for (int64_t s = 0; s < n_seg; ++s) {
    hb[s] = begin[s]; hl[s] = length[s]; hf[s] = p;
    if (length[s] > 0)
      for (int64_t T = begin[s] / kTile; T <= (begin[s] + length[s] - 1) / kTile; ++T) { ht[p] = T; hs[p] = s; ++p; }
  }
  hf[n_seg] = p;
  *n_pieces_out = n_pieces;
  return QA_OK;
}

extern "C" int qa_segment_plan_host(int64_t d, int64_t n_seg, const int64_t* begin,
                                    const int64_t* length, int64_t* table_host, size_t table_bytes,
                                    int64_t* n_pieces_out) {
  if (!n_pieces_out) return QA_ERR_INVALID_ARG;
  std::vector<int64_t> h;
  int rc = build_table(d, n_seg, begin, length, h, n_pieces_out);
  if (rc != QA_OK) return rc;
  if (table_host) {
    if (table_bytes < h.size() * sizeof(int64_t)) return QA_ERR_WORKSPACE;
    for (size_t i = 0; i < h.size(); ++i) table_host[i] = h[i];
  }
  return QA_OK;
}

extern "C" int qa_segment_plan_init(int64_t d, int64_t n_seg, const int64_t* begin,
                                    const int64_t* length, void* table, size_t table_bytes,
                                    qa_segment_plan* plan_out, void* stream) {
  using namespace qa;
  if (!begin || !length || !table || !plan_out) return QA_ERR_INVALID_ARG;
  if (qa_segment_plan_bytes(d, n_seg) == 0) return QA_ERR_INVALID_ARG;
  if (!aligned(table, 8)) return QA_ERR_ALIGNMENT;
  std::vector<int64_t> h;
  int64_t n_pieces = 0;
  int rc = build_table(d, n_seg, begin, length, h, &n_pieces);
  if (rc != QA_OK) return rc;
  if (table_bytes < h.size() * sizeof(int64_t)) return QA_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(table, h.data(), h.size() * sizeof(int64_t), hipMemcpyHostToDevice, st) != hipSuccess)
    return QA_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return QA_ERR_LAUNCH;
  plan_out->d = d; plan_out->n_seg = n_seg; plan_out->n_pieces = n_pieces; plan_out->table = table;
  return QA_OK;
}

extern "C" int qa_quantize_pack_segments(const qa_layout* layout, const qa_segment_plan* plan,
                                         const float* g, int64_t g_stride, uint32_t* codes,
                                         float* scales, float* thresholds, void* ws,
                                         size_t ws_bytes, void* stream) {
  using namespace qa;
  int rc = check_layout(layout);
  if (rc != QA_OK) return rc;
  rc = check_plan(plan, layout);
  if (rc != QA_OK) return rc;
  if (!g || !codes || !scales) return QA_ERR_INVALID_ARG;
  if (g_stride < layout->d || (g_stride & 3) != 0) return QA_ERR_INVALID_ARG;
  if (!aligned(g, 16) || !aligned(codes, 4) || !aligned(scales, 4) || !aligned(thresholds, 4))
    return QA_ERR_ALIGNMENT;
  return quantize_segments_launch(layout, plan, g, g_stride, codes, scales, thresholds, ws, ws_bytes,
                                  static_cast<hipStream_t>(stream));
}

// A list of tensors in one flat vector: the device table behind qa_segment_plan and the
// decomposition of the vector into pieces.  Internal to libqadagrad.
//
// A piece is the intersection of one 4096-coordinate tile with one tensor; a work-group of the
// tensor-list kernels handles one piece, so that all its coordinates share their scales.  Pieces
// are numbered in order of (tensor, tile); the pieces of tensor s are piece_first[s] ..
// piece_first[s+1]-1.
//
// Table layout in device memory, in int64 units:
//   [0] magic  [1] d  [2] n_seg  [3] n_pieces
//   begin[n_seg]  length[n_seg]  piece_first[n_seg+1]  piece_tile[n_pieces]  piece_seg[n_pieces]
#pragma once
#include "qa_common.h"

namespace qa {

constexpr int64_t kSegMagic = 0x7161736567746162LL;
constexpr int64_t kSegHeader = 4;

struct SegTable {
  const int64_t* begin;
  const int64_t* length;
  const int64_t* piece_first;
  const int64_t* piece_tile;       // null: not a tensor-list launch
  const int64_t* piece_seg;
  int64_t n_seg, n_pieces;
};

inline SegTable seg_table_of(const qa_segment_plan* P) {
  SegTable T{};
  const int64_t* t = static_cast<const int64_t*>(P->table) + kSegHeader;
  T.begin = t;                      t += P->n_seg;
  T.length = t;                     t += P->n_seg;
  T.piece_first = t;                t += P->n_seg + 1;
  T.piece_tile = t;                 t += P->n_pieces;
  T.piece_seg = t;
  T.n_seg = P->n_seg; T.n_pieces = P->n_pieces;
  return T;
}

// Host-side consistency of a plan with a layout (the table's contents were validated when
// qa_segment_plan_init wrote it; the kernels additionally clamp every range to [0, d)).
inline int check_plan(const qa_segment_plan* P, const qa_layout* L) {
  if (!P || !P->table) return QA_ERR_INVALID_ARG;
  if (P->d != L->d || P->n_seg < 1 || P->n_pieces < 0) return QA_ERR_INVALID_ARG;
  if (P->n_pieces > tiles_of(P->d) + P->n_seg || P->n_pieces > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  if (P->n_seg > 0x7fffffffLL) return QA_ERR_INVALID_ARG;
  if (L->bucket != 0) return QA_ERR_INVALID_ARG;              // one scale per tensor
  if (L->scale_stride < P->n_seg) return QA_ERR_INVALID_ARG;
  if (!aligned(P->table, 8)) return QA_ERR_ALIGNMENT;
  return QA_OK;
}

#if defined(__HIPCC__)
struct Piece {
  int64_t tile, seg;
  int64_t lo, hi;                  // absolute coordinates, tile*4096 <= lo <= hi <= tile*4096+4096
};

// Uniform per work-group (scalar loads).  Every bound is clamped so that a damaged table cannot
// lead outside [0, d).
__device__ __forceinline__ Piece load_piece(const SegTable& T, int64_t p, int64_t d) {
  Piece q;
  const int64_t ntiles = (d + kTile - 1) / kTile;
  int64_t tile = T.piece_tile[p], seg = T.piece_seg[p];
  tile = tile < 0 ? 0 : (tile >= ntiles ? ntiles - 1 : tile);
  seg = seg < 0 ? 0 : (seg >= T.n_seg ? T.n_seg - 1 : seg);
  const int64_t b = T.begin[seg], e = b + T.length[seg];
  const int64_t t0 = tile * kTile;
  int64_t t1 = t0 + kTile;
  t1 = t1 < d ? t1 : d;
  int64_t lo = b > t0 ? b : t0, hi = e < t1 ? e : t1;
  lo = lo > t1 ? t1 : lo;
  lo &= ~int64_t(15);
  hi = hi < lo ? lo : hi;
  q.tile = tile; q.seg = seg; q.lo = lo; q.hi = hi;
  return q;
}
#endif

// defined in qa_segments.hip
size_t quantize_segments_workspace_bytes(const qa_segment_plan* P, int M);
int quantize_segments_launch(const qa_layout* L, const qa_segment_plan* P, const float* g,
                             int64_t g_stride, uint32_t* codes, float* scales, float* thresholds,
                             void* ws, size_t ws_bytes, hipStream_t stream);

}  // namespace qa

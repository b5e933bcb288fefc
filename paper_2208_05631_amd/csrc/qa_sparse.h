// Device helpers shared by the kernels that read or write the sparse encoding (indicator bits +
// compact per-bucket code stream; Section 3.2, Encode paragraph).  Internal to libqadagrad.
#pragma once
#include "qa_common.h"

namespace qa {

// Inclusive prefix sum over the 64 lanes with DPP: shifts within each row of 16 lanes, then the
// last lane of a row is broadcast into the following rows.  A lane without a source adds 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v) {
  v += dpp_or_zero<0x111, 0xF>(v);      // row_shr:1
  v += dpp_or_zero<0x112, 0xF>(v);      // row_shr:2
  v += dpp_or_zero<0x114, 0xF>(v);      // row_shr:4
  v += dpp_or_zero<0x118, 0xF>(v);      // row_shr:8
  v += dpp_or_zero<0x142, 0xA>(v);      // row_bcast:15 into rows 1 and 3
  v += dpp_or_zero<0x143, 0xC>(v);      // row_bcast:31 into rows 2 and 3
  return v;
}

// Deposit table: entry [nib][s] spreads the low 2-bit codes of s to the 2-bit fields of a byte
// whose positions are the set bits of the 4-bit mask nib (first code to the lowest set bit).
struct DepositLut { uint8_t v[16 * 256]; };
constexpr DepositLut make_deposit_lut() {
  DepositLut t{};
  for (int nib = 0; nib < 16; ++nib)
    for (int s = 0; s < 256; ++s) {
      uint32_t w = (uint32_t)s, out = 0;
      for (int b = 0; b < 4; ++b)
        if ((nib >> b) & 1) { out |= (w & 3u) << (2 * b); w >>= 2; }
      t.v[nib * 256 + s] = (uint8_t)out;
    }
  return t;
}
static __device__ const DepositLut kDepositLut = make_deposit_lut();

}  // namespace qa

// MFMA operand fragments read out of LDS tiles whose reduction index is the slow one.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cdp {

typedef short frag_v4s __attribute__((ext_vector_type(4)));

// Operand of one 32x32x16 bf16 MFMA from a tile stored tile[k][r] (r contiguous, `pitch`
// elements per k): rows r0..r0+31, reduction indices k0..k0+15.  Lane l of the MFMA wants the
// eight values tile[k0 + 8*(l/32) + 0..7][r0 + l%32], a column of the stored tile.  The
// transposing LDS read of gfx950 (ds_read_b64_tr_b16) hands every lane of a 16-lane group four
// 16-bit values taken from the 8-byte rows that four OTHER lanes of the group address: with
// the 16 addresses arranged as (k offset = lane/4, r offset = 4*(lane%4)) lane i receives
// tile[k..k+3][rbase + i].  Two such reads make the fragment.
// Requirements: pitch and r0 multiples of 4 elements, tile 8-byte aligned.  Rows k..k+3 are
// read together, so a pitch of 32 bytes modulo 128 keeps the four 32-byte pieces on distinct banks.
__device__ __forceinline__ uint4 frag_tr_bf16(const uint16_t* tile, int pitch, int k0, int r0, int lane) {
  const int rho = lane & 15;
  const uint16_t* p = tile + (k0 + 8 * (lane >> 5) + (rho >> 2)) * pitch + r0 + 16 * ((lane >> 4) & 1) + 4 * (rho & 3);
  typedef __attribute__((address_space(3))) frag_v4s* lds_v4s_ptr;
  const frag_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p));
  const frag_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p + 4 * pitch));
  union { frag_v4s v[2]; uint4 u; } r;
  r.v[0] = lo;
  r.v[1] = hi;
  return r.u;
}

}  // namespace cdp

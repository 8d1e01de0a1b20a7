// Device-side helpers shared by the kernels of libnosa (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "../../include/nosa.h"

namespace nosa {
namespace dev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// x + (x of another lane), the other lane chosen by a DPP control word: one VALU instruction.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
}

// Sum over the LPR adjacent lanes (8, 16 or 32) that hold one row; every one of them receives the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  static_assert(LPR == 8 || LPR == 16 || LPR == 32, "rows span 8, 16 or 32 lanes");
  x = dpp_add<0xB1>(x);                            // quad_perm [1,0,3,2] : lane ^ 1
  x = dpp_add<0x4E>(x);                            // quad_perm [2,3,0,1] : lane ^ 2
  x = dpp_add<0x141>(x);                           // row_half_mirror     : the other quad of 8
  if constexpr (LPR >= 16) x = dpp_add<0x140>(x);  // row_mirror          : the other half of 16
  if constexpr (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

// Order-preserving map float -> uint32 (larger float, larger key).  NaN ranks with -inf; every key is
// >= 0x007fffff, so 0 can mark "not a candidate".
__device__ __forceinline__ uint32_t order_key(float f) {
  if (f != f) f = -INFINITY;
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// fp64 -> bf16, round to nearest even, for finite values in the normal fp32 range (or zero).
__device__ __forceinline__ uint16_t f64_to_bf16(double x) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  const uint32_t sign = (uint32_t)(u >> 48) & 0x8000u;
  const int e = (int)((u >> 52) & 0x7ff) - 1023 + 127;   // fp32-biased exponent
  if (e <= 0) return (uint16_t)sign;                      // below the normal range: flush to zero
  if (e >= 255) return (uint16_t)(sign | 0x7f80u);
  const uint64_t man = u & 0xfffffffffffffull;            // 52 bits
  const uint32_t top = (uint32_t)(man >> 45);             // 7 kept bits
  const uint64_t rest = man & ((1ull << 45) - 1), half = 1ull << 44;
  uint32_t mag = ((uint32_t)e << 7) | top;
  if (rest > half || (rest == half && (top & 1u))) mag += 1;   // a carry may bump the exponent: still correct
  return (uint16_t)(sign | mag);
}

// 16 bytes of a row -> fp32 elements (8 for bf16, 4 for fp32).
template <int DT>
__device__ __forceinline__ void widen16(const uint4& raw, float* f);
template <>
__device__ __forceinline__ void widen16<NOSA_DTYPE_BF16>(const uint4& raw, float* f) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
template <>
__device__ __forceinline__ void widen16<NOSA_DTYPE_F32>(const uint4& raw, float* f) {
  f[0] = __uint_as_float(raw.x);
  f[1] = __uint_as_float(raw.y);
  f[2] = __uint_as_float(raw.z);
  f[3] = __uint_as_float(raw.w);
}

}  // namespace dev
}  // namespace nosa

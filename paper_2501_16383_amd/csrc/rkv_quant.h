// Device helpers shared by the write-half kernels: fp16 row loads and the quantizer of Eq. 6-9.
#pragma once
#include "rkv_internal.h"

template <int PL>
__device__ inline void load_halves(const __half* p, float (&x)[PL]) {
  if constexpr (PL >= 8) {
#pragma unroll
    for (int k = 0; k < PL / 8; ++k) {
      uint4 u = reinterpret_cast<const uint4*>(p)[k];
      const __half2* h = reinterpret_cast<const __half2*>(&u);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float2 f = __half22float2(h[i]);
        x[8 * k + 2 * i] = f.x;
        x[8 * k + 2 * i + 1] = f.y;
      }
    }
  } else if constexpr (PL == 4) {
    uint2 u = *reinterpret_cast<const uint2*>(p);
    const __half2* h = reinterpret_cast<const __half2*>(&u);
    float2 f0 = __half22float2(h[0]), f1 = __half22float2(h[1]);
    x[0] = f0.x; x[1] = f0.y; x[2] = f1.x; x[3] = f1.y;
  } else {
    uint32_t u = *reinterpret_cast<const uint32_t*>(p);
    float2 f = __half22float2(*reinterpret_cast<const __half2*>(&u));
    x[0] = f.x; x[1] = f.y;
  }
}

// Eq. 8-9 for one block given its min and max and the largest code qmax = 2^bits - 1: fp16 scale actually stored, integer zero,
// and the reciprocal of the scale (one IEEE division per block; elements multiply by it, which
// differs from x / s only within ~1.5 ulp, far inside the rounding-tie window of the parity tests).
// meta8: the scale is stored in FP8 E4M3 rounded up (a positive range then never rounds to 0) and
// the zero-point in INT8.
__device__ inline void quant_params(float mn, float mx, float& s, float& zero, float& inv_s, bool meta8 = false, float qmax = 3.0f) {
  float raw = (mx - mn) / qmax;
  if (meta8) {
    s = rkv_e4m3_round_up(raw);
    if (s == 0.0f) {
      s = rkv_e4m3_round_up(fabsf(mn));
      if (s == 0.0f) s = 1.0f;
    }
    inv_s = 1.0f / s;
    zero = fminf(fmaxf(-rintf(mn * inv_s), -128.0f), 127.0f);
    return;
  }
  s = __half2float(__float2half_rn(raw));
  if (!(s <= 65504.0f)) s = 65504.0f;
  if (s == 0.0f) {
    s = __half2float(__float2half_rn(fabsf(mn)));
    if (!(s <= 65504.0f)) s = 65504.0f;
    if (s == 0.0f) s = 1.0f;
  }
  inv_s = 1.0f / s;
  zero = -rintf(mn * inv_s);
  zero = fminf(fmaxf(zero, -2048.0f), 2048.0f);
}
// Eq. 6
__device__ inline uint32_t quant_code(float x, float inv_s, float zero, float qmax = 3.0f) {
  // adding 1.5 * 2^23 rounds x * inv_s to an integer (ties to even, as rintf) in the same FMA and
  // leaves that integer in the low mantissa bits, which saves the float -> int conversion
  const float magic = 12582912.0f;
  float q = fmaf(x, inv_s, magic) + zero;
  q = fminf(fmaxf(q, magic), magic + qmax);
  return __float_as_uint(q) & 15u;
}

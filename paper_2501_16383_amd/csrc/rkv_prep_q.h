// Query preparation of the read half: RoPE at the query's position (Eq. 5's q, rotated once per
// step instead of once per key), scaled by 1/sqrt(128), in the layouts the decode kernels read.
#pragma once
#include "rkv_internal.h"

// One output channel c (0..127) of (virtual) query head h of sequence b.
// q~[b][h][c] = RoPE(q, q_pos)[c] / sqrt(128), angles in double (q_pos may lie beyond the table).
__device__ __forceinline__ void rkv_prep_q_one(const RkvView& v, const __half* __restrict__ q, const int* __restrict__ q_pos,
                                               int cur, float* __restrict__ qr, int share, int nq, int h, int b, int c) {
  // v.Hq counts virtual heads when nq > 1 (several query tokens, each at its own position)
  const RkvVHead vh = rkv_virtual_head(v, h, nq);
  // default position: the last cached token's, or one past it when the token being decoded is not in the cache yet (cur = 1)
  const int pos = q_pos ? q_pos[b * nq + vh.qi] : rkv_len(v, b) - 1 + cur;
  const size_t base = ((size_t)b * v.Hq + h) * RKV_D;                       // where the rotated query goes
  const size_t src = (((size_t)b * nq + vh.qi) * (v.Hq / nq) + vh.h) * RKV_D; // where the raw query is
  int j, partner;
  float sgn;
  if (v.rope_style == 0) {
    j = c & 63;
    partner = c ^ 64;
    sgn = c < 64 ? -1.f : 1.f;
  } else {
    j = c >> 1;
    partner = c ^ 1;
    sgn = (c & 1) ? 1.f : -1.f;
  }
  const float x = __half2float(q[src + c]), p = __half2float(q[src + partner]);
  // The matrix-core kernel keeps RoPE angles for the first of a lane's four consecutive tokens only
  // and rotates all four keys by them; the difference is put on the query side, which is exact:
  // <R(t + r) k, R(pos) q> = <R(t) k, R(pos - r) q>.  So it gets the query at positions pos - r,
  // r = 0..3, in its own layout:
  //   [b][rot group][rr / share][r][p 0..3][f / 4][n 0..15][f % 4],  f = (KV head a * share + rr % share) * 2 + half
  // (rr = which of the query heads sharing KV head a; one workgroup serves `share` of them; the 16
  // channel lanes n read consecutive 16-byte pieces, which LDS serves without bank conflicts) with
  // entry (n, p, half) = channel 16p + n + 64*half (interleaved pairs: 2 (16p + n) + half), pre-multiplied by 2/sqrt(rotation size)
  // (FP4 nibbles hold code/2; 1/sqrt(n) is the normalisation of Eq. 10).
  const int g = v.g, rep = v.Hq / v.Hkv;
  const int kvh = h / rep, rr = h - kvh * rep, rg = kvh / g, a = kvh - rg * g;
  float* qt = qr + (size_t)v.B * v.Hq * RKV_D;
  const int nn = v.rope_style ? (c >> 1) & 15 : c & 15, pp = v.rope_style ? (c >> 5) & 3 : (c >> 4) & 3, half = v.rope_style ? c & 1 : c >> 6;
  const int rrg = rr / share, rri = rr - rrg * share;
  const float lane_scale = 2.0f * rsqrtf((float)v.n);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    // angles: from the table (computed in double, stored as float) when the position lies inside
    // it - the usual case -, else computed here
    const int pr = pos - r;
    double sn, cs;
    if (pr >= 0 && pr < v.Tpad) {
      const float2 t = v.rope[(size_t)pr * 64 + j];
      cs = t.x;
      sn = t.y;
    } else {
      sincos((double)pr * pow((double)v.theta, -(double)j / 64.0), &sn, &cs);
    }
    const float val = (float)(((double)x * cs + (double)sgn * (double)p * sn) * 0.08838834764831845);
    if (r == 0) qr[base + c] = val;
    const int f = (a * share + rri) * 2 + half, nh2 = g * share / 2;
    size_t o = ((size_t)b * v.NRG + rg) * (rep / share) + rrg;
    o = (o * 4 + r) * 4 + pp;
    o = (o * nh2 + (f >> 2)) * 16 + nn;
    qt[o * 4 + (f & 3)] = val * lane_scale;
  }
}

// Write half, matrix-core kernel for gfx950: quantize-append for reorders that keep the 128-blocks
// of the rotated row (gid[c] == c/128), rot_heads 2 or 4, values quantized as given (v_rotate = 0).
//
// The grouped-head rotation of Sec. 4.2 is H_n = H_g (x) H_128 (Eq. 10).  The per-head factor H_128
// is a dense product of the fp16 keys with a +-1 matrix and runs on v_mfma_f32_16x16x32_f16: the
// products are exact, the accumulation is fp32 (measured: as accurate as a sequential fp32 sum).
// The operand roles are chosen so that the result lands in the physical K layout with no
// transpose: A = 16 rows of H_128, B = the keys of 16 tokens, so lane (token, q) of the result
// holds rows 4q..4q+3; the 16 rows of product p are channels 32q + 8(p>>1) + 4(p&1) + r, which makes
// the 32 channels a lane collects over 8 products exactly the 32 codes of its 16-byte piece of the
// K tile.  The H_g factor is a 2- or 4-point butterfly over the heads inside the lane; Eq. 6-9
// follow in registers.  Values take the vector path: lane = 2g consecutive channels of a token.
//
// One workgroup = (sequence, rotation group, slab of 32 token slots, role) so that every V dword
// (16 tokens of one channel), every K tile and every metadata row it touches is written whole.
// Three workgroups share a slab: one per K tile and one for the values, so that matrix-heavy and
// load-heavy workgroups share a compute unit, each kind holds only its own operands, and the
// register count leaves room for six waves per SIMD.
//   keys    the tile's fp16 rows are staged in LDS (whole-row loads); wave w computes dword
//           d = w&1 of every 16-byte piece (channels with bit 4 of the in-block index equal to d)
//           and of its 4 products per head the two with pp>>1 == w>>1, K = 128 each.
//   values  wave w: tokens 8w..8w+7.
#include "rkv_internal.h"
#include "rkv_quant.h"
#include "rkv_prep_q.h"

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v8h as_v8h(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  union { uint32_t u[4]; v8h h; } x;
  x.u[0] = a; x.u[1] = b; x.u[2] = c; x.u[3] = d;
  return x.h;
}
__device__ __forceinline__ uint32_t parity_mask(int x, uint32_t m) { return (__popc(x) & 1) ? m : 0u; }

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }
// packed fp16 min / max as single instructions (the builtin forms add a canonicalizing instruction
// per operand, which costs as much as the operation itself)
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// float minimum / maximum into LDS (ds_min_f32, ds_max_f32; nothing is returned)
typedef __attribute__((address_space(3))) float lds_float;
__device__ __forceinline__ void lds_fmin(float* p, float x) { __builtin_amdgcn_ds_fminf((lds_float*)p, x, 0, 0, false); }
__device__ __forceinline__ void lds_fmax(float* p, float x) { __builtin_amdgcn_ds_fmaxf((lds_float*)p, x, 0, 0, false); }
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}

// Eq. 8-9 for one block given its min and max, as quant_params but without IEEE divisions: the
// division by 3 (or 7, or 15) is a multiplication (error below 1.5 ulp of fp32, which can change the fp16 scale
// only within 2^-23 of a rounding boundary) and the reciprocal of the scale is v_rcp_f32 refined by
// one Newton step.
// meta8: FP8 E4M3 scale rounded up, INT8 zero-point.
// inv_qmax: 1 / (2^bits - 1) rounded to fp32.
__device__ __forceinline__ void quant_params_nodiv(float mn, float mx, float& s, float& zero, float& inv_s, bool meta8,
                                                   float inv_qmax = 0.33333334f) {
  const float raw = (mx - mn) * inv_qmax;
  if (meta8) {
    s = rkv_e4m3_round_up(raw);
    if (s == 0.0f) {
      s = rkv_e4m3_round_up(fabsf(mn));
      if (s == 0.0f) s = 1.0f;
    }
  } else {
    s = __half2float(__float2half_rn(raw));
    if (!(s <= 65504.0f)) s = 65504.0f;
    if (s == 0.0f) {
      s = __half2float(__float2half_rn(fabsf(mn)));
      if (!(s <= 65504.0f)) s = 65504.0f;
      if (s == 0.0f) s = 1.0f;
    }
  }
  const float r0 = __builtin_amdgcn_rcpf(s);
  inv_s = fmaf(fmaf(-s, r0, 1.0f), r0, r0);
  zero = -rintf(mn * inv_s);
  zero = meta8 ? fminf(fmaxf(zero, -128.0f), 127.0f) : fminf(fmaxf(zero, -2048.0f), 2048.0f);
}

// value of x in lane `src_lane` (the address operand is the lane number times 4)
__device__ __forceinline__ float lane_read(float x, int src_lane4) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane4, __float_as_int(x)));
}

// Eq. 6 with one FMA per element.  Adding 1.5 * 2^23 rounds to an integer, ties to even, as rintf;
// adding the (integer) zero-point in the same FMA keeps that rounding only if the constant added is
// even, so an odd zero-point is raised by one and the clamp bounds and the packing bias move with
// it.  `base` = 1.5 * 2^23 + (zero & 1); `add` = base + zero; codes are float_bits - bits(base).
__device__ __forceinline__ void fused_round_consts(float zero, float& base, float& add) {
  const float odd = (float)((int)zero & 1);
  base = 12582912.0f + odd;
  add = base + zero;
}

// bx, rg, b: the workgroup's place in the (3 x slabs, rotation groups, sequences) grid
// HB = 1: 3-bit codes, 7 steps; the third bits go to their plane, whose dwords take the bits of
// one matrix operand each (see the layout notes): the four key waves of a tile, and the four
// value waves of a slab, each contribute one bit in four to a dword of it.
// HB = 2: 4-bit codes.  The same arithmetic with 15 steps; the upper two bits of every code go to a
// second plane with the layout of the first (a second image in LDS, written the same way).
// XW: the reorder crosses 128-blocks inside the rotation group: a rotated channel's
// quantization block is looked up (gid), the minima and maxima are kept per quantization block,
// and every element takes the parameters of its own block.  Codes stay where they are - by
// rotated channel - so only the key role differs.
// SUB = 2 or 4: quantization groups of 64 or 32 channels (either metadata format; with XW the reorder may
// cross the heads of the rotation group, and a channel's block is any of its G * SUB, 4 bits in the table;
// else it stays inside the heads): a rotated 128-block holds SUB quantization blocks, block head * SUB + sub of
// the rotation group, and a rotated channel's sub-block follows from its reordered position (the
// same per-cache table, 2 bits per channel).  Keys: the minima and maxima of a token's G * SUB
// blocks are gathered with LDS float atomics (every element goes to its own block's pair), one
// thread per (token, block) then works out the parameters and leaves them in LDS, where every
// element fetches its block's.  Values are not reordered: a sub-block is 128 / SUB consecutive
// channels of a head, so the lane-exchange reduction simply stops earlier.
template <int G, int HB, bool XW = false, int SUB = 0>
__device__ __forceinline__ void append_mfma_body(const RkvView& v, const __half* __restrict__ kin, const __half* __restrict__ vin,
                                                 int n_new, int slab0, int bx, int rg, int b) {
  constexpr int PL = 2 * G;                    // value channels per lane
  constexpr int LPB = 128 / PL;                // lanes per 128-block in the value role
  constexpr int n = 128 * G;
  constexpr int ROW16 = 16 * G;                // 16-byte pieces per token row of the rotation group
  constexpr int STRIDE16 = ROW16 + 1;          // padded row: the matrix operand reads then touch every LDS bank once
  // key roles: the fp16 keys of one K tile, [16 tokens][STRIDE16] pieces, later overwritten by the two
  // halves of the tile image (2 x 128 G dwords); value role: per wave the partial V dwords of its 8
  // tokens, [wave][i][lane]
  // (with 4-bit codes: twice the images - 4 x 128 G and 8 x 64 PL dwords -, which still fit)
  static_assert(16 * STRIDE16 * 4 >= 8 * 64 * PL && 16 * STRIDE16 * 4 >= 4 * 128 * G, "the images of both planes fit the key tile's space");
  __shared__ __attribute__((aligned(16))) uint32_t lds[16 * STRIDE16 * 4 > 4 * 64 * PL ? 16 * STRIDE16 * 4 : 4 * 64 * PL];
  uint32_t* img = lds;
  uint32_t* imgh = lds + (PL == 8 ? 2048 : 1024);          // the upper plane's images: after 2 x 128 G (keys) or 4 x 64 PL (values) dwords
  constexpr bool HI = HB == 2, H1 = HB == 1;
  constexpr float QMAX = HI ? 15.0f : (H1 ? 7.0f : 3.0f), INV_QMAX = HI ? 0.06666667f : (H1 ? 0.14285715f : 0.33333334f);
  constexpr int NSB = SUB ? SUB : 1, GM = G * NSB;      // quantization blocks per 128-block, per rotation group
  // bits of a channel's block number in the per-cache table, and what is added to it: the sub-block of the
  // channel's own head (2 bits, plus head * SUB), or any block of the rotation group (2 bits; 4 with sub-blocks)
  constexpr int GB = (XW && SUB) ? 4 : 2;
  constexpr bool OWN = SUB != 0 || XW;          // every element looks up its own quantization block (keys)
  __shared__ uint32_t meta[32 * GM];
  __shared__ float2 s_mm[OWN ? 1 : 2][OWN ? 1 : 2][OWN ? 1 : 16][OWN ? 1 : G];   // [dword half][product pair][token][head] (min, max) of a quarter block
  // groups of 64 / 32: extrema of the tile [lane group q][token][block] (a copy per lane group, so
  // that the four lanes of a token never meet on one word; rows padded to an odd length, so that the
  // 64 lanes of an instruction spread over the banks) and [token][block] (reciprocal scale, constant
  // added, base) of Eq. 6
  constexpr int GMP = GM + 1;
  __shared__ float s_mn[OWN ? 64 * GMP : 1], s_mx[OWN ? 64 * GMP : 1];
  __shared__ float4 s_par[OWN ? 16 * GMP : 1];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: everything that depends only on it stays scalar
  const int role = bx % 3;                     // 0, 1: the keys of K tile 0 / 1 of a slab; 2: the slab's values
  // n_new: rows per sequence in kin and vin; sequence b holds len_b tokens and appends the first
  // n_b rows (all of them, at the common length, unless the view carries per-sequence arrays)
  const int len_b = rkv_len(v, b), n_b = v.nnew ? v.nnew[b] : n_new;
  const int slab = (v.lens ? (len_b >> 5) : slab0) + bx / 3;
  const int t_lo = len_b, t_hi = len_b + n_b;
  const int ts = slab * 32;
  if (ts >= t_hi || n_b <= 0) return;                 // the grid covers the longest append: nothing here for this sequence
  const int tau_first = max(0, t_lo - ts), tau_last = min(31, t_hi - 1 - ts);
  const size_t mrow = ((size_t)(b * v.NRG + rg) * v.Tpad + ts) * GM;    // metadata row of the slab's first token

  if (role < 2) {
    // ================================================================== keys of one tile
    const int ti = role;
    if (!((ts + 16 * ti < t_hi) && (ts + 16 * ti + 16 > t_lo))) return;   // no token of this call in the tile
    const int d = wave & 1, pph = wave >> 1;               // this wave: products pp = 2 pph + {0, 1} of dword half d
    const int col = lane & 15, q = lane >> 4;              // result: token `col` of the tile, rows 4q..4q+3
    const float rs = v.keys_rotated ? 1.0f : rsqrtf((float)n);   // rotated keys arrive normalised
    // the tile's keys go to LDS once, whole rows at a time (wave w: tokens 4w..4w+3)
    {
      constexpr int TPI = 64 / ROW16;                      // token rows per wave-wide 16-byte load
      uint4 st[4 / TPI];
#pragma unroll
      for (int k = 0; k < 4 / TPI; ++k) {
        // rows of tokens outside this call are replaced by a row inside it (their codes are never stored)
        const int tau = min(max(16 * ti + 4 * wave + TPI * k + lane / ROW16, tau_first), tau_last);
        const uint4* rowp = reinterpret_cast<const uint4*>(kin + ((size_t)b * n_new + (ts + tau - t_lo)) * v.E + (size_t)rg * n);
        st[k] = rkv_ld_stream(rowp + lane % ROW16);
      }
#pragma unroll
      for (int k = 0; k < 4 / TPI; ++k) {
        const int m = 4 * wave + TPI * k + lane / ROW16;
        reinterpret_cast<uint4*>(lds)[m * STRIDE16 + lane % ROW16] = st[k];
      }
    }
    if constexpr (OWN) {
      static_assert(16 * GM <= 256, "one thread per (token, block) of a tile");
      for (int i = tid; i < 64 * GMP; i += 256) {
        s_mn[i] = 3.0e38f;
        s_mx[i] = -3.0e38f;
      }
    }
    __syncthreads();
    v4f acc[G][2];
    if (v.keys_rotated) {
      // the keys already are what enters Eq. 6, in reordered order: the lane only picks up, for each
      // rotated channel it packs, the value at that channel's reordered position
      const __half* xh = reinterpret_cast<const __half*>(lds) + col * (STRIDE16 * 8);
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            const int chan = 128 * h + 32 * q + 8 * (2 * d + pph) + 4 * ppl + rr;
            acc[h][ppl][rr] = __half2float(xh[v.pinv[rg * n + chan] - rg * n]);
          }
    } else {
      const uint4* xrow = reinterpret_cast<const uint4*>(lds) + col * STRIDE16 + q;   // lane (token col, k-group q)
      // A operands: lane (row m = lane & 15, k-group kg = lane >> 4) holds H_128[channel][32ks + 8kg + i],
      // channel = 32(m>>2) + 8(2d + pph) + 4 ppl + (m&3); the sign is the parity of (channel & k),
      // which splits into (e & i), (v & kg) and ((m>>2) & ks)
      const int m = lane & 15, kg = lane >> 4, r = m & 3, qa = m >> 2;
      uint32_t base[2][4];
#pragma unroll
      for (int eb = 0; eb < 2; ++eb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int e = 4 * eb + r;
          base[eb][j] = (0x3C003C00u ^ parity_mask(e & (2 * j), 0x00008000u)) ^ parity_mask(e & (2 * j + 1), 0x80000000u);
        }
      const uint32_t maskv = parity_mask((2 * d + pph) & kg, 0x80008000u);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint32_t mk = maskv ^ parity_mask(qa & ks, 0x80008000u);
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl) {
          const v8h a = as_v8h(base[ppl][0] ^ mk, base[ppl][1] ^ mk, base[ppl][2] ^ mk, base[ppl][3] ^ mk);
#pragma unroll
          for (int h = 0; h < G; ++h) {
            const uint4 xb = xrow[16 * h + 4 * ks];                      // keys 32ks + 8q .. +7 of head h
            const v8h x = as_v8h(xb.x, xb.y, xb.z, xb.w);
            const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
            acc[h][ppl] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, x, ks == 0 ? zero4 : acc[h][ppl], 0, 0, 0);
          }
        }
      }
      // H_g over the heads (Sylvester order: the head index is the high part of the rotated channel)
#pragma unroll
      for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          if constexpr (G == 4) {
            const float x0 = acc[0][ppl][rr], x1 = acc[1][ppl][rr], x2 = acc[2][ppl][rr], x3 = acc[3][ppl][rr];
            const float a0 = x0 + x1, a1 = x0 - x1, a2 = x2 + x3, a3 = x2 - x3;
            acc[0][ppl][rr] = a0 + a2; acc[1][ppl][rr] = a1 + a3; acc[2][ppl][rr] = a0 - a2; acc[3][ppl][rr] = a1 - a3;
          } else {
            const float x0 = acc[0][ppl][rr], x1 = acc[1][ppl][rr];
            acc[0][ppl][rr] = x0 + x1; acc[1][ppl][rr] = x0 - x1;
          }
        }
    }
    // cross-block variant: quantization block (within the group) of each of the lane's channels, 2 bits each
    uint32_t gsel[G];
    if constexpr (OWN) {
      // the block of each of the lane's channels, 2 bits each (a per-cache table written by rkv_set_perm):
      // the sub-block inside the head (groups of 64 / 32), or the quantization block of the rotation group
      // (a reorder across blocks: any head's channel may belong to it)
#pragma unroll
      for (int h = 0; h < G; ++h) gsel[h] = v.xgsel[(((size_t)rg * 4 + wave) * 4 + q) * G + h];
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            const int blk = (q * 16 + col) * GMP + ((SUB && !XW) ? h * SUB : 0) + (int)((gsel[h] >> (GB * (4 * ppl + rr))) & ((1u << GB) - 1u));
            lds_fmin(&s_mn[blk], acc[h][ppl][rr]);
            lds_fmax(&s_mx[blk], acc[h][ppl][rr]);
          }
    } else {
      // min / max of this wave's quarter of every block: 8 values in the lane, then the four q groups
#pragma unroll
      for (int a = 0; a < G; ++a) {
        float mn = acc[a][0][0], mx = mn;
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            mn = fminf(mn, acc[a][ppl][rr]);
            mx = fmaxf(mx, acc[a][ppl][rr]);
          }
        mn = fminf(mn, __shfl_xor(mn, 16)); mx = fmaxf(mx, __shfl_xor(mx, 16));
        mn = fminf(mn, __shfl_xor(mn, 32)); mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (q == 0) s_mm[d][pph][col][a] = make_float2(mn, mx);
      }
    }
    __syncthreads();
    if constexpr (OWN) {
      // Eq. 8-9 per (token, block), one thread each; Eq. 6 with each element's own block's parameters
      if (tid < 16 * GM) {
        const int tk = tid / GM, bk = tid - tk * GM;
        float mn = s_mn[tk * GMP + bk], mx = s_mx[tk * GMP + bk];
#pragma unroll
        for (int qq = 1; qq < 4; ++qq) {
          mn = fminf(mn, s_mn[(qq * 16 + tk) * GMP + bk]);
          mx = fmaxf(mx, s_mx[(qq * 16 + tk) * GMP + bk]);
        }
        float sc, zero_b, inv, base_b, add_b;
        quant_params_nodiv(mn * rs, mx * rs, sc, zero_b, inv, v.meta8, INV_QMAX);
        fused_round_consts(zero_b, base_b, add_b);
        s_par[tk * GMP + bk] = make_float4(inv * rs, add_b, base_b, 0.f);
        meta[tid] = rkv_pack_meta(sc, zero_b);
      }
      __syncthreads();
#pragma unroll
      for (int a = 0; a < G; ++a) {
        uint32_t word = 0;
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            const float4 pr = s_par[col * GMP + ((SUB && !XW) ? a * SUB : 0) + (int)((gsel[a] >> (GB * (4 * ppl + rr))) & ((1u << GB) - 1u))];
            const float c = __builtin_amdgcn_fmed3f(fmaf(acc[a][ppl][rr], pr.x, pr.y), pr.z, pr.z + QMAX);
            word += (__float_as_uint(c) - __float_as_uint(pr.z)) << (16 * ppl + 4 * rr);
          }
        // (a code per nibble; wider codes: the bits above the low two go to their plane, as below)
        const int io = pph * (128 * G) + ((((a >> 1) * 4 + q) * 16 + col) * 4) + (a & 1) * 2 + d;
        if constexpr (HI) {
          img[io] = (word & 0x33333333u) << (2 * pph);
          imgh[io] = ((word >> 2) & 0x33333333u) << (2 * pph);
        } else if constexpr (H1) {
          img[io] = (word & 0x33333333u) << (2 * pph);
          imgh[(2 * pph + d) * (64 * G) + ((io - pph * (128 * G) - d) >> 1)] = ((word >> 2) & 0x11111111u) << (2 * d + pph);
        } else {
          img[io] = word << (2 * pph);
        }
      }
    } else {
      // Eq. 6-9 on y = (raw rotation) / sqrt(n): min and max scale exactly (rounding is monotone),
      // the elements take the factor inside the reciprocal scale.  Lane group q works out the
      // parameters of head q & (G-1) for its token; the others fetch them with lane exchanges.
      const int ah = q & (G - 1);
      const float2 m0 = s_mm[0][0][col][ah], m1 = s_mm[0][1][col][ah], m2 = s_mm[1][0][col][ah], m3 = s_mm[1][1][col][ah];
      float sc, zero_h, inv;
      quant_params_nodiv(fminf(fminf(m0.x, m1.x), fminf(m2.x, m3.x)) * rs, fmaxf(fmaxf(m0.y, m1.y), fmaxf(m2.y, m3.y)) * rs, sc,
                         zero_h, inv, v.meta8, INV_QMAX);
      const float inv2_h = inv * rs;
      if (wave == 0 && q < G) meta[col * G + ah] = rkv_pack_meta(sc, zero_h);
      float base_h, add_h;
      fused_round_consts(zero_h, base_h, add_h);
      {
#pragma unroll
      for (int a = 0; a < G; ++a) {
        const int src4 = 4 * (col + 16 * a);
        const float inv2 = lane_read(inv2_h, src4), add = lane_read(add_h, src4), base = lane_read(base_h, src4);
        const float top = base + QMAX;
        uint32_t word = 0;
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            const float c = __builtin_amdgcn_fmed3f(fmaf(acc[a][ppl][rr], inv2, add), base, top);
            word += __float_as_uint(c) << (16 * ppl + 4 * rr);
          }
        // the 8 float bit patterns add up to bits(base) * 0x11111111 plus the packed codes, mod 2^32
        // (a code per nibble: 4-bit codes just fit);
        // this wave's codes sit 2 pph bits up in the dword it shares with the wave of the other pph
        word -= __float_as_uint(base) * 0x11111111u;
        const int io = pph * (128 * G) + ((((a >> 1) * 4 + q) * 16 + col) * 4) + (a & 1) * 2 + d;
        if constexpr (HI) {
          img[io] = (word & 0x33333333u) << (2 * pph);
          imgh[io] = ((word >> 2) & 0x33333333u) << (2 * pph);
        } else if constexpr (H1) {
          // code m = 2 j + pph of dword d of the pair: bit 4 j + 2 d + pph of the pair's dword of third bits
          img[io] = (word & 0x33333333u) << (2 * pph);
          imgh[(2 * pph + d) * (64 * G) + ((io - pph * (128 * G) - d) >> 1)] = ((word >> 2) & 0x11111111u) << (2 * d + pph);
        } else {
          img[io] = word << (2 * pph);
        }
      }
      }
    }
    __syncthreads();
    // the K tile: every 16-byte piece belongs to one token
#pragma unroll
    for (int k = 0; k < (128 * G + 255) / 256; ++k) {
      const int off = tid + 256 * k;
      if (off < 128 * G) {
        const int t = ts + ti * 16 + rkv_k_tile_token(G, off);
        if (t >= t_lo && t < t_hi) {
          rkv_st_stream(&v.kc[rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off], img[off] | img[128 * G + off]);
          if constexpr (HI) rkv_st_stream(&v.kh[rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off], imgh[off] | imgh[128 * G + off]);
          if constexpr (H1) {
            if (!(off & 1)) {
              const int o2 = off >> 1;
              rkv_st_stream(&v.kh[(rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off) >> 1],
                            imgh[o2] | imgh[64 * G + o2] | imgh[128 * G + o2] | imgh[192 * G + o2]);
            }
          }
        }
      }
    }
    for (int i = tid; i < 16 * GM; i += 256) {
      const int tau = 16 * ti + i / GM;
      if (tau >= tau_first && tau <= tau_last) rkv_store_meta_word(v, v.km, mrow + 16 * ti * GM + i, meta[i]);
    }
    return;
  }

  // ==================================================================== values
  // slots of this slab that belong to tokens outside this call are kept
  uint32_t keep[2] = {0, 0};
  for (int tau = 0; tau < 32; ++tau) {
    const int t = ts + tau;
    if (!(t >= t_lo && t < t_hi)) keep[tau >> 4] |= 3u << rkv_v_shift(tau);
  }
  const size_t vbase = rkv_v_slabbase(v, b, rg, slab);
  uint32_t oldv[G], oldvh[HB ? G : 1];
#pragma unroll
  for (int k = 0; k < G; ++k) oldv[k] = 0;
  if constexpr (HB != 0) {
#pragma unroll
    for (int k = 0; k < G; ++k) oldvh[k] = 0;
  }
  // third bits (HB = 1): token tau of the slab sits at bit 4 (tau & 7) + (tau >> 3) of a channel's dword
  uint32_t keeph = 0;
  if constexpr (H1) {
    for (int tau = 0; tau < 32; ++tau) {
      const int t = ts + tau;
      if (!(t >= t_lo && t < t_hi)) keeph |= 1u << (4 * (tau & 7) + (tau >> 3));
    }
  }
  if (keep[0] | keep[1]) {
#pragma unroll
    for (int k = 0; k < G; ++k) oldv[k] = v.vc[vbase + tid + 256 * k];
    if constexpr (HI) {
#pragma unroll
      for (int k = 0; k < G; ++k) oldvh[k] = v.vh[vbase + tid + 256 * k];
    }
    if constexpr (H1) {
#pragma unroll
      for (int k = 0; k < G; ++k) oldvh[k] = v.vh[(vbase + tid + 256 * k) >> 1];
    }
  }
  uint32_t vraw[8][PL / 2];                                // rows of this wave's 8 tokens: lane = PL consecutive channels
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    // a token outside this call is replaced by one inside it (its codes are never used)
    const int tau = min(max(8 * wave + k, tau_first), tau_last);
    const uint32_t* p = reinterpret_cast<const uint32_t*>(vin + ((size_t)b * n_new + (ts + tau - t_lo)) * v.E + (size_t)rg * n + PL * lane);
    if constexpr (PL == 8) {
      const uint4 u = rkv_ld_stream(reinterpret_cast<const uint4*>(p));
      vraw[k][0] = u.x; vraw[k][1] = u.y; vraw[k][2] = u.z; vraw[k][3] = u.w;
    } else {
      const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(p));
      vraw[k][0] = u.x; vraw[k][1] = u.y;
    }
  }
  // min and max of a block travel together as one packed pair (min, -max), so that one packed
  // fp16 minimum per step reduces both (fp16 min/max of fp16 inputs is exact)
  constexpr int LPS = LPB / NSB;                           // lanes per quantization block
  static_assert(LPS >= 4, "a quantization block spans at least four lanes");
  const int blk = lane / LPS;                              // quantization block (KV head, or a sub-block of it) of this lane's channels
  uint32_t mm[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    uint32_t lo = vraw[k][0], hi = vraw[k][0];
#pragma unroll
    for (int i = 1; i < PL / 2; ++i) {
      lo = pk_min(lo, vraw[k][i]);
      hi = pk_max(hi, vraw[k][i]);
    }
    lo = pk_min(lo, __builtin_amdgcn_perm(lo, lo, 0x01000302u));          // both halves = min of the lane's channels
    hi = pk_max(hi, __builtin_amdgcn_perm(hi, hi, 0x01000302u));
    uint32_t p = __builtin_amdgcn_perm(hi, lo, 0x05040100u) ^ 0x80000000u;   // (min, -max)
    p = pk_min(p, dpp_u<0xB1>(p));                                        // quad_perm [1,0,3,2]
    p = pk_min(p, dpp_u<0x4E>(p));                                        // quad_perm [2,3,0,1]
    if constexpr (LPS >= 8) p = pk_min(p, dpp_u<0x141>(p));               // row_half_mirror
    if constexpr (LPS >= 16) p = pk_min(p, dpp_u<0x140>(p));              // row_mirror
    if constexpr (LPS == 32) p = pk_min(p, (uint32_t)__shfl_xor((int)p, 16));
    mm[k] = p;
  }
  // lane j of every block works out the parameters of token 8 wave + j (blocks of four lanes: of
  // tokens j and j + 4, in two rounds); the others fetch them
  constexpr int NRND = LPS >= 8 ? 1 : 8 / LPS, TPR = 8 / NRND;   // rounds, tokens per round
  float inv_v[NRND], base_v[NRND], add_v[NRND];
#pragma unroll
  for (int r = 0; r < NRND; ++r) {
    uint32_t mine = mm[TPR * r];
#pragma unroll
    for (int k = 1; k < TPR; ++k) mine = ((lane & (LPS - 1)) == k) ? mm[TPR * r + k] : mine;
    float sc_v, zero_v;
    const h2 pr = as_h2(mine);
    quant_params_nodiv((float)pr[0], -(float)pr[1], sc_v, zero_v, inv_v[r], v.meta8, INV_QMAX);
    fused_round_consts(zero_v, base_v[r], add_v[r]);
    const int tau = 8 * wave + TPR * r + (lane & (LPS - 1));
    if ((lane & (LPS - 1)) < TPR) meta[tau * GM + blk] = rkv_pack_meta(sc_v, zero_v);
  }
  uint32_t vword[PL], vwordh[HB ? PL : 1];
#pragma unroll
  for (int i = 0; i < PL; ++i) vword[i] = 0;
  if constexpr (HB != 0) {
#pragma unroll
    for (int i = 0; i < PL; ++i) vwordh[i] = 0;
  }
  uint32_t bias = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int tau = 8 * wave + k;
    if (tau < tau_first || tau > tau_last) continue;       // wave-uniform
    const int src4 = 4 * ((lane & ~(LPS - 1)) | (k % TPR));
    const float inv = lane_read(inv_v[k / TPR], src4), add = lane_read(add_v[k / TPR], src4), base = lane_read(base_v[k / TPR], src4);
    const float top = base + QMAX;
    const int sh = rkv_v_shift(tau);
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      const h2 pr = as_h2(vraw[k][i >> 1]);
      const float c = __builtin_amdgcn_fmed3f(fmaf((float)pr[i & 1], inv, add), base, top);
      if constexpr (HI) {
        const uint32_t code = __float_as_uint(c) - __float_as_uint(base);
        vword[i] += (code & 3u) << sh;
        vwordh[i] += (code >> 2) << sh;
      } else if constexpr (H1) {
        const uint32_t code = __float_as_uint(c) - __float_as_uint(base);
        vword[i] += (code & 3u) << sh;
        vwordh[i] += (code >> 2) << (4 * k + wave);        // tau = 8 wave + k
      } else {
        vword[i] += __float_as_uint(c) << sh;
      }
    }
    if constexpr (HB == 0) bias += __float_as_uint(base) << sh;
  }
#pragma unroll
  for (int i = 0; i < PL; ++i) img[(wave * PL + i) * 64 + lane] = vword[i] - bias;
  if constexpr (HB != 0) {
#pragma unroll
    for (int i = 0; i < PL; ++i) imgh[(wave * PL + i) * 64 + lane] = vwordh[i];
  }
  __syncthreads();
  // V slab: dword idx = (((w*G + hh)*16 + nn)*2 + ct)*2 + d, channel c = 128hh + 32w + 16ct + nn;
  // waves 2d and 2d+1 hold the two halves of its 16 token slots
#pragma unroll
  for (int k = 0; k < G; ++k) {
    const int idx = tid + 256 * k;
    const int d = idx & 1, ct = (idx >> 1) & 1, nn = (idx >> 2) & 15, rest = idx >> 6;
    const int hh = rest % G, w = rest / G;
    const int c = 128 * hh + 32 * w + 16 * ct + nn;
    const int ln = c / PL, i = c - ln * PL;
    uint32_t word = img[((2 * d) * PL + i) * 64 + ln] | img[((2 * d + 1) * PL + i) * 64 + ln];
    if (keep[d]) word |= oldv[k] & keep[d];
    if (keep[d] != 0xffffffffu) rkv_st_stream(&v.vc[vbase + idx], word);
    if constexpr (HI) {
      word = imgh[((2 * d) * PL + i) * 64 + ln] | imgh[((2 * d + 1) * PL + i) * 64 + ln];
      if (keep[d]) word |= oldvh[k] & keep[d];
      if (keep[d] != 0xffffffffu) rkv_st_stream(&v.vh[vbase + idx], word);
    }
    if constexpr (H1) {
      if (d == 0) {                                         // one dword of third bits per pair (d = 0, 1): all four waves' tokens
        word = imgh[(0 * PL + i) * 64 + ln] | imgh[(1 * PL + i) * 64 + ln] | imgh[(2 * PL + i) * 64 + ln] | imgh[(3 * PL + i) * 64 + ln];
        if (keeph) word |= oldvh[k] & keeph;
        rkv_st_stream(&v.vh[(vbase + idx) >> 1], word);
      }
    }
  }
  for (int i = tid; i < 32 * GM; i += 256) {
    const int tau = i / GM;
    if (tau >= tau_first && tau <= tau_last) rkv_store_meta_word(v, v.vm, mrow + i, meta[i]);
  }
}

template <int G, int HB, bool XW = false, int SUB = 0>
__global__ void __launch_bounds__(256, (HB || XW || SUB) ? 4 : 6) k_append_mfma(RkvView v, const __half* __restrict__ kin, const __half* __restrict__ vin,
                                                                      int n_new, int slab0) {
  append_mfma_body<G, HB, XW, SUB>(v, kin, vin, n_new, slab0, blockIdx.x, blockIdx.y, blockIdx.z);
}

// the value role alone (grid x = slabs): the keys of a reorder over the whole row have a kernel of their own
template <int G, int HB = 0, int SUB = 0>
__global__ void __launch_bounds__(256, (HB || SUB) ? 4 : 6) k_append_values(RkvView v, const __half* __restrict__ vin, int n_new, int slab0) {
  append_mfma_body<G, HB, false, SUB>(v, nullptr, vin, n_new, slab0, 3 * blockIdx.x + 2, blockIdx.y, blockIdx.z);
}

// Keys under a reorder over the whole token row (perm_span = n_kv_heads * 128, Alg. 1 as printed;
// HB as in k_append_mfma: codes of 3 or 4 bits, the bits above the low two to their plane).  A rotated channel then belongs to any of the row's E / quant_group
// quantization blocks, so a block's minimum and maximum (Eq. 8-9) need the rotated values of all
// rotation groups of the token.  One workgroup = (sequence, tile of 16 tokens) takes the groups one
// after the other, twice: the first pass rotates (H_128 on fp16 matrix products, H_g in the lane,
// as k_append_mfma) and gathers the extrema of the tile's 16 x E/128 blocks with LDS float atomics;
// one thread per (token, block) then works out the parameters, stores the metadata and leaves
// (reciprocal scale, constant added, base) in LDS; the second pass rotates again - the tile's keys
// come back from the last-level cache - and quantizes every element with its own block's
// parameters.  Codes stay where they are, by rotated channel.  The quantization block of each of a
// lane's channels comes from a per-cache table of bytes (xgid8, written by rkv_set_perm).
// dynamic LDS: [NG][16 tokens] float minima, the same of maxima, [NG][16] float4 parameters (block-major: the 16
// tokens of a row of lanes, which share their channels and hence their blocks, touch 16 different LDS banks).
template <int G, int HB = 0>
__global__ void __launch_bounds__(256, 3) k_append_row_keys(RkvView v, const __half* __restrict__ kin, int n_new, int slab0) {
  constexpr int n = 128 * G;
  constexpr bool HI = HB == 2, H1 = HB == 1;
  constexpr float QMAX = HI ? 15.0f : (H1 ? 7.0f : 3.0f), INV_QMAX = HI ? 0.06666667f : (H1 ? 0.14285715f : 0.33333334f);
  constexpr int ROW16 = 16 * G, STRIDE16 = ROW16 + 1;
  __shared__ __attribute__((aligned(16))) uint32_t lds[16 * STRIDE16 * 4];
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_row[];
  const int NG = v.NG, NGP = NG | 1;           // the row's quantization blocks (of 128, 64 or 32 positions); the allocation counts NGP
  float* s_mn = reinterpret_cast<float*>(dyn_row);
  float* s_mx = s_mn + 16 * NGP;
  float4* s_par = reinterpret_cast<float4*>(dyn_row + (size_t)2 * 16 * NGP * 4);      // (128 NGP bytes in: 16-byte aligned)
  __shared__ uint32_t img[2 * 128 * G];        // the tile image of one rotation group, in two halves (see k_append_mfma)
  __shared__ uint32_t imgh[HB ? 2 * 128 * G : 1];   // the upper plane's: two halves (4-bit codes) or four quarter-size pieces (3-bit)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y, ti = blockIdx.x & 1;
  const int len_b = rkv_len(v, b), n_b = v.nnew ? v.nnew[b] : n_new;
  const int slab = (v.lens ? (len_b >> 5) : slab0) + (blockIdx.x >> 1);
  const int t_lo = len_b, t_hi = len_b + n_b;
  const int ts = slab * 32;
  if (ts >= t_hi || n_b <= 0) return;
  if (!((ts + 16 * ti < t_hi) && (ts + 16 * ti + 16 > t_lo))) return;   // no token of this call in the tile
  const int tau_first = max(0, t_lo - ts), tau_last = min(31, t_hi - 1 - ts);
  const int d = wave & 1, pph = wave >> 1;                 // this wave: products pp = 2 pph + {0, 1} of dword half d
  const int col = lane & 15, q = lane >> 4;                // result: token `col` of the tile, rows 4q..4q+3
  const float rs = rsqrtf((float)n);
  // A operands (see k_append_mfma): lane (row m, k-group kg) holds H_128[channel][32 ks + 8 kg + i]
  const int m = lane & 15, kg = lane >> 4, r = m & 3, qa = m >> 2;
  uint32_t base[2][4];
#pragma unroll
  for (int eb = 0; eb < 2; ++eb)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = 4 * eb + r;
      base[eb][j] = (0x3C003C00u ^ parity_mask(e & (2 * j), 0x00008000u)) ^ parity_mask(e & (2 * j + 1), 0x80000000u);
    }
  const uint32_t maskv = parity_mask((2 * d + pph) & kg, 0x80008000u);

  constexpr int TPI = 64 / ROW16;                        // token rows per wave-wide 16-byte load
  // the tile's rows of one rotation group (wave w: tokens 4w..4w+3), requested one group ahead and
  // held in registers meanwhile (named registers: as an array they were given a place in memory)
  uint4 st0 = make_uint4(0, 0, 0, 0), st1 = st0, st2 = st0, st3 = st0;
  auto row_ptr = [&](int rg, int k) __attribute__((always_inline)) {
    // rows of tokens outside this call are replaced by a row inside it (their codes are never stored)
    const int tau = min(max(16 * ti + 4 * wave + TPI * k + lane / ROW16, tau_first), tau_last);
    return reinterpret_cast<const uint4*>(kin + ((size_t)b * n_new + (ts + tau - t_lo)) * v.E + (size_t)rg * n) + lane % ROW16;
  };
#define RKV_ROW_REQUEST(rg_)                    \
  do {                                          \
    st0 = *row_ptr(rg_, 0);                     \
    st1 = *row_ptr(rg_, 1);                     \
    if constexpr (TPI == 1) {                   \
      st2 = *row_ptr(rg_, 2);                   \
      st3 = *row_ptr(rg_, 3);                   \
    }                                           \
  } while (0)
#define RKV_ROW_DEPOSIT()                                                                             \
  do {                                                                                                \
    uint4* rows_ = reinterpret_cast<uint4*>(lds);                                                     \
    rows_[(4 * wave + TPI * 0 + lane / ROW16) * STRIDE16 + lane % ROW16] = st0;                       \
    rows_[(4 * wave + TPI * 1 + lane / ROW16) * STRIDE16 + lane % ROW16] = st1;                       \
    if constexpr (TPI == 1) {                                                                         \
      rows_[(4 * wave + 2 + lane / ROW16) * STRIDE16 + lane % ROW16] = st2;                           \
      rows_[(4 * wave + 3 + lane / ROW16) * STRIDE16 + lane % ROW16] = st3;                           \
    }                                                                                                 \
  } while (0)
  auto rotate = [&](v4f (&acc)[G][2]) __attribute__((always_inline)) {
    const uint4* xrow = reinterpret_cast<const uint4*>(lds) + col * STRIDE16 + q;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const uint32_t mk = maskv ^ parity_mask(qa & ks, 0x80008000u);
#pragma unroll
      for (int ppl = 0; ppl < 2; ++ppl) {
        const v8h a = as_v8h(base[ppl][0] ^ mk, base[ppl][1] ^ mk, base[ppl][2] ^ mk, base[ppl][3] ^ mk);
#pragma unroll
        for (int h = 0; h < G; ++h) {
          const uint4 xb = xrow[16 * h + 4 * ks];
          const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
          acc[h][ppl] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, as_v8h(xb.x, xb.y, xb.z, xb.w), ks == 0 ? zero4 : acc[h][ppl], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        if constexpr (G == 4) {
          const float x0 = acc[0][ppl][rr], x1 = acc[1][ppl][rr], x2 = acc[2][ppl][rr], x3 = acc[3][ppl][rr];
          const float a0 = x0 + x1, a1 = x0 - x1, a2 = x2 + x3, a3 = x2 - x3;
          acc[0][ppl][rr] = a0 + a2; acc[1][ppl][rr] = a1 + a3; acc[2][ppl][rr] = a0 - a2; acc[3][ppl][rr] = a1 - a3;
        } else {
          const float x0 = acc[0][ppl][rr], x1 = acc[1][ppl][rr];
          acc[0][ppl][rr] = x0 + x1; acc[1][ppl][rr] = x0 - x1;
        }
      }
  };
  // quantization blocks (of the row) of the lane's eight channels of head h, one byte each (element 4 ppl + rr)
  auto blocks_of = [&](int rg, int h) __attribute__((always_inline)) { return v.xgid8[(((size_t)rg * 4 + wave) * 4 + q) * G + h]; };

  for (int i = tid; i < 16 * NGP; i += 256) {
    s_mn[i] = 3.0e38f;
    s_mx[i] = -3.0e38f;
  }
  // ---- first pass: extrema
  RKV_ROW_REQUEST(0);
  for (int rg = 0; rg < v.NRG; ++rg) {
    RKV_ROW_DEPOSIT();
    __syncthreads();
    if (rg + 1 < v.NRG) RKV_ROW_REQUEST(rg + 1);
    v4f acc[G][2];
    rotate(acc);
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const uint2 gb = blocks_of(rg, h);
#pragma unroll
      for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int blk = (int)(((ppl ? gb.y : gb.x) >> (8 * rr)) & 0xffu) * 16 + col;
          lds_fmin(&s_mn[blk], acc[h][ppl][rr]);
          lds_fmax(&s_mx[blk], acc[h][ppl][rr]);
        }
    }
    __syncthreads();                                       // the rows are read: the next group's may come
  }
  // ---- Eq. 8-9 per (token, block)
  RKV_ROW_REQUEST(0);
  for (int e = tid; e < 16 * NG; e += 256) {
    const int tk = e & 15, bk = e >> 4;
    float sc, zero_b, inv, base_b, add_b;
    quant_params_nodiv(s_mn[e] * rs, s_mx[e] * rs, sc, zero_b, inv, v.meta8, INV_QMAX);
    fused_round_consts(zero_b, base_b, add_b);
    s_par[e] = make_float4(inv * rs, add_b, base_b, 0.f);
    const int tau = 16 * ti + tk;
    if (tau >= tau_first && tau <= tau_last) rkv_store_meta(v, v.km, rkv_meta_index(v, b, ts + tau, bk), sc, zero_b);
  }
  // ---- second pass: Eq. 6 with each element's own block's parameters
  for (int rg = 0; rg < v.NRG; ++rg) {
    RKV_ROW_DEPOSIT();
    __syncthreads();                                       // (also: the parameters are complete)
    if (rg + 1 < v.NRG) RKV_ROW_REQUEST(rg + 1);
    v4f acc[G][2];
    rotate(acc);
    uint32_t words[G];
#pragma unroll
    for (int a = 0; a < G; ++a) {
      const uint2 gb = blocks_of(rg, a);
      uint32_t word = 0;
#pragma unroll
      for (int ppl = 0; ppl < 2; ++ppl)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const float4 pr = s_par[(int)(((ppl ? gb.y : gb.x) >> (8 * rr)) & 0xffu) * 16 + col];
          const float c = __builtin_amdgcn_fmed3f(fmaf(acc[a][ppl][rr], pr.x, pr.y), pr.z, pr.z + QMAX);
          word += (__float_as_uint(c) - __float_as_uint(pr.z)) << (16 * ppl + 4 * rr);
        }
      words[a] = word;                                     // a code per nibble
    }
    // (the previous group's image was stored before this group's first barrier)
#pragma unroll
    for (int a = 0; a < G; ++a) {
      const int io = pph * (128 * G) + ((((a >> 1) * 4 + q) * 16 + col) * 4) + (a & 1) * 2 + d;
      if constexpr (HI) {
        img[io] = (words[a] & 0x33333333u) << (2 * pph);
        imgh[io] = ((words[a] >> 2) & 0x33333333u) << (2 * pph);
      } else if constexpr (H1) {
        img[io] = (words[a] & 0x33333333u) << (2 * pph);
        imgh[(2 * pph + d) * (64 * G) + ((io - pph * (128 * G) - d) >> 1)] = ((words[a] >> 2) & 0x11111111u) << (2 * d + pph);
      } else {
        img[io] = words[a] << (2 * pph);
      }
    }
    __syncthreads();                                       // the image is complete; the rows are read: the next group's may come
#pragma unroll
    for (int k = 0; k < (128 * G + 255) / 256; ++k) {
      const int off = tid + 256 * k;
      if (off < 128 * G) {
        const int t = ts + ti * 16 + rkv_k_tile_token(G, off);
        if (t >= t_lo && t < t_hi) {
          rkv_st_stream(&v.kc[rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off], img[off] | img[128 * G + off]);
          if constexpr (HI) rkv_st_stream(&v.kh[rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off], imgh[off] | imgh[128 * G + off]);
          if constexpr (H1) {
            if (!(off & 1)) {
              const int o2 = off >> 1;
              rkv_st_stream(&v.kh[(rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off) >> 1],
                            imgh[o2] | imgh[64 * G + o2] | imgh[128 * G + o2] | imgh[192 * G + o2]);
            }
          }
        }
      }
    }
  }
#undef RKV_ROW_REQUEST
#undef RKV_ROW_DEPOSIT
}

// One decode step's write half and query preparation in one launch: the first 3 * n_slabs
// workgroups of a (rotation group, sequence) append the step's token as k_append_mfma does, the
// rest prepare that rotation group's query heads (two heads per workgroup) for the decode kernel,
// which saves a launch of its own for a few microseconds of work.  The query's default position
// is the appended token's: one past the last token the view knows of.
template <int G, int HB, bool XW = false, int SUB = 0>
__global__ void __launch_bounds__(256, 4) k_step_mfma(RkvView v, const __half* __restrict__ kin, const __half* __restrict__ vin,
                                                   int slab0, int n_append_blocks, const __half* __restrict__ q,
                                                   const int* __restrict__ q_pos, float* __restrict__ qr, int share) {
  if ((int)blockIdx.x < n_append_blocks) {
    append_mfma_body<G, HB, XW, SUB>(v, kin, vin, 1, slab0, blockIdx.x, blockIdx.y, blockIdx.z);
    return;
  }
  const int rep = v.Hq / v.Hkv;
  const int h = blockIdx.y * G * rep + 2 * ((int)blockIdx.x - n_append_blocks) + (threadIdx.x >> 7);
  rkv_prep_q_one(v, q, q_pos, 1, qr, share, 1, h, blockIdx.z, threadIdx.x & 127);
}

// a reorder over the whole row: k_append_row_keys + k_append_values
static bool append_row(const rkv_cache* c) {
  const RkvView& v = c->v;
  // (a block's number is a byte in the kernel's table; its dynamic LDS beside 26 KB of static)
  return !c->blocks_aligned && !c->in_groups && (v.g == 2 || v.g == 4) && v.v_rotate == 0 &&
         !c->cfg.keys_rotated && v.NG <= 255 && (size_t)384 * (v.NG | 1) <= 120 * 1024;
}
int rkv_append_mfma_variant(const rkv_cache* c) {
  return append_row(c) ? RKV_KERNEL_MFMA_ROW : c->v.qg != 128 ? RKV_KERNEL_MFMA_SUB : c->blocks_aligned ? RKV_KERNEL_MFMA : RKV_KERNEL_MFMA_CROSS;
}

bool rkv_append_mfma_supported(const rkv_cache* c) {
  const RkvView& v = c->v;
  if (append_row(c)) return true;
  // 2-bit codes, or wider ones (a second plane); a reorder across 128-blocks inside the rotation groups
  // with keys in the original basis
  if (!c->blocks_aligned && !(c->in_groups && !c->cfg.keys_rotated)) return false;
  // groups of 64 / 32: a reorder inside the heads (codes of 2, 3 or 4 bits)
  if (v.qg != 128 && !c->blocks_aligned && !c->in_groups) return false;   // (or inside the rotation groups)
  return (v.g == 2 || v.g == 4) && v.v_rotate == 0;
}

// max_slabs: most 32-token slabs any sequence's new tokens touch, or 0 to work it out for n_new
// tokens per sequence
int rkv_launch_append_mfma(rkv_cache* c, const __half* k, const __half* vv, int n_new, int max_slabs, hipStream_t s) {
  const RkvView& v = c->v;
  if (!rkv_append_mfma_supported(c)) return RKV_EINVAL;
  const int slab0 = v.len >> 5, slab1 = (v.len + n_new - 1) >> 5;
  if (max_slabs <= 0) {
    max_slabs = slab1 - slab0 + 1;
    if (c->ragged)
      for (int b = 0; b < v.B; ++b) {
        const int sl = ((c->hlens[b] + n_new - 1) >> 5) - (c->hlens[b] >> 5) + 1;
        max_slabs = sl > max_slabs ? sl : max_slabs;
      }
  }
  dim3 grid(3 * max_slabs, v.NRG, v.B);
  if (c->ev_start) RKV_HIP_CHECK(hipEventRecord(c->ev_start, s));
  if (append_row(c)) {
    const size_t dyn = (size_t)384 * (v.NG | 1);
#define RKV_AP_VAL(G_, H_, S_) hipLaunchKernelGGL((k_append_values<G_, H_, S_>), dim3(max_slabs, v.NRG, v.B), dim3(256), 0, s, v, vv, n_new, slab0)
#define RKV_AP_ROW(G_, H_)                                                                                                        \
  do {                                                                                                                            \
    if (dyn > 48 * 1024)                                                                                                          \
      RKV_HIP_CHECK(hipFuncSetAttribute((const void*)k_append_row_keys<G_, H_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn)); \
    hipLaunchKernelGGL((k_append_row_keys<G_, H_>), dim3(2 * max_slabs, v.B), dim3(256), dyn, s, v, k, n_new, slab0);             \
    if (v.qg == 64) RKV_AP_VAL(G_, H_, 2); else if (v.qg == 32) RKV_AP_VAL(G_, H_, 4); else RKV_AP_VAL(G_, H_, 0);                \
  } while (0)
    if (v.g == 4) {
      if (v.hb == 2) RKV_AP_ROW(4, 2); else if (v.hb == 1) RKV_AP_ROW(4, 1); else RKV_AP_ROW(4, 0);
    } else {
      if (v.hb == 2) RKV_AP_ROW(2, 2); else if (v.hb == 1) RKV_AP_ROW(2, 1); else RKV_AP_ROW(2, 0);
    }
#undef RKV_AP_ROW
#undef RKV_AP_VAL
  } else {
    // (G, bits above the low two, cross-block flag, sub-blocks per head)
#define RKV_AP(G_, H_, X_, S_) hipLaunchKernelGGL((k_append_mfma<G_, H_, X_, S_>), grid, dim3(256), 0, s, v, k, vv, n_new, slab0)
#define RKV_AP_G(H_, X_, S_) do { if (v.g == 4) RKV_AP(4, H_, X_, S_); else RKV_AP(2, H_, X_, S_); } while (0)
#define RKV_AP_H(X_, S_) do { if (v.hb == 2) RKV_AP_G(2, X_, S_); else if (v.hb == 1) RKV_AP_G(1, X_, S_); else RKV_AP_G(0, X_, S_); } while (0)
    if (v.qg == 64 && c->blocks_aligned) RKV_AP_H(false, 2);
    else if (v.qg == 32 && c->blocks_aligned) RKV_AP_H(false, 4);
    else if (v.qg == 64) RKV_AP_H(true, 2);
    else if (v.qg == 32) RKV_AP_H(true, 4);
    else if (!c->blocks_aligned) RKV_AP_H(true, 0);
    else RKV_AP_H(false, 0);
#undef RKV_AP_H
#undef RKV_AP_G
#undef RKV_AP
  }
  if (c->ev_stop) RKV_HIP_CHECK(hipEventRecord(c->ev_stop, s));
  return rkv_check_launch();
}

// The fused launch of k_step_mfma: one token per sequence from k, vv [batch][1][...], queries q.
int rkv_launch_step_mfma(rkv_cache* c, const __half* k, const __half* vv, const __half* q, const int* q_pos, float* qr, int share,
                         hipStream_t s) {
  const RkvView& v = c->v;
  if (!rkv_append_mfma_supported(c) || append_row(c)) return RKV_EINVAL;
  int max_slabs = 1;                                        // one token touches one slab of its sequence
  const int n_append = 3 * max_slabs, rep = v.Hq / v.Hkv;
  dim3 grid(n_append + v.g * rep / 2, v.NRG, v.B);
#define RKV_ST(G_, H_, X_, S_) \
  hipLaunchKernelGGL((k_step_mfma<G_, H_, X_, S_>), grid, dim3(256), 0, s, v, k, vv, v.len >> 5, n_append, q, q_pos, qr, share)
#define RKV_ST_G(H_, X_, S_) do { if (v.g == 4) RKV_ST(4, H_, X_, S_); else RKV_ST(2, H_, X_, S_); } while (0)
#define RKV_ST_H(X_, S_) do { if (v.hb == 2) RKV_ST_G(2, X_, S_); else if (v.hb == 1) RKV_ST_G(1, X_, S_); else RKV_ST_G(0, X_, S_); } while (0)
  if (v.qg == 64 && c->blocks_aligned) RKV_ST_H(false, 2);
  else if (v.qg == 32 && c->blocks_aligned) RKV_ST_H(false, 4);
  else if (v.qg == 64) RKV_ST_H(true, 2);
  else if (v.qg == 32) RKV_ST_H(true, 4);
  else if (!c->blocks_aligned) RKV_ST_H(true, 0);
  else RKV_ST_H(false, 0);
#undef RKV_ST_H
#undef RKV_ST_G
#undef RKV_ST
  return rkv_check_launch();
}

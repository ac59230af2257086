// Read half, a reorder over the whole token row (perm_span = n_kv_heads * head_dim: Alg. 1 as
// printed sorts all h * d channels of a layer): the scores of the compressed stream.
//
// With such a reorder a rotated channel belongs to any of the row's E / 128 quantization blocks, so
// the scales no longer factor out of the per-head Hadamard product and the FP4 route of the plain
// kernel (exact products of raw codes, scales afterwards) is closed.  Here every element is
// dequantized first, u = s (c - z) (Eq. 7; exact in fp32: an 11-bit scale times a 12-bit integer),
// split into two fp16 numbers u = hi + lo (what is lost is below 2^-22 of u), and the rotation
// H_128 of both parts runs on v_mfma_f32_16x16x32_f16 - products with +-1 are exact, the
// accumulation is fp32 -, as in the write half's kernel.  H_g over the heads, RoPE (Sec. 4.4 keeps
// the cache pre-RoPE) and the dot with the query follow on the vector ALU in fp32.
//
// One workgroup = (sequence, rotation group, 64 tokens), four waves, one tile of 16 tokens at a
// time:
//   stage   thread (token, rotated block, quarter q): the 32 codes of its 8 bytes of the K tile ->
//           fp16 rows [token][channel] of the two parts in LDS.  A token's (scale, zero-point) of
//           all E / 128 blocks come from a table in LDS that holds, per (token, block), the four
//           values s (c - z) / 64, c = 0..3 (the factor keeps |u| inside fp16 for any fp16 input);
//           a channel's block is looked up in a per-workgroup copy of gid (as a byte offset).
//   rotate  wave w: A = 16 rows of H_128 (signs made in registers), B = the rows of 16 tokens, so
//           lane (token, q) of the result holds channels 16q + 4w + r and 64 + 16q + 4w + r,
//           r = 0..3, of every head: both channels of a RoPE pair, whichever the pairing.
//   dot     per lane over its 8 channels of each head, over the four lane groups q with lane
//           exchanges, over the four waves through LDS (in a fixed order: the result does not
//           depend on timing).
// The scores go to a buffer [sequence][query head][token slot] (-infinity at retained sink tokens);
// the matrix-core decode kernel takes them from there in place of its own key phase and does the
// softmax, the values and the partial results as for any other configuration.
#include "rkv_internal.h"

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));

#define RS_TILES 4                      // tiles of 16 tokens per workgroup
static_assert(16 * RS_TILES == RKV_ROW_CHUNK, "the launch grid counts chunks of RKV_ROW_CHUNK tokens");

__device__ __forceinline__ v8h row_v8h(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  union { uint32_t u[4]; v8h h; } x;
  x.u[0] = a; x.u[1] = b; x.u[2] = c; x.u[3] = d;
  return x.h;
}
__device__ __forceinline__ uint32_t row_parity(int x, uint32_t m) { return (__popc(x) & 1) ? m : 0u; }

// dynamic LDS: [16][NG | 1] float4 table, [G * rep][128] float queries, [4][G * rep][16] float partial scores
// STYLE: the RoPE pairing (rkv_config.rope_style)
template <int G, int STYLE>
__global__ void __launch_bounds__(256, 3) k_scores_row(RkvView v, const float* __restrict__ qr, float* __restrict__ sc, int rep) {
  constexpr int n = 128 * G;
  constexpr int ROW16 = 16 * G;                // 16-byte pieces per fp16 row of the rotation group
  constexpr int STRIDE16 = ROW16 + 1;          // padded: the matrix operand reads touch every LDS bank once
  __shared__ __attribute__((aligned(16))) uint4 s_hi[16 * STRIDE16], s_lo[16 * STRIDE16];
  // byte offset of a channel's block inside a token's table row; four dwords of padding after every
  // 32 channels, so that the lanes of a wave (two quarters q of two rotated blocks) read from different banks
  __shared__ __attribute__((aligned(16))) uint32_t s_goff[n + n / 8];
  __shared__ int s_sink[64];
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
  // (table rows of an odd number of entries: the 16 tokens of a tile then start in different LDS banks)
  const int NG = v.E >> 7, NGP = NG | 1, nqh = G * rep;
  float4* s_tab = reinterpret_cast<float4*>(dyn);
  float* s_qp = reinterpret_cast<float*>(dyn + (size_t)16 * NGP * 16);
  float* s_pw = s_qp + nqh * RKV_D;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int chunk = blockIdx.x, rg = blockIdx.y, b = blockIdx.z;
  const int len = rkv_len(v, b);
  const int t0 = chunk * (16 * RS_TILES);
  if (t0 >= len) return;                               // (the grid covers the longest sequence)
  const int cnt = v.max_sinks > 0 ? v.sink_cnt[b] : 0;
  if (tid < 64) s_sink[tid] = tid < cnt ? v.sink_pos[b * v.max_sinks + tid] : -1;
  for (int c = tid; c < n; c += 256) s_goff[c + ((c >> 5) << 2)] = (uint32_t)v.gid[rg * n + c] * 16u;
  for (int i = tid; i < nqh * RKV_D; i += 256) s_qp[i] = qr[((size_t)b * v.Hq + (size_t)rg * nqh) * RKV_D + i];

  // stage role: piece p of the K tile (16 bytes: two rotated blocks x 2 dwords), one block of it
  const int p = tid >> 1, half = tid & 1;
  const bool stager = p < 32 * G;
  const int s_q = (p >> 4) & 3, s_tok = p & 15, s_blk = 2 * (p >> 6) + half;
  // rotate role: A operand rows: lane (row m, k-group kg) holds H_128[channel][32 ks + 8 kg + i], channel =
  // 64 ppl + 16 (m >> 2) + 4 wave + (m & 3); the sign is the parity of (channel & k), which splits into
  // the low three bits (base) and the rest (a flip of all eight)
  const int col = lane & 15, kg = lane >> 4;
  const int m_row = lane & 15;
  uint32_t abase[4];
  {
    const int e7 = 4 * (wave & 1) + (m_row & 3);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      abase[j] = (0x3C003C00u ^ row_parity(e7 & (2 * j), 0x00008000u)) ^ row_parity(e7 & (2 * j + 1), 0x80000000u);
  }
  const int chi = 2 * (m_row >> 2) + (wave >> 1);          // bits 3..5 of the channel, without ppl
  uint32_t flips = 0;                                      // bit 2 ks + ppl: the flip of product (ks, ppl)
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int ppl = 0; ppl < 2; ++ppl) flips |= (uint32_t)(__popc((8 * ppl + chi) & (4 * ks + kg)) & 1) << (2 * ks + ppl);
  const float out_scale = 64.0f * rsqrtf((float)n);        // the table's 1/64 and the normalisation of Eq. 10

  // What a tile needs from memory - the thread's 8 bytes of codes, its share of the tile's metadata
  // (entry e = 16 * rotation group + token: that token's G blocks of that group; two rounds cover up
  // to 32 rotation groups) and the RoPE angles of the lane's token - is requested a tile ahead.
  constexpr int MROUNDS = 2;
  uint2 cw = make_uint2(0, 0);
  uint32_t mw[MROUNDS][G];
  float4 ang[2];
  auto request = [&](int ti) {
    const int tt = t0 + 16 * ti;
    if (stager) cw = rkv_ld_stream(reinterpret_cast<const uint2*>(v.kc + rkv_k_tilebase(v, b, rg, tt >> 4) + (size_t)p * 4 + half * 2));
#pragma unroll
    for (int k = 0; k < MROUNDS; ++k) {
      const int e = tid + 256 * k;
      if (e < 16 * v.NRG) {
        const uint32_t* mp = v.km + ((size_t)(b * v.NRG + (e >> 4)) * v.Tpad + tt + (e & 15)) * G;
        if constexpr (G == 4) {
          const uint4 u = *reinterpret_cast<const uint4*>(mp);
          mw[k][0] = u.x; mw[k][1] = u.y; mw[k][2] = u.z; mw[k][3] = u.w;
        } else {
          const uint2 u = *reinterpret_cast<const uint2*>(mp);
          mw[k][0] = u.x; mw[k][1] = u.y;
        }
      }
    }
    if constexpr (STYLE == 0) {
      const float4* rp = reinterpret_cast<const float4*>(v.rope + (size_t)(tt + col) * 64 + 16 * kg + 4 * wave);
      ang[0] = rp[0];
      ang[1] = rp[1];
    }
  };
  request(0);

  // the four waves' shares of a tile's scores, added in a fixed order; retained sink tokens are
  // masked out of the stream
  auto sum_tile = [&](int tt) {
    for (int i = tid; i < nqh * 16; i += 256) {
      const int hr = i >> 4, tk = tt + (i & 15);
      if (tk < len) {
        float tot = s_pw[(0 * nqh + hr) * 16 + (i & 15)];
#pragma unroll
        for (int w = 1; w < 4; ++w) tot += s_pw[(w * nqh + hr) * 16 + (i & 15)];
        bool sink = false;
        for (int k = 0; k < cnt; ++k) sink |= (s_sink[k] == tk);
        sc[((size_t)b * v.Hq + (size_t)rg * nqh + hr) * v.Tpad + tk] = sink ? -INFINITY : tot * out_scale;
      }
    }
  };

  // Two barriers per tile: [table of tile i] B1 [sums of tile i - 1; rows of tile i] B2 [products and
  // dots of tile i].  The table is next written after B2, when nobody reads it any more; the partial
  // scores are written after B2 and read after the next B1; the rows are read after B2 and next
  // written after the next B1.
  int ti = 0;
  for (; ti < RS_TILES; ++ti) {
    const int tt = t0 + 16 * ti;
    if (tt >= len) break;                                  // workgroup-uniform
    // ---- stage: table of dequantized values, then the tile's elements
#pragma unroll
    for (int k = 0; k < MROUNDS; ++k) {
      const int e = tid + 256 * k;
      if (e < 16 * v.NRG) {
        const int g2 = e >> 4, tok = e & 15;
#pragma unroll
        for (int j = 0; j < G; ++j) {
          float s_, z_;
          rkv_unpack_meta(mw[k][j], s_, z_);
          s_ *= 0.015625f;
          s_tab[tok * NGP + g2 * G + j] = make_float4(s_ * (0.f - z_), s_ * (1.f - z_), s_ * (2.f - z_), s_ * (3.f - z_));
        }
      }
    }
    const float4 ang0 = ang[0], ang1 = ang[1];
    __syncthreads();
    if (ti > 0) sum_tile(tt - 16);
    if (stager) {
      const unsigned char* trow = reinterpret_cast<const unsigned char*>(s_tab) + (size_t)s_tok * NGP * 16;
#pragma unroll
      for (int dw = 0; dw < 2; ++dw) {
        const uint32_t w = dw ? cw.y : cw.x;
#pragma unroll
        for (int vl = 0; vl < 2; ++vl) {
          // channels 32 q + 16 dw + 8 vl + e, e = 0..7, of the block: code field 2 e + vl of the dword
          const int c0 = 128 * s_blk + 32 * s_q + 16 * dw + 8 * vl;
          const int ci = c0 + ((c0 >> 5) << 2);
          const uint4 g0 = *reinterpret_cast<const uint4*>(&s_goff[ci]), g1 = *reinterpret_cast<const uint4*>(&s_goff[ci + 4]);
          const uint32_t go[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
          float u[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t code = (w >> (2 * (2 * e + vl))) & 3u;
            u[e] = *reinterpret_cast<const float*>(trow + go[e] + 4u * code);
          }
          uint32_t hi[4], lo[4];
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            hi[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(u[e], u[e + 1]));
            // what the fp16 pair misses: u - hi, straight from the packed halves (one mixed-precision FMA each)
            float l0, l1;
            asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(l0) : "v"(hi[e >> 1]), "v"(u[e]));
            asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(l1) : "v"(hi[e >> 1]), "v"(u[e + 1]));
            lo[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(l0, l1));
          }
          const int piece = s_tok * STRIDE16 + (c0 >> 3);
          s_hi[piece] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
          s_lo[piece] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
      }
    }
    if (ti + 1 < RS_TILES && tt + 16 < len) request(ti + 1);   // (in flight during the matrix products)
    __syncthreads();
    // ---- rotate: H_128 of every head for this wave's 32 channels, both parts onto one accumulator
    v4f acc[G][2];
    {
      const uint4* xh = s_hi + col * STRIDE16 + kg;
      const uint4* xl = s_lo + col * STRIDE16 + kg;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int ppl = 0; ppl < 2; ++ppl) {
          const uint32_t mk = ((flips >> (2 * ks + ppl)) & 1u) * 0x80008000u;
          const v8h a = row_v8h(abase[0] ^ mk, abase[1] ^ mk, abase[2] ^ mk, abase[3] ^ mk);
#pragma unroll
          for (int h = 0; h < G; ++h) {
            const uint4 bh = xh[16 * h + 4 * ks], bl = xl[16 * h + 4 * ks];
            const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
            acc[h][ppl] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, row_v8h(bh.x, bh.y, bh.z, bh.w), ks == 0 ? zero4 : acc[h][ppl], 0, 0, 0);
            acc[h][ppl] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, row_v8h(bl.x, bl.y, bl.z, bl.w), acc[h][ppl], 0, 0, 0);
          }
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
    // RoPE at the token's position (pairs (j, j + 64): a lane's channels c and c + 64; interleaved
    // pairs: its channels r = 0, 1 and r = 2, 3 of either half), then the dot with the query
    const int tok = tt + col;                              // (inside the padded allocation)
    const int cb = 16 * kg + 4 * wave;                     // the lane's first channel
    float klo[G][4], khi[G][4];                            // rotated pair halves, [head][pair of the lane]
    {
      float2 cs[4];
      if constexpr (STYLE == 0) {
        const float4 r0 = ang0, r1 = ang1;
        cs[0] = make_float2(r0.x, r0.y); cs[1] = make_float2(r0.z, r0.w); cs[2] = make_float2(r1.x, r1.y); cs[3] = make_float2(r1.z, r1.w);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int c_even = 64 * (i >> 1) + cb + 2 * (i & 1);
          cs[i] = v.rope[(size_t)tok * 64 + (c_even >> 1)];
        }
      }
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float x = STYLE == 0 ? acc[h][0][i] : acc[h][i >> 1][2 * (i & 1)];
          const float y = STYLE == 0 ? acc[h][1][i] : acc[h][i >> 1][2 * (i & 1) + 1];
          klo[h][i] = x * cs[i].x - y * cs[i].y;
          khi[h][i] = x * cs[i].y + y * cs[i].x;
        }
    }
    for (int r = 0; r < rep; ++r) {
#pragma unroll
      for (int h = 0; h < G; ++h) {
        // the query at the lane's channels cb .. cb + 3 and 64 + cb .. + 3
        const float4 qa = *reinterpret_cast<const float4*>(s_qp + (h * rep + r) * RKV_D + cb);
        const float4 qb = *reinterpret_cast<const float4*>(s_qp + (h * rep + r) * RKV_D + cb + 64);
        float d;
        if constexpr (STYLE == 0) {
          d = fmaf(khi[h][0], qb.x, klo[h][0] * qa.x);
          d = fmaf(khi[h][1], qb.y, fmaf(klo[h][1], qa.y, d));
          d = fmaf(khi[h][2], qb.z, fmaf(klo[h][2], qa.z, d));
          d = fmaf(khi[h][3], qb.w, fmaf(klo[h][3], qa.w, d));
        } else {
          d = fmaf(khi[h][0], qa.y, klo[h][0] * qa.x);
          d = fmaf(khi[h][1], qa.w, fmaf(klo[h][1], qa.z, d));
          d = fmaf(khi[h][2], qb.y, fmaf(klo[h][2], qb.x, d));
          d = fmaf(khi[h][3], qb.w, fmaf(klo[h][3], qb.z, d));
        }
        d += __shfl_xor(d, 16);
        d += __shfl_xor(d, 32);
        if (kg == 0) s_pw[(wave * nqh + h * rep + r) * 16 + col] = d;
      }
    }
  }
  if (ti > 0) {
    __syncthreads();
    sum_tile(t0 + 16 * (ti - 1));
  }
}

// ---------------------------------------------------------------------------------------------
// The same scores with one wave per tile of 16 tokens and no traffic of dequantized rows through
// LDS (rows of at most 63 quantization blocks; the kernel above serves longer rows).
//
// A lane of the K tile's 16-byte load, (token, quarter q), holds exactly the codes the matrix
// instruction wants from it as the B operand [k][token]: four channels per product, each as its
// (hi, lo) pair of fp16 numbers in two neighbouring k slots (the A operand repeats its +-1 for
// both, so the instruction adds the two parts by itself).  The pairs come ready-made from a table
// in LDS, one dword (hi | lo << 16) per (token, quantization block, code), laid out [entry][token]
// so that the 16 tokens of a row of lanes read 16 different banks whatever their codes are; the
// byte address of a channel's entry is (block << 8 | code << 6 | token << 2): the block is a
// per-layer constant that sits in a small table, four channels to a dword, the low byte is made
// for four code fields of the stream at once, and one byte permute per channel joins the two.
//
// H_128 = H_8 (x) H_16: a product contracts the channel bits {1, 2} (the four channels of a lane's
// dword) and {5, 6} (the quarter) against the same bits of the output channel (rows of A), and
// the bits {0, 3, 4} by accumulation - the eight products of a head's eight steps s onto output
// tile mt carry the sign (-1)^popc(mt & s), the same for every lane, i.e. A or -A (equal partial
// sums are shared, and the stage of bit 4 is a pair of additions in the lane: 22 products and 32
// additions per head; a matrix product keeps the vector pipe from issuing for most of its 16
// cycles, so trading 21 of them for 32 additions pays).  A lane
// (token, g4) of the result holds, per head, tiles mt = 0..7 x rows r = 0..3: output channel bits
// 6 = r & 1, 5 = g4 >> 1, 4 3 0 = mt, 2 = g4 & 1, 1 = r >> 1 - both channels of a RoPE pair of either
// pairing.  H_g over the heads is split: P0 = X0 + X1, P1 = X0 - X1 of a pair of heads go through
// RoPE and are multiplied with the queries of the output heads that take them (a of the same
// parity; the second pair of heads enters with the sign of H_g's second stage), so that only two
// heads' results are in registers at a time.  The query values of a lane's 32 channels are spread
// over the four lanes of its quad (the four lanes hold the same channels for different tokens) and
// reach the multiply-adds through the quad-broadcast operand modifier.
// Everything a wave touches between two tiles is its own (table, partial sums), so the tile loop
// has no workgroup barrier.
#ifndef RS2_TILES
#define RS2_TILES 1                     // tiles of 16 tokens per wave (measured on config 2's geometry: 1: 157 us, 2: 171, 4: 175, 8: 180 -
#endif                                  // short-lived waves drift apart, so one wave's matrix products run beside another's vector work)
#define RS2_CHUNK (64 * RS2_TILES)      // tokens per workgroup
#define RS2_MPRE 3                      // rounds of metadata (4 rotation groups x 16 tokens each) requested a tile ahead
#ifndef RS2_OCC
#define RS2_OCC 3                       // workgroups per compute unit the register budget is set for
#endif
#ifndef RS2_EARLY
#define RS2_EARLY 0
#endif
#ifndef RS2_HALVES
#define RS2_HALVES 1                    // 1: the last stage of H_8 as additions in the lane (22 products and 32 additions per head instead of 43 products)
#endif
#ifndef RS2_LOOK
#define RS2_LOOK 4                      // steps looked up at a time (4 registers each)
#endif
#define RS2_MAX_NG 63                   // longest row in quantization blocks (a wave's table takes 256 bytes per block)

// d += (q of lane U of the quad) * k.  The operand modifier reads q from another lane; the hardware wants two
// instructions between a vector write of q and this read: q is loaded from LDS and pinned by rs2_settle below.
// (scale byte j of sw as FP8 E4M3, zero-point byte j of zw as value + 128) -> the fp16 (scale, zero-point) pair of
// the other format (both numbers are exact in fp16), so that the table is made by one piece of code
__device__ __forceinline__ uint32_t rs2_meta8_pair(uint32_t sw, uint32_t zw, int j) {
  const float s_ = j == 0 ? __builtin_amdgcn_cvt_f32_fp8((int)sw, 0) : j == 1 ? __builtin_amdgcn_cvt_f32_fp8((int)sw, 1)
                 : j == 2 ? __builtin_amdgcn_cvt_f32_fp8((int)sw, 2) : __builtin_amdgcn_cvt_f32_fp8((int)sw, 3);
  return rkv_pack_meta(s_, (float)((zw >> (8 * j)) & 0xffu) - 128.0f);
}

typedef __attribute__((address_space(3))) unsigned char rs2_lds_u8;
typedef __attribute__((address_space(3))) uint32_t rs2_lds_u32;

template <int U>
__device__ __forceinline__ void fmac_quad(float& d, float q, float k) {
  if constexpr (U == 0) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf" : "+v"(d) : "v"(q), "v"(k));
  if constexpr (U == 1) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf" : "+v"(d) : "v"(q), "v"(k));
  if constexpr (U == 2) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf" : "+v"(d) : "v"(q), "v"(k));
  if constexpr (U == 3) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf" : "+v"(d) : "v"(q), "v"(k));
}
template <int U>
__device__ __forceinline__ float fmul_quad(float q, float k) {       // (q of lane U of the quad) * k
  float d;
  if constexpr (U == 0) asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf" : "=v"(d) : "v"(q), "v"(k));
  if constexpr (U == 1) asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf" : "=v"(d) : "v"(q), "v"(k));
  if constexpr (U == 2) asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf" : "=v"(d) : "v"(q), "v"(k));
  if constexpr (U == 3) asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf" : "=v"(d) : "v"(q), "v"(k));
  return d;
}
__device__ __forceinline__ void rs2_settle(float (&q)[2][4]) {
  asm volatile("s_nop 1" : "+v"(q[0][0]), "+v"(q[0][1]), "+v"(q[0][2]), "+v"(q[0][3]), "+v"(q[1][0]), "+v"(q[1][1]), "+v"(q[1][2]), "+v"(q[1][3]));
}

// dynamic LDS: [4 waves][NG * 4 entries][16 tokens] dwords, [4 waves][G * rep][16] float partial sums, [G * rep][128] float
// queries, [4 waves][4 * G * 8] dwords of block bytes, 64 sink positions
// LOCAL: groups of 64 / 32 with the reorder inside the heads - the table holds the rotation group's own v.gm blocks
// HB = 1, 2 (with LOCAL): codes of 3 and 4 bits, c = c_lo + 4 c_hi.  A wave's table gets a second half for the
// plane of upper bits, with entries s * 4 c_hi, and every step looks up both planes and runs its products
// twice onto the same accumulators (the rotation is linear).
// HB = 1, 2 without LOCAL (a reorder over the whole row, where two table halves would not fit): this launch
// takes the plane of upper bits alone - the table holds s * 4 c_hi - and adds its scores to those a launch
// with HB = 0 has left in the buffer.
// PART (a reorder over the whole row with groups of 64 / 32, whose 2 to 4 times as many blocks do not fit a
// wave's table): this launch takes the row's blocks b0 .. b0 + cnt - 1 alone.  A channel of any other block
// looks up an all-zero block behind them, and the launches' scores add up in the buffer.
// part = b0 | cnt << 12 | (add to the scores in the buffer) << 24.
template <int G, int STYLE, bool LOCAL, int HB = 0, bool PART = false>
__global__ void __launch_bounds__(256, (HB && LOCAL) ? 2 : RS2_OCC) k_scores_row2(RkvView v, const float* __restrict__ qr, float* __restrict__ sc, int rep,
                                                                                 int part) {
  static_assert(!PART || !LOCAL, "a share of the row's blocks: the whole-row reorder");
  constexpr int n = 128 * G;
  const int pb0 = part & 0xfff, pcnt = (part >> 12) & 0xfff;
  const bool padd = (part >> 24) != 0;
  constexpr bool UPPER = HB != 0 && !LOCAL;             // the upper plane's launch of a pair
  constexpr int NPL = (HB && LOCAL) ? 2 : 1;            // planes of code bits in this launch, each with its half of the table
  // (no static LDS in this kernel: the tables start where the workgroup's LDS starts, so that a table's byte
  // address >> 8 plus a block index stays below 256 for rows of up to RS2_MAX_NG blocks)
  extern __shared__ __attribute__((aligned(256))) unsigned char dyn2[];
  const int NG = LOCAL ? v.gm : PART ? pcnt + 1 : v.E >> 7, nqh = G * rep;   // blocks in a wave's table
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int NGT = NG * NPL;                              // blocks of a wave's table, both halves
  uint32_t* s_tab = reinterpret_cast<uint32_t*>(dyn2) + (size_t)wave * NGT * 64;
  float* s_pd = reinterpret_cast<float*>(dyn2 + (size_t)4 * NGT * 256) + wave * nqh * 16;
  const float* s_qp = reinterpret_cast<const float*>(dyn2 + (size_t)4 * NGT * 256 + (size_t)4 * nqh * 64);
  // [wave][q][head][dword dw][shift ksh]: four channels' quantization blocks, a byte each, plus (the wave's table >> 8)
  uint32_t* s_g4 = reinterpret_cast<uint32_t*>(dyn2 + (size_t)4 * NGT * 256 + (size_t)4 * nqh * 64 + (size_t)nqh * RKV_D * 4);
  int* s_sink = reinterpret_cast<int*>(s_g4 + 4 * 4 * G * 8);
  const int chunk = blockIdx.x, rg = blockIdx.y, b = blockIdx.z;
  const int len = rkv_len(v, b);
  const int t0 = chunk * RS2_CHUNK;
  if (t0 >= len) return;                               // (the grid covers the longest sequence)
  const int tok = lane & 15, kq = lane >> 4;           // B operand and result: (token, quarter / row group g4)
  const uint32_t tokrep = 4u * tok * 0x01010101u;      // token << 2 in every byte
  // A operand: lane (row m, k-group kg) holds +-1 for k = (channel j of the step, part): the sign is the parity of
  // m0 & in6 ^ m3 & in5 ^ m1 & in1 ^ m2 & in2, in6 in5 = kg, in2 in1 = j
  uint32_t a_pos[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int m = lane & 15, kg = lane >> 4;
    const int sg = ((m & 1) & (kg >> 1)) ^ ((m >> 3) & (kg & 1)) ^ (((m >> 1) & 1) & (j & 1)) ^ (((m >> 2) & 1) & (j >> 1));
    a_pos[j] = 0x3C003C00u ^ (sg ? 0x80008000u : 0u);
  }
  const v8h A_pos = row_v8h(a_pos[0], a_pos[1], a_pos[2], a_pos[3]);
  const v8h A_neg = row_v8h(a_pos[0] ^ 0x80008000u, a_pos[1] ^ 0x80008000u, a_pos[2] ^ 0x80008000u, a_pos[3] ^ 0x80008000u);
  const float out_scale = 64.0f * rsqrtf((float)n);        // the table's 1/64 and the normalisation of Eq. 10
  const int g4hi = kq >> 1, g4lo = kq & 1, qu = lane & 3;
  const int rounds = (v.NRG + 3) >> 2;

  uint4 cw[G / 2], cwh[HB ? G / 2 : 1];
  uint32_t mb[PART ? 16 : 1];                            // PART: the lane's token's entries of blocks b0 + kq + 4 i
  uint32_t mw[RS2_MPRE][G];
  uint32_t ml[4] = {0, 0, 0, 0};
  const int bpl = LOCAL ? (v.gm >= 4 ? v.gm >> 2 : 1) : 0;                // blocks per lane group (1, 2 or 4; with two blocks, lane groups 0 and 1 take one each)
  const bool lact = LOCAL && kq * bpl < v.gm;
  const uint32_t loff = LOCAL ? (uint32_t)(tok * v.gm + kq * bpl) : 0u;
  const uint32_t roff = (uint32_t)(tok * 64 + (STYLE == 0 ? 32 * g4hi + 4 * g4lo : 16 * g4hi + 2 * g4lo));   // the lane's place in a tile's RoPE rows
  const uint32_t moff = (uint32_t)(kq * v.Tpad + tok);   // metadata entry of (rotation group kq of a round, token), in units of G dwords
  auto request = [&](int tt) {
    const uint4* kt = reinterpret_cast<const uint4*>(v.kc + rkv_k_tilebase(v, b, rg, tt >> 4));
#pragma unroll
    for (int bp = 0; bp < G / 2; ++bp) cw[bp] = rkv_ld_stream(kt + 64 * bp + lane);
    if constexpr (HB == 2) {                               // the plane of the upper two bits: the layout of the lower one
      const uint4* kth = reinterpret_cast<const uint4*>(v.kh + rkv_k_tilebase(v, b, rg, tt >> 4));
#pragma unroll
      for (int bp = 0; bp < G / 2; ++bp) cwh[bp] = rkv_ld_stream(kth + 64 * bp + lane);
    } else if constexpr (HB == 1) {                        // the plane of third bits: one dword per pair of code dwords
      const uint2* kth = reinterpret_cast<const uint2*>(v.kh + (rkv_k_tilebase(v, b, rg, tt >> 4) >> 1));
#pragma unroll
      for (int bp = 0; bp < G / 2; ++bp) {
        const uint2 u = rkv_ld_stream(kth + 64 * bp + lane);
        cwh[bp] = make_uint4(u.x, u.y, 0, 0);
      }
    }
    if constexpr (PART) {
      const int lg = __builtin_ctz((unsigned)v.gm);        // (v.gm = G * 128 / quant_group: a power of two)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int bi = kq + 4 * i;
        if (bi < pcnt) {
          const int blk = pb0 + bi, rgb = blk >> lg, j = blk & (v.gm - 1);
          const size_t e = ((size_t)(b * v.NRG + rgb) * v.Tpad + tt + tok) * v.gm;
          if (v.meta8) {
            const uint8_t* m8 = reinterpret_cast<const uint8_t*>(v.km) + 2 * e;
            mb[i] = rs2_meta8_pair(m8[j], m8[v.gm + j], 0);
          } else {
            mb[i] = v.km[e + j];
          }
        }
      }
      return;
    }
    if constexpr (LOCAL) {
      // the token's v.gm entries of this rotation group: a quarter of them per lane group
      if (v.meta8) {                                       // v.gm scale bytes, then v.gm zero-point bytes
        const uint8_t* m8 = reinterpret_cast<const uint8_t*>(v.km) + ((size_t)(b * v.NRG + rg) * v.Tpad + tt + tok) * (2 * v.gm) + kq * bpl;
        uint32_t sw, zw;                                     // the lane's bpl scale bytes and zero-point bytes, one load each
        if (bpl == 4) {
          sw = *reinterpret_cast<const uint32_t*>(m8);
          zw = *reinterpret_cast<const uint32_t*>(m8 + v.gm);
        } else if (bpl == 2) {
          sw = *reinterpret_cast<const uint16_t*>(m8);
          zw = *reinterpret_cast<const uint16_t*>(m8 + v.gm);
        } else {
          sw = lact ? m8[0] : 0u;
          zw = lact ? m8[v.gm] : 0u;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) ml[i] = rs2_meta8_pair(sw, zw, i);
        return;
      }
      const uint32_t* mrow = v.km + ((size_t)(b * v.NRG + rg) * v.Tpad + tt) * v.gm;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < bpl && lact) ml[i] = mrow[loff + i];
      return;
    }
#pragma unroll
    for (int k = 0; k < RS2_MPRE; ++k) {
      const int g2 = kq + 4 * k;
      if (g2 < v.NRG) {
        // (a base that is the same for all lanes plus a 32-bit lane offset: one register per lane, not an address pair)
        if (v.meta8) {                                     // G scale bytes, then G zero-point bytes per (token, rotation group)
          const uint8_t* m8 = reinterpret_cast<const uint8_t*>(v.km) + ((size_t)(b * v.NRG + 4 * k) * v.Tpad + tt + moff) * (2 * G);
          uint32_t sw, zw;
          if constexpr (G == 4) {
            const uint2 u = *reinterpret_cast<const uint2*>(m8);
            sw = u.x; zw = u.y;
          } else {
            sw = *reinterpret_cast<const uint32_t*>(m8);
            zw = sw >> 16;
          }
#pragma unroll
          for (int j = 0; j < G; ++j) mw[k][j] = rs2_meta8_pair(sw, zw, j);
          continue;
        }
        const uint32_t* mrow = v.km + ((size_t)(b * v.NRG + 4 * k) * v.Tpad + tt) * G;
        if constexpr (G == 4) {
          const uint4 u = reinterpret_cast<const uint4*>(mrow)[moff];
          mw[k][0] = u.x; mw[k][1] = u.y; mw[k][2] = u.z; mw[k][3] = u.w;
        } else {
          const uint2 u = reinterpret_cast<const uint2*>(mrow)[moff];
          mw[k][0] = u.x; mw[k][1] = u.y;
        }
      }
    }
  };
  request(t0 + 16 * RS2_TILES * wave);                             // (in flight during the set-up)
  const int cnt = v.max_sinks > 0 ? v.sink_cnt[b] : 0;
  if (tid < 64) s_sink[tid] = tid < cnt ? v.sink_pos[b * v.max_sinks + tid] : -1;
  if (tid < 4 * G * 8) {
    const int q = tid / (8 * G), h = (tid >> 3) % G, dw = (tid >> 2) & 1, ksh = tid & 3;
    const int c0 = 128 * h + 32 * q + 16 * dw + 8 * (ksh & 1) + (ksh >> 1);
    uint32_t w = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t bid = (uint32_t)(v.gid[rg * n + c0 + 2 * j] - (LOCAL ? rg * v.gm : PART ? pb0 : 0));
      if (PART && bid >= (uint32_t)pcnt) bid = (uint32_t)pcnt;       // another launch's block: the all-zero one
      w |= bid << (8 * j);
    }
    const uint32_t tab0 = (uint32_t)(uintptr_t)(rs2_lds_u8*)dyn2;     // LDS byte address of the first table (a multiple of 256)
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) s_g4[ww * (4 * G * 8) + tid] = w + (((tab0 >> 8) + (uint32_t)(ww * NGT)) * 0x01010101u);
  }
  {
    float* qp = const_cast<float*>(s_qp);
    for (int i = tid; i < nqh * RKV_D; i += 256) qp[i] = qr[((size_t)b * v.Hq + (size_t)rg * nqh) * RKV_D + i];
  }
  __syncthreads();

  // the four table entries of one quantization block of the lane's token
  auto put_four = [&](int blk, float u0, float u1, float u2, float u3) {
    const uint32_t h01 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(u0, u1));
    const uint32_t h23 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(u2, u3));
    float l0, l1, l2, l3;                                   // what the fp16 number misses (exact)
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(l0) : "v"(h01), "v"(u0));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(l1) : "v"(h01), "v"(u1));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(l2) : "v"(h23), "v"(u2));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(l3) : "v"(h23), "v"(u3));
    const uint32_t l01 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(l0, l1));
    const uint32_t l23 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(l2, l3));
    uint32_t* e = s_tab + (blk * 4) * 16 + tok;
    e[0] = __builtin_amdgcn_perm(l01, h01, 0x05040100u);
    e[16] = __builtin_amdgcn_perm(l01, h01, 0x07060302u);
    e[32] = __builtin_amdgcn_perm(l23, h23, 0x05040100u);
    e[48] = __builtin_amdgcn_perm(l23, h23, 0x07060302u);
  };
  auto put_block = [&](int blk, uint32_t word) {
    float s_, z_;
    rkv_unpack_meta(word, s_, z_);                         // (8-bit metadata were turned into this form when they were fetched)
    s_ *= 0.015625f;
    if constexpr (!UPPER) put_four(blk, s_ * (0.f - z_), s_ * (1.f - z_), s_ * (2.f - z_), s_ * (3.f - z_));
    if constexpr (HB != 0) put_four(UPPER ? blk : NG + blk, 0.f, s_ * 4.f, s_ * 8.f, s_ * 12.f);   // the upper bits' share s * 4 c_hi
  };

  for (int it = 0; it < RS2_TILES; ++it) {
    const int tt = t0 + 16 * RS2_TILES * wave + 16 * it;
    if (tt >= len) break;                                  // wave-uniform
    // ---- the tile's table (the lanes of a wave write and read it in program order)
    if constexpr (LOCAL) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < bpl && lact) put_block(kq * bpl + i, ml[i]);
    }
    if constexpr (PART) {
      if (kq == 0) {
        uint32_t* e = s_tab + (pcnt * 4) * 16 + tok;
        e[0] = e[16] = e[32] = e[48] = 0u;
      }
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (kq + 4 * i < pcnt) put_block(kq + 4 * i, mb[i]);
    }
#pragma unroll
    for (int k = 0; k < ((LOCAL || PART) ? 0 : RS2_MPRE); ++k) {
      const int g2 = kq + 4 * k;
      if (g2 < v.NRG) {
#pragma unroll
        for (int j = 0; j < G; ++j) put_block(g2 * G + j, mw[k][j]);
      }
    }
    for (int k = RS2_MPRE; k < ((LOCAL || PART) ? 0 : rounds); ++k) {
      const int g2 = kq + 4 * k;
      if (g2 < v.NRG) {
        if (v.meta8) {
          const uint8_t* m8 = reinterpret_cast<const uint8_t*>(v.km) + ((size_t)(b * v.NRG + 4 * k) * v.Tpad + tt + moff) * (2 * G);
#pragma unroll
          for (int j = 0; j < G; ++j) put_block(g2 * G + j, rs2_meta8_pair(m8[j], m8[G + j], 0));
        } else {
          const uint32_t* mrow = v.km + ((size_t)(b * v.NRG + 4 * k) * v.Tpad + tt) * G;
#pragma unroll
          for (int j = 0; j < G; ++j) put_block(g2 * G + j, mrow[moff * G + j]);
        }
      }
    }
    // RoPE angles of the lane's token at its 16 pairs (eight 16-byte pieces of the table row)
    float4 ang[4][2];
    {
      const float2* rrow = v.rope + (size_t)tt * 64;
#pragma unroll
      for (int mq = 0; mq < 4; ++mq)
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const int j = STYLE == 0 ? 8 * mq + 2 * x : 32 * x + 4 * mq;
          ang[mq][x] = *reinterpret_cast<const float4*>(rrow + (roff + j));
        }
    }
    const uint4 cw0 = cw[0], ch0 = cwh[0];
    uint4 cw1 = cw0, ch1 = ch0;
    if constexpr (G == 4) cw1 = cw[1];
    if constexpr (G == 4 && HB != 0) ch1 = cwh[1];
    asm volatile("" ::: "memory");                        // (the LDS unit takes a wave's accesses in program order)
    __builtin_amdgcn_wave_barrier();
#if RS2_EARLY
    if (it + 1 < RS2_TILES && tt + 16 < len) request(tt + 16);   // (in flight during the products)
#endif

#pragma unroll
    for (int ph = 0; ph < G / 2; ++ph) {
      // ---- H_128 of heads 2 ph and 2 ph + 1
      v4f acc[2][8];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int h = 2 * ph + hh;
        const uint4 cwp = ph == 0 ? cw0 : cw1;
        const uint32_t wd[2] = {hh ? cwp.z : cwp.x, hh ? cwp.w : cwp.y};
        const uint4 chp = ph == 0 ? ch0 : ch1;
        // upper plane: two dwords like the lower one's (4-bit codes), or the pair's dword of third bits
        const uint32_t wdh[2] = {HB == 1 ? (hh ? chp.y : chp.x) : (hh ? chp.z : chp.x), HB == 1 ? (hh ? chp.y : chp.x) : (hh ? chp.w : chp.y)};
        const uint4* gp = reinterpret_cast<const uint4*>(s_g4 + wave * (4 * G * 8) + (kq * G + h) * 8);
        const uint4 gA = gp[0], gB = gp[1];
        const uint32_t g4w[8] = {gA.x, gA.y, gA.z, gA.w, gB.x, gB.y, gB.z, gB.w};
#if RS2_HALVES
        v4f wpart[2][4];
#endif
#pragma unroll
        for (int sh = 0; sh < 8; sh += RS2_LOOK) {         // look-ups of RS2_LOOK steps, then their products
#pragma unroll
         for (int pl = 0; pl < NPL; ++pl) {                // (wider codes: the plane of the low two bits, then the upper one)
          uint32_t bv[RS2_LOOK][4];
#pragma unroll
          for (int sl = 0; sl < RS2_LOOK; ++sl) {
            const int s = sh + sl, dw = s >> 2, ksh = s & 3;
            // LDS byte address of (block, code, token) = (table >> 8 + block) << 8 | code << 6 | token << 2: the low bytes of four
            // channels at once, then one byte permute per channel puts the block above
            uint32_t low4 = ((wd[dw] << (6 - 2 * ksh)) & 0xC0C0C0C0u) | tokrep;
            uint32_t gw = g4w[s];
            if (UPPER || pl == 1) {
              if (pl == 1) gw += (uint32_t)NG * 0x01010101u;   // the table's upper half
              if constexpr (HB == 2) low4 = ((wdh[dw] << (6 - 2 * ksh)) & 0xC0C0C0C0u) | tokrep;
              // third bit of code m = 4 j + ksh of dword dw: bit 8 j + 4 (ksh >> 1) + 2 dw + (ksh & 1) of the pair's dword
              else low4 = (((wdh[dw] >> (4 * (ksh >> 1) + 2 * dw + (ksh & 1))) & 0x01010101u) << 6) | tokrep;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const uint32_t addr = __builtin_amdgcn_perm(gw, low4, 0x0c0c0000u | ((4u + j) << 8) | j);
              bv[sl][j] = *reinterpret_cast<const rs2_lds_u32*>((uintptr_t)addr);
            }
          }
#pragma unroll
          for (int sl = 0; sl < RS2_LOOK; ++sl) {
            const int s = sh + sl, dw = s >> 2, ksh = s & 3;
            const v8h B = row_v8h(bv[sl][0], bv[sl][1], bv[sl][2], bv[sl][3]);
#if RS2_HALVES
            // the steps of either dword onto four partial tiles (bits 3, 0 of the tile against ksh & 1, ksh >> 1)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
              const int neg = (((bb >> 1) & (ksh & 1)) ^ ((bb & 1) & (ksh >> 1))) & 1;
              const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
              wpart[dw][bb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(neg ? A_neg : A_pos, B, (ksh == 0 && pl == 0) ? zero4 : wpart[dw][bb], 0, 0, 0);
            }
#else
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
              // input bits 4, 3, 0 = dw, ksh & 1, ksh >> 1 against the tile's bits 4, 3, 0 = mt >> 2, (mt >> 1) & 1, mt & 1
              const int neg = (((mt >> 2) & dw) ^ (((mt >> 1) & 1) & (ksh & 1)) ^ ((mt & 1) & (ksh >> 1))) & 1;
              const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
              acc[hh][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(neg ? A_neg : A_pos, B, (s == 0 && pl == 0) ? zero4 : acc[hh][mt], 0, 0, 0);
            }
#endif
          }
         }
        }
#if RS2_HALVES
        // bit 4 of the tile against the dword: the last stage of the transform in the lane
#pragma unroll
        for (int mt = 0; mt < 8; ++mt)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            acc[hh][mt][r] = (mt >> 2) ? wpart[0][mt & 3][r] - wpart[1][mt & 3][r] : wpart[0][mt & 3][r] + wpart[1][mt & 3][r];
#endif
      }
      // ---- first stage of H_g, RoPE at the token's position
#pragma unroll
      for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float x0 = acc[0][mt][r], x1 = acc[1][mt][r];
          acc[0][mt][r] = x0 + x1;
          acc[1][mt][r] = x0 - x1;
        }
#pragma unroll
      for (int pi = 0; pi < 2; ++pi) {
        if constexpr (STYLE == 0) {
          // pairs (j, j + 64): rows 2 r1 and 2 r1 + 1 of a tile; angle piece r1 of the tile's group mq, entry mt & 1
#pragma unroll
          for (int mt = 0; mt < 8; ++mt)
#pragma unroll
            for (int r1 = 0; r1 < 2; ++r1) {
              const float4 a4 = ang[mt >> 1][r1];
              const float c = (mt & 1) ? a4.z : a4.x, s = (mt & 1) ? a4.w : a4.y;
              const float x = acc[pi][mt][2 * r1], y = acc[pi][mt][2 * r1 + 1];
              acc[pi][mt][2 * r1] = x * c - y * s;
              acc[pi][mt][2 * r1 + 1] = x * s + y * c;
            }
        } else {
          // pairs (2 j, 2 j + 1): tiles mt and mt + 1 (mt even); angle piece r & 1, entry r >> 1
#pragma unroll
          for (int mt = 0; mt < 8; mt += 2)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float4 a4 = ang[mt >> 1][r & 1];
              const float c = (r >> 1) ? a4.z : a4.x, s = (r >> 1) ? a4.w : a4.y;
              const float x = acc[pi][mt][r], y = acc[pi][mt + 1][r];
              acc[pi][mt][r] = x * c - y * s;
              acc[pi][mt + 1][r] = x * s + y * c;
            }
        }
      }
      // ---- dots with the queries of the output heads a = pi, pi + 2 (second stage of H_g: sign -1 for a >= 2 in the second phase)
      for (int rq = 0; rq < rep; ++rq) {
#pragma unroll
        for (int pi = 0; pi < 2; ++pi)
#pragma unroll
          for (int ah = 0; ah < G / 2; ++ah) {
            const int a = 2 * ah + pi;
            // this lane's share of the query row: channels of tiles mt = 2 qu, 2 qu + 1
            const float* qrow = s_qp + (a * rep + rq) * RKV_D + 32 * g4hi + 16 * (qu >> 1) + 8 * (qu & 1) + 4 * g4lo;
            float qv[2][4];
#pragma unroll
            for (int b0 = 0; b0 < 2; ++b0)
#pragma unroll
              for (int r = 0; r < 4; ++r) qv[b0][r] = qrow[64 * (r & 1) + 2 * (r >> 1) + b0];
            rs2_settle(qv);
            float dd[4];                                   // four chains: no multiply-add reads the result of the one before it
#pragma unroll
            for (int r = 0; r < 4; ++r) dd[r] = fmul_quad<0>(qv[0][r], acc[pi][0][r]);
#pragma unroll
            for (int mt = 1; mt < 8; ++mt)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                if ((mt >> 1) == 0) fmac_quad<0>(dd[r], qv[mt & 1][r], acc[pi][mt][r]);
                if ((mt >> 1) == 1) fmac_quad<1>(dd[r], qv[mt & 1][r], acc[pi][mt][r]);
                if ((mt >> 1) == 2) fmac_quad<2>(dd[r], qv[mt & 1][r], acc[pi][mt][r]);
                if ((mt >> 1) == 3) fmac_quad<3>(dd[r], qv[mt & 1][r], acc[pi][mt][r]);
              }
            float d = (dd[0] + dd[1]) + (dd[2] + dd[3]);
            d += __shfl_xor(d, 16);
            d += __shfl_xor(d, 32);
            if (kq == 0) {
              float* slot = s_pd + (a * rep + rq) * 16 + tok;
              if (ph == 0) *slot = d;
              else *slot = (ah & ph) ? *slot - d : *slot + d;
            }
          }
      }
    }
#if !RS2_EARLY
    if (it + 1 < RS2_TILES && tt + 16 < len) request(tt + 16);
#endif
    asm volatile("" ::: "memory");                        // (the LDS unit takes a wave's accesses in program order)
    __builtin_amdgcn_wave_barrier();
    // ---- the tile's scores; retained sink tokens are masked out of the stream
    for (int i = lane; i < nqh * 16; i += 64) {
      const int hr = i >> 4, tk = tt + (i & 15);
      if (tk < len) {
        bool sink = false;
        for (int k = 0; k < cnt; ++k) sink |= (s_sink[k] == tk);
        float* srow = sc + ((size_t)b * v.Hq + (size_t)rg * nqh) * v.Tpad + tt;
        float* dst = &srow[(uint32_t)(hr * v.Tpad + (i & 15))];
        *dst = sink ? -INFINITY : ((UPPER || (PART && padd)) ? *dst + s_pd[i] * out_scale : s_pd[i] * out_scale);
      }
    }
  }
}

static size_t row2_lds_of(const RkvView& v, int NG) {
  const int nqh = v.g * (v.Hq / v.Hkv);
  return (size_t)4 * NG * 256 + (size_t)4 * nqh * 64 + (size_t)nqh * RKV_D * 4 + (size_t)4 * 4 * v.g * 8 * 4 + 256;
}
// A whole-row reorder with groups of 64 / 32: the row's E / quant_group blocks go to the scores kernel in shares of
// at most RS2_PART_MAX (each share a launch, with an all-zero block behind its own in the table).
#define RS2_PART_MAX 40
static int row2_parts(const RkvView& v) { return v.qg < 128 ? (v.NG + RS2_PART_MAX - 1) / RS2_PART_MAX : 1; }
static int row2_part_blocks(const RkvView& v) { const int np = row2_parts(v); return (v.NG + np - 1) / np; }
static size_t row2_dynamic_lds(const RkvView& v, bool local) {
  // (wider codes, own blocks: a table half per plane; shares of the row's blocks: the all-zero block besides)
  return row2_lds_of(v, local ? v.gm * (v.hb ? 2 : 1) : v.qg < 128 ? row2_part_blocks(v) + 1 : v.E >> 7);
}
static bool row2_applies(const RkvView& v) {
  if (v.qg < 128) return v.NG <= 4095 && row2_dynamic_lds(v, false) + 1024 <= (size_t)RKV_LDS_BYTES / 2;
  return (v.E >> 7) <= RS2_MAX_NG && row2_dynamic_lds(v, false) + 1024 <= (size_t)RKV_LDS_BYTES / 2;
}

// Whether a cache takes this path: a reorder that leaves the rotation groups (else the plain kernel or
// rkv_scores_local's route serves it), rot_heads 2 or 4 (8-bit metadata, wider codes and groups of 64 / 32 where
// the table-per-wave kernel applies).
static size_t row_dynamic_lds(const RkvView& v) {
  const int nqh = v.g * (v.Hq / v.Hkv), NG = v.E >> 7;
  return (size_t)16 * (NG | 1) * 16 + (size_t)nqh * RKV_D * 4 + (size_t)4 * nqh * 16 * 4;
}

bool rkv_row_supported(const rkv_cache* c) {
  const RkvView& v = c->v;
  if (c->blocks_aligned || c->in_groups || !(v.g == 2 || v.g == 4)) return false;
  if (v.qg < 128) return row2_applies(v);                   // (groups of 64 / 32: the table-per-wave kernel, a share of the blocks per launch)
  if ((v.meta8 || v.hb) && !row2_applies(v)) return false; // (8-bit metadata, wider codes: the table-per-wave kernel only)
  // two workgroups per compute unit must fit its LDS; a tile's metadata: at most 32 rotation groups
  const size_t fixed = (size_t)2 * 16 * (16 * v.g + 1) * 16 + (size_t)144 * v.g * 4 + 256;
  return row_dynamic_lds(v) + fixed <= 80 * 1024 && v.NRG <= 32;
}

// Groups of 64 / 32, and a reorder across 128-blocks inside the rotation groups (with either group size),
// take the same route (scores from k_scores_row2 with the rotation group's own
// blocks in the table, then the softmax and value phases of the matrix-core kernel): key phases of
// masked passes over the blocks, the first design, cost more (measured on config 2's geometry:
// 177, 292 and 160 us against 162, 175 and 153).
bool rkv_scores_local(const rkv_cache* c) {
  const RkvView& v = c->v;
  const bool sub = (c->blocks_aligned || c->in_groups) && v.qg < 128;       // (2-, 3- or 4-bit codes)
  const bool cross = !c->blocks_aligned && c->in_groups && v.qg == 128;
  return (sub || cross) && (v.g == 2 || v.g == 4) && row2_dynamic_lds(v, true) + 1024 <= (size_t)RKV_LDS_BYTES / 2;
}
bool rkv_scores_path(const rkv_cache* c) { return rkv_row_supported(c) || rkv_scores_local(c); }

size_t rkv_row_scores_bytes(int batch, int n_q_heads, int max_tokens) {
  const size_t Tpad = ((size_t)max_tokens + 255) & ~(size_t)255;
  return (size_t)batch * n_q_heads * Tpad * 4;
}

// Several query tokens per step: the scores kernel sees them as further query heads of a KV head (virtual
// heads, as the matrix-core kernel does); it serves up to 8 rows per KV head, in its table-per-wave form.
bool rkv_scores_multi_ok(const rkv_cache* c, int n_queries) {
  if (!rkv_scores_path(c)) return false;
  RkvView v = c->v;
  v.Hq *= n_queries;
  if (v.Hq / v.Hkv > 8) return false;
  const bool local = rkv_scores_local(c);
  if (!local && !row2_applies(v)) return false;
  return row2_dynamic_lds(v, local) + 1024 <= (size_t)RKV_LDS_BYTES / 2;
}

// scores of every cached token for every query head of `v` (prepared queries qr)
// v: the cache's view, with virtual heads where several query tokens are served
int rkv_launch_scores_row(const rkv_cache* c, const RkvView& v, const float* qr, float* sc, hipStream_t s) {
  if (!rkv_scores_path(c)) return RKV_EINVAL;
  const int rep = v.Hq / v.Hkv;
  if (v.len == 0) return RKV_OK;
  const bool local = rkv_scores_local(c);
  if (local || row2_applies(v)) {
    const size_t dyn = row2_dynamic_lds(v, local);
    dim3 grid((v.len + RS2_CHUNK - 1) / RS2_CHUNK, v.NRG, v.B);
    typedef void (*ScoresFn)(RkvView, const float*, float*, int, int);
    // (G, RoPE pairing) x (own blocks, planes of code bits, a share of the row's blocks)
#define RS2_FN_GS(L_, H_, P_)                                                                                       \
  (v.g == 4 ? (v.rope_style == 0 ? (ScoresFn)k_scores_row2<4, 0, L_, H_, P_> : (ScoresFn)k_scores_row2<4, 1, L_, H_, P_>) \
            : (v.rope_style == 0 ? (ScoresFn)k_scores_row2<2, 0, L_, H_, P_> : (ScoresFn)k_scores_row2<2, 1, L_, H_, P_>))
    auto launch = [&](ScoresFn fn, int part) -> int {
      if (dyn > 48 * 1024) RKV_HIP_CHECK(hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn));
      hipLaunchKernelGGL(fn, grid, dim3(256), dyn, s, v, qr, sc, rep, part);
      return RKV_OK;
    };
    int rc = RKV_OK;
    if (local) {
      rc = launch(v.hb == 2 ? RS2_FN_GS(true, 2, false) : v.hb == 1 ? RS2_FN_GS(true, 1, false) : RS2_FN_GS(true, 0, false), 0);
    } else if (v.qg == 128) {
      rc = launch(RS2_FN_GS(false, 0, false), 0);
      // the plane of upper bits: a launch of its own, onto the same scores
      if (rc == RKV_OK && v.hb) rc = launch(v.hb == 2 ? RS2_FN_GS(false, 2, false) : RS2_FN_GS(false, 1, false), 0);
    } else {
      // groups of 64 / 32: a launch per share of the row's blocks (and per plane of code bits), all onto the same scores
      const int np = row2_parts(v), per = row2_part_blocks(v);
      for (int p = 0; p < np && rc == RKV_OK; ++p) {
        const int b0 = p * per, cnt = (b0 + per <= v.NG ? per : v.NG - b0);
        rc = launch(RS2_FN_GS(false, 0, true), b0 | (cnt << 12) | ((p > 0 ? 1 : 0) << 24));
        if (rc == RKV_OK && v.hb)
          rc = launch(v.hb == 2 ? RS2_FN_GS(false, 2, true) : RS2_FN_GS(false, 1, true), b0 | (cnt << 12) | (1 << 24));
      }
    }
#undef RS2_FN_GS
    if (rc != RKV_OK) return rc;
    return rkv_check_launch();
  }
  const size_t dyn = row_dynamic_lds(v);
  const int nch = (v.len + RKV_ROW_CHUNK - 1) / RKV_ROW_CHUNK;
  dim3 grid(nch, v.NRG, v.B);
  if (v.g == 4) {
    if (v.rope_style == 0) hipLaunchKernelGGL((k_scores_row<4, 0>), grid, dim3(256), dyn, s, v, qr, sc, rep);
    else hipLaunchKernelGGL((k_scores_row<4, 1>), grid, dim3(256), dyn, s, v, qr, sc, rep);
  } else {
    if (v.rope_style == 0) hipLaunchKernelGGL((k_scores_row<2, 0>), grid, dim3(256), dyn, s, v, qr, sc, rep);
    else hipLaunchKernelGGL((k_scores_row<2, 1>), grid, dim3(256), dyn, s, v, qr, sc, rep);
  }
  return rkv_check_launch();
}

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

// Whether a cache takes this path: a reorder that leaves the rotation groups (else the plain or the
// cross-block kernel serves it), 2-bit codes in groups of 128 with fp16 metadata, rot_heads 2 or 4.
static size_t row_dynamic_lds(const RkvView& v) {
  const int nqh = v.g * (v.Hq / v.Hkv), NG = v.E >> 7;
  return (size_t)16 * (NG | 1) * 16 + (size_t)nqh * RKV_D * 4 + (size_t)4 * nqh * 16 * 4;
}

bool rkv_row_supported(const rkv_cache* c) {
  const RkvView& v = c->v;
  if (c->blocks_aligned || c->in_groups || v.qg != 128 || v.hb != 0 || v.meta8 || !(v.g == 2 || v.g == 4)) return false;
  // two workgroups per compute unit must fit its LDS; a tile's metadata: at most 32 rotation groups
  const size_t fixed = (size_t)2 * 16 * (16 * v.g + 1) * 16 + (size_t)144 * v.g * 4 + 256;
  return row_dynamic_lds(v) + fixed <= 80 * 1024 && v.NRG <= 32;
}

size_t rkv_row_scores_bytes(int batch, int n_q_heads, int max_tokens) {
  const size_t Tpad = ((size_t)max_tokens + 255) & ~(size_t)255;
  return (size_t)batch * n_q_heads * Tpad * 4;
}

// scores of every cached token for every query head of `v` (one query token per sequence, prepared queries qr)
int rkv_launch_scores_row(const rkv_cache* c, const float* qr, float* sc, hipStream_t s) {
  const RkvView& v = c->v;
  if (!rkv_row_supported(c)) return RKV_EINVAL;
  const int rep = v.Hq / v.Hkv;
  const size_t dyn = row_dynamic_lds(v);
  const int nch = (v.len + RKV_ROW_CHUNK - 1) / RKV_ROW_CHUNK;
  if (nch == 0) return RKV_OK;
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

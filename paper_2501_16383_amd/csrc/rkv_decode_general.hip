// Read half, general kernel: any supported configuration, plain vector ALU.
//   k_prep_q        RoPE of the query at q_pos, scaled by 1/sqrt(d)                 (Eq. 5)
//   k_decode_gen    split-K over the context: one workgroup = (sequence, rotation group, chunk)
//                   dequantize -> inverse reorder (gid) -> inverse rotation -> RoPE -> scores,
//                   chunk-local softmax, p.V on the 2-bit values; writes (m, l, acc) partials
//   k_merge         combines the partials with the fp16 sink rows (Sec. 4.3) -> out, lse
#include "rkv_internal.h"
#include "rkv_prep_q.h"

#define GEN_CHUNK RKV_GEN_CHUNK

template <int PL, typename T>
__device__ inline void fwht_lanes_d(T (&x)[PL], int lane, int xstages) {
#pragma unroll
  for (int h = 1; h < PL; h <<= 1) {
#pragma unroll
    for (int i = 0; i < PL; i += 2 * h) {
#pragma unroll
      for (int j = i; j < i + h; ++j) {
        T a = x[j], b = x[j + h];
        x[j] = a + b;
        x[j + h] = a - b;
      }
    }
  }
  for (int s = 0; s < xstages; ++s) {
    const int mask = 1 << s;
    const bool up = (lane & mask) != 0;
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      T o = __shfl_xor(x[i], mask);
      x[i] = up ? (o - x[i]) : (x[i] + o);
    }
  }
}

__global__ void __launch_bounds__(128) k_prep_q(RkvView v, const __half* __restrict__ q, const int* __restrict__ q_pos,
                                                int cur, float* __restrict__ qr, int share, int nq) {
  rkv_prep_q_one(v, q, q_pos, cur, qr, share, nq, blockIdx.x, blockIdx.y, threadIdx.x);
}

__device__ inline bool is_sink(const int* sp, int cnt, int t) {
  bool s = false;
  for (int i = 0; i < cnt; ++i) s |= (sp[i] == t);
  return s;
}

// WIDE: codes of 3 or 4 bits (a second plane of bits is read)
// q_lim, nqt: several query tokens per sequence (else null, 1): v.Hq then counts virtual heads (nqt per
// real head, see rkv_virtual_head) and a virtual head only attends tokens at positions <= q_lim[b][its token]
template <int PL, bool WIDE>
__global__ void __launch_bounds__(256) k_decode_gen(RkvView v, const float* __restrict__ qr, float* __restrict__ part, int nch,
                                                    const int* __restrict__ q_lim, int nqt) {
  // LDS: q~ of this group's query heads, scores / probabilities, V meta, per-head stats
  extern __shared__ float sm[];
  const int rep = v.Hq / v.Hkv, g = v.g, n = v.n;
  const int nq = rep * g;                       // query heads served by this rotation group
  float* s_q = sm;                              // [nq][128]
  float* s_p = s_q + nq * RKV_D;                // [nq][GEN_CHUNK]
  const int gm = v.gm;                          // quantization blocks of the group's n channels
  float* s_vs = s_p + nq * GEN_CHUNK;           // [gm][GEN_CHUNK]
  float* s_vz = s_vs + gm * GEN_CHUNK;          // [gm][GEN_CHUNK]
  float* s_m = s_vz + gm * GEN_CHUNK;           // [nq]
  float* s_l = s_m + nq;                        // [nq]
  __shared__ int s_sink[64];

  const int chunk = blockIdx.x, rg = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = chunk * GEN_CHUNK, t1 = min(t0 + GEN_CHUNK, rkv_len(v, b));
  if (t0 >= t1) return;                              // the grid covers the longest sequence
  const int cnt = v.max_sinks > 0 ? v.sink_cnt[b] : 0;
  if (tid < 64) s_sink[tid] = tid < cnt ? v.sink_pos[b * v.max_sinks + tid] : -1;
  for (int i = tid; i < nq * RKV_D; i += 256) s_q[i] = qr[((size_t)b * v.Hq + (size_t)rg * nq) * RKV_D + i];
  __syncthreads();

  // ---- phase 1: scores.  One wave per token; lane holds rotated channels PL*lane .. +PL-1.
  const int lanes_per_head = RKV_D / PL;
  const int hh = lane / lanes_per_head;                       // KV head inside the group
  const int idx0 = (PL * lane) & (RKV_D - 1);                 // first channel inside the head
  const float rs = rsqrtf((float)n);
  // What does not depend on the token: a lane's PL consecutive rotated channels share one dword of
  // a K tile (the layout keeps 16 aligned channels of a token together), at a fixed offset and with
  // fixed shifts; each channel's quantization block, hence the place of its metadata in a token's row.
  int sh[PL];
  size_t mi0[PL];
  int dw_off = 0;
#pragma unroll
  for (int i = 0; i < PL; ++i) {
    const int c = PL * lane + i;
    const int off = rkv_k_off(g, 0, c, sh[i]);
    if (i == 0) dw_off = off;
    mi0[i] = rkv_meta_index(v, b, 0, v.gid[rg * n + c]);
  }
  const int tok_stride = g == 1 ? 2 : 4;                       // dwords between consecutive tokens of a tile
  // bits above the low two (wider codes).  4-bit codes: a second plane, same dword and shifts;
  // 3-bit codes: the third bits sit in the dword that belongs to the lane's dword and its
  // neighbour, at places that follow from the shifts (rkv_h1_loc)
  const int hb = WIDE ? v.hb : 0;
  int hsh[PL];
#pragma unroll
  for (int i = 0; i < PL; ++i) {
    hsh[i] = sh[i];
    if (hb == 1) rkv_h1_loc((size_t)dw_off, sh[i], hsh[i]);
  }
  for (int t = t0 + wave; t < t1; t += 4) {
    float x[PL];
    const uint32_t w = v.kc[rkv_k_tilebase(v, b, rg, t >> 4) + dw_off + (t & 15) * tok_stride];
    uint32_t hw = 0u;
    if (hb == 2) hw = v.kh[rkv_k_tilebase(v, b, rg, t >> 4) + dw_off + (t & 15) * tok_stride];
    else if (hb == 1) hw = v.kh[(rkv_k_tilebase(v, b, rg, t >> 4) + dw_off + (t & 15) * tok_stride) >> 1];
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      float sc, zero;
      rkv_load_meta(v, v.km, mi0[i] + (size_t)t * gm, sc, zero);
      const uint32_t hi = (hw >> hsh[i]) & (hb == 2 ? 3u : (uint32_t)hb);
      x[i] = sc * ((float)(((w >> sh[i]) & 3u) | (hi << 2)) - zero);          // Eq. 7
    }
    fwht_lanes_d<PL>(x, lane, 6);                               // inverse rotation (H is its own inverse)
    float y[PL];
    if (v.rope_style == 0) {
      const float sgn = idx0 < 64 ? -1.f : 1.f;
#pragma unroll
      for (int i = 0; i < PL; ++i) {
        const float p = __shfl_xor(x[i], 64 / PL);
        const float2 cs = v.rope[(size_t)t * 64 + ((idx0 + i) & 63)];
        y[i] = rs * (x[i] * cs.x + sgn * p * cs.y);
      }
    } else {
#pragma unroll
      for (int i = 0; i < PL; i += 2) {
        const float2 cs = v.rope[(size_t)t * 64 + ((idx0 + i) >> 1)];
        y[i] = rs * (x[i] * cs.x - x[i + 1] * cs.y);
        y[i + 1] = rs * (x[i] * cs.y + x[i + 1] * cs.x);
      }
    }
    const bool sink = is_sink(s_sink, cnt, t);
    for (int r = 0; r < rep; ++r) {
      const float* qh = s_q + (hh * rep + r) * RKV_D + idx0;
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < PL; ++i) d += y[i] * qh[i];
      for (int s = 1; s < lanes_per_head; s <<= 1) d += __shfl_xor(d, s);
      // (virtual head r of a KV head belongs to query token r / (real heads per KV head))
      const bool hidden = sink || (q_lim && t > q_lim[b * nqt + r / (rep / nqt)]);
      if ((lane & (lanes_per_head - 1)) == 0) s_p[(hh * rep + r) * GEN_CHUNK + (t - t0)] = hidden ? -INFINITY : d;
    }
  }
  for (int i = tid; i < gm * GEN_CHUNK; i += 256) {
    const int h = i / GEN_CHUNK, tt = i - h * GEN_CHUNK;
    float sc = 0.f, zero = 0.f;
    if (t0 + tt < t1) rkv_load_meta(v, v.vm, rkv_meta_index(v, b, t0 + tt, rg * gm + h), sc, zero);
    s_vs[i] = sc;
    s_vz[i] = zero;
  }
  __syncthreads();

  // ---- phase 2: chunk-local softmax per query head
  for (int h = wave; h < nq; h += 4) {
    float* p = s_p + h * GEN_CHUNK;
    float m = -INFINITY;
    for (int tt = lane; tt < t1 - t0; tt += 64) m = fmaxf(m, p[tt]);
    for (int s = 1; s < 64; s <<= 1) m = fmaxf(m, __shfl_xor(m, s));
    float l = 0.f;
    for (int tt = lane; tt < GEN_CHUNK; tt += 64) {
      float e = 0.f;
      if (tt < t1 - t0 && m > -INFINITY) e = __expf(p[tt] - m);
      p[tt] = e;
      l += e;
    }
    for (int s = 1; s < 64; s <<= 1) l += __shfl_xor(l, s);
    if (lane == 0) {
      s_m[h] = m;
      s_l[h] = l;
    }
  }
  __syncthreads();

  // ---- phase 3: acc[c] = sum_t p_t * s_t * (code - zero)   (Eq. 7 folded into the weights)
  for (int c = tid; c < n; c += 256) {
    const int h = c >> 7, blk = c / v.qg;
    float acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) acc[r] = 0.f;
    for (int tt = 0; tt < t1 - t0; tt += 16) {
      int sh;
      const size_t wi = rkv_v_dword(v, b, rg, t0 + tt, c, sh);
      const uint32_t w = v.vc[wi], w2 = hb == 2 ? v.vh[wi] : (hb == 1 ? v.vh[wi >> 1] : 0u);
      for (int k = 0; k < 16 && tt + k < t1 - t0; ++k) {
        uint32_t code = (w >> rkv_v_shift(k)) & 3u;
        if (hb == 2) code |= ((w2 >> rkv_v_shift(k)) & 3u) << 2;
        else if (hb == 1) {
          int bit;
          rkv_h1_loc(wi, rkv_v_shift(k), bit);
          code |= ((w2 >> bit) & 1u) << 2;
        }
        const float val = s_vs[blk * GEN_CHUNK + tt + k] * ((float)code - s_vz[blk * GEN_CHUNK + tt + k]);
#pragma unroll
        for (int r = 0; r < 8; ++r)
          if (r < rep) acc[r] += s_p[(h * rep + r) * GEN_CHUNK + tt + k] * val;
      }
    }
    for (int r = 0; r < rep; ++r) {
      const int qh = rg * nq + h * rep + r;
      float* dst = part + (((size_t)b * v.Hq + qh) * nch + chunk) * RKV_PART_STRIDE;
      dst[4 + (c & 127)] = acc[r];
      if ((c & 127) == 0) {
        dst[0] = s_m[h * rep + r];
        dst[1] = s_l[h * rep + r];
      }
    }
  }
}

// One workgroup per (query head, sequence); thread = output channel.  All global loads whose
// addresses do not depend on loaded data are issued up front (two dependent round trips in all).
// NGRP groups of 128 threads share the chunks (long contexts: with 128 chunks a single group spends
// its time waiting for one batch of partial sums after the other); group 0 also does everything
// that is not per chunk, and adds up the groups' sums at the end.
#define MERGE_MAX_CH 512
template <int NGRP>
__global__ void __launch_bounds__(128 * NGRP) k_merge(RkvView v, const float* __restrict__ qr, const float* __restrict__ part,
                                                      int nch_all, int chunk_tokens, const __half* __restrict__ k_cur,
                                                      const __half* __restrict__ v_cur, const int* __restrict__ q_lim, int nq,
                                                      float* __restrict__ out, float* __restrict__ lse) {
  __shared__ float s_w[MERGE_MAX_CH];     // chunk maxima, then chunk weights
  __shared__ float s_l[MERGE_MAX_CH];
  __shared__ float s_part[2][64];         // per-wave partial sink scores
  __shared__ float s_score[64];
  __shared__ float s_cur[2];
  __shared__ float red[128];
  __shared__ float s_accg[NGRP][128], s_Lg[NGRP];
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int grp = NGRP > 1 ? tid >> 7 : 0, c = tid & 127, lane = c & 63, wave = c >> 6;
  const bool lead = grp == 0;
  const int kvh = h / (v.Hq / v.Hkv);
  const size_t qbase = ((size_t)b * v.Hq + h) * RKV_D;
  // partials are laid out for nch_all chunks (the longest sequence); this sequence wrote its first nch
  const int len_b = rkv_len(v, b);
  const int nch = min(nch_all, (len_b + chunk_tokens - 1) / chunk_tokens);
  const float* P = part + ((size_t)b * v.Hq + h) * nch_all * RKV_PART_STRIDE;
  const int cnt = v.max_sinks > 0 ? v.sink_cnt[b] : 0;
  // with several query tokens (q_lim set) a query only sees tokens up to its own position
  const RkvVHead vh = rkv_virtual_head(v, h, nq);
  const int lim = q_lim ? min(q_lim[b * nq + vh.qi], len_b - 1) : len_b - 1;
  // this group's chunks
  const int per = (nch + NGRP - 1) / NGRP, k_lo = min(grp * per, nch), k_hi = min(k_lo + per, nch);

  for (int k = tid; k < nch; k += 128 * NGRP) {
    s_w[k] = P[(size_t)k * RKV_PART_STRIDE];
    s_l[k] = P[(size_t)k * RKV_PART_STRIDE + 1];
  }
  // scores of the retained sink rows: exact fp16 keys, RoPE at their own position
  int j, partner;
  float sgn;
  if (v.rope_style == 0) { j = c & 63; partner = c ^ 64; sgn = c < 64 ? -1.f : 1.f; }
  else { j = c >> 1; partner = c ^ 1; sgn = (c & 1) ? 1.f : -1.f; }
  const float qc = qr[qbase + c];
  // the first partial sums of this channel are requested now: they do not depend on anything
  // computed here, and the latency of the sink rows below hides theirs
  constexpr int PRE = 16;
  float pv[PRE];
#pragma unroll
  for (int k = 0; k < PRE; ++k) pv[k] = k_lo + k < k_hi ? P[(size_t)(k_lo + k) * RKV_PART_STRIDE + 4 + c] : 0.f;
  // Sink rows four at a time, so that their loads overlap.  Row indices are clamped to the store's
  // capacity, not to the count of retained rows: the first group's loads then do not wait for that
  // count to arrive (slots never written hold position 0 and zeros; their scores are not used).
  const int smax = v.max_sinks > 0 ? v.max_sinks - 1 : 0;
  // the value rows of the first four sinks are requested here as well, long before they are used
  float sv[4] = {0.f, 0.f, 0.f, 0.f};
  if (lead) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      sv[i] = __half2float(v.sink_v[((size_t)b * v.max_sinks + min(i, smax)) * v.E + (size_t)kvh * RKV_D + c]);
  }
  auto sink_group = [&](int s0) {
    float d[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int s = min(s0 + i, smax);
      const int pos = v.sink_pos[b * v.max_sinks + s];
      const __half* kr = v.sink_k + ((size_t)b * v.max_sinks + s) * v.E + (size_t)kvh * RKV_D;
      const float2 cs = v.rope[(size_t)pos * 64 + j];
      const float x = __half2float(kr[c]), p = __half2float(kr[partner]);
      d[i] = qc * (x * cs.x + sgn * p * cs.y);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      for (int o = 32; o > 0; o >>= 1) d[i] += __shfl_xor(d[i], o);
      if (lane == 0 && s0 + i < cnt) s_part[wave][s0 + i] = v.sink_pos[b * v.max_sinks + s0 + i] <= lim ? d[i] : -INFINITY;
    }
  };
  if (lead) {                                                // whole waves: a group is two of them
    if (v.max_sinks > 0) sink_group(0);
    for (int s0 = 4; s0 < cnt; s0 += 4) sink_group(s0);
  }
  // the token being decoded, if it is attended in full precision: an exact row at position len
  // (which may lie one past the angle table, so its angles are computed here)
  float cur_score = -INFINITY;
  if (k_cur && lead) {
    const __half* kr = k_cur + ((size_t)b * v.Hkv + kvh) * RKV_D;
    double sn, cs;
    sincos((double)len_b * pow((double)v.theta, -(double)j / 64.0), &sn, &cs);
    const float x = __half2float(kr[c]), p = __half2float(kr[partner]);
    float d = qc * (x * (float)cs + sgn * p * (float)sn);
    for (int o = 32; o > 0; o >>= 1) d += __shfl_xor(d, o);
    if (lane == 0) s_cur[wave] = d;
  }
  __syncthreads();
  if (lead && c < cnt) s_score[c] = s_part[0][c] + s_part[1][c];
  if (k_cur) cur_score = s_cur[0] + s_cur[1];
  __syncthreads();

  float M = -INFINITY;
  for (int k = 0; k < nch; ++k) M = fmaxf(M, s_w[k]);
  for (int s = 0; s < cnt; ++s) M = fmaxf(M, s_score[s]);
  M = fmaxf(M, cur_score);
  float L = 0.f, acc = 0.f;
#pragma unroll
  for (int k = 0; k < PRE; ++k) {
    if (k_lo + k < k_hi) {
      const float mk = s_w[k_lo + k];
      const float w = mk > -INFINITY ? __expf(mk - M) : 0.f;
      L += w * s_l[k_lo + k];
      acc += w * pv[k];                                      // partial sums are always finite
    }
  }
  for (int k0 = k_lo + PRE; k0 < k_hi; k0 += 8) {            // longer contexts: eight loads in flight at a time
    float pw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pw[i] = k0 + i < k_hi ? P[(size_t)(k0 + i) * RKV_PART_STRIDE + 4 + c] : 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (k0 + i < k_hi) {
        const float mk = s_w[k0 + i];
        const float w = mk > -INFINITY ? __expf(mk - M) : 0.f;
        L += w * s_l[k0 + i];
        acc += w * pw[i];
      }
    }
  }
  if constexpr (NGRP > 1) {                                  // group 0 takes the other groups' sums
    s_accg[grp][c] = acc;
    if (c == 0) s_Lg[grp] = L;
    __syncthreads();
    if (lead) {
#pragma unroll
      for (int g2 = 1; g2 < NGRP; ++g2) {
        acc += s_accg[g2][c];
        L += s_Lg[g2];
      }
    }
  }
  if (v.v_rotate) {   // the 2-bit stream holds rotated values: undo the per-head Hadamard once
    if (lead) red[c] = acc;
    __syncthreads();
    for (int hstep = 1; hstep < 128; hstep <<= 1) {
      float a = 0.f, o = 0.f;
      if (lead) { a = red[c]; o = red[c ^ hstep]; }
      __syncthreads();
      if (lead) red[c] = (c & hstep) ? (o - a) : (a + o);
      __syncthreads();
    }
    if (lead) acc = red[c] * 0.08838834764831845f;
  }
  if (!lead) return;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    if (s < cnt) {
      const float w = s_score[s] > -INFINITY ? __expf(s_score[s] - M) : 0.f;
      L += w;
      acc += w * sv[s];
    }
  }
  for (int s = 4; s < cnt; ++s) {
    const float w = s_score[s] > -INFINITY ? __expf(s_score[s] - M) : 0.f;
    L += w;
    acc += w * __half2float(v.sink_v[((size_t)b * v.max_sinks + s) * v.E + (size_t)kvh * RKV_D + c]);
  }
  if (k_cur) {
    const float w = __expf(cur_score - M);
    L += w;
    acc += w * __half2float(v_cur[((size_t)b * v.Hkv + kvh) * RKV_D + c]);
  }
  const size_t orow = ((size_t)b * nq + vh.qi) * (v.Hq / nq) + vh.h;        // [batch][query token][real head]
  out[orow * RKV_D + c] = acc / L;
  if (lse && c == 0) lse[orow] = M + logf(L);
}

void rkv_launch_prep_q(const RkvView& v, const __half* q, const int* q_pos, int cur, float* qr, int share, int nq,
                       hipStream_t s) {
  hipLaunchKernelGGL(k_prep_q, dim3(v.Hq, v.B), dim3(128), 0, s, v, q, q_pos, cur, qr, share, nq);
}
void rkv_launch_merge(const RkvView& v, const float* qr, const float* part, int nch, int chunk_tokens, const __half* k_cur,
                      const __half* v_cur, const int* q_lim, int nq, float* out, float* lse, hipStream_t s) {
  // long contexts: share the chunks among four groups of threads (128 chunks: 9 instead of 17 us;
  // at 32 chunks the wider workgroups cost more than they save)
  if (nch > 32) hipLaunchKernelGGL(k_merge<4>, dim3(v.Hq, v.B), dim3(512), 0, s, v, qr, part, nch, chunk_tokens, k_cur, v_cur, q_lim, nq, out, lse);
  else hipLaunchKernelGGL(k_merge<1>, dim3(v.Hq, v.B), dim3(128), 0, s, v, qr, part, nch, chunk_tokens, k_cur, v_cur, q_lim, nq, out, lse);
}

// the split-K partial results of a launch over Tpad token slots (chunks of 128 tokens at the finest)
size_t rkv_partial_bytes(int batch, int n_q_heads, int Tpad) {
  return ((size_t)batch * n_q_heads * (Tpad / 128) * RKV_PART_STRIDE * 4 + 255) & ~(size_t)255;
}

size_t rkv_decode_scratch_bytes(const rkv_config* cfg) {
  const size_t Tpad = (cfg->max_tokens + 255) & ~255;
  size_t bytes = rkv_query_scratch_bytes(cfg->batch, cfg->n_q_heads) + rkv_partial_bytes(cfg->batch, cfg->n_q_heads, (int)Tpad) + 256;
  // a reorder over the whole row: the scores of the compressed stream pass through a buffer (k_scores_row)
  // (and groups of 64 / 32 where they take the same route)
  if (cfg->perm_span > RKV_D || cfg->quant_group < 128) bytes += rkv_row_scores_bytes(cfg->batch, cfg->n_q_heads, cfg->max_tokens);
  return bytes;
}

// n_queries == 0: the usual step.  n_queries >= 1: that many query tokens per sequence, token i at
// position q_pos[b][i] and blind to cached tokens behind it (q, out, lse [batch][n_queries][heads][...];
// the scratch buffer holds n_queries times the single-query size); at most 8 virtual heads per KV head.
int rkv_launch_decode_general(rkv_cache* c, const __half* q, const int* q_pos, int n_queries, float* out, float* lse, void* scratch,
                              hipStream_t s) {
  const bool multi = n_queries > 0;
  if (multi && (c->cur_k || !q_pos)) return RKV_EINVAL;
  const int nqt = multi ? n_queries : 1;
  RkvView v = c->v;
  v.Hq *= nqt;                                              // virtual heads
  if (v.Hq / v.Hkv > 8) return RKV_EINVAL;
  float* qr = (float*)scratch;
  const size_t qbytes = rkv_query_scratch_bytes(v.B, v.Hq);
  float* part = (float*)((char*)scratch + qbytes);
  const int nch = (v.len + GEN_CHUNK - 1) / GEN_CHUNK;
  rkv_launch_prep_q(v, q, q_pos, c->cur_k ? 1 : 0, qr, 1, nqt, s);
  const int rep = v.Hq / v.Hkv, nq = rep * v.g;
  const size_t lds = ((size_t)nq * RKV_D + (size_t)nq * GEN_CHUNK + 2 * (size_t)v.gm * GEN_CHUNK + 2 * nq) * 4;
  dim3 grid(nch, v.NRG, v.B);
  void (*fn)(RkvView, const float*, float*, int, const int*, int) = nullptr;
  switch (v.n / 64) {
    case 2: fn = v.hb ? k_decode_gen<2, true> : k_decode_gen<2, false>; break;
    case 4: fn = v.hb ? k_decode_gen<4, true> : k_decode_gen<4, false>; break;
    case 8: fn = v.hb ? k_decode_gen<8, true> : k_decode_gen<8, false>; break;
    case 16: fn = v.hb ? k_decode_gen<16, true> : k_decode_gen<16, false>; break;
    default: return RKV_EINVAL;
  }
  if (lds > 48 * 1024) RKV_HIP_CHECK(hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  if (c->ev_start) RKV_HIP_CHECK(hipEventRecord(c->ev_start, s));
  if (nch > 0)                                              // (an empty cache has only the current token)
    hipLaunchKernelGGL(fn, grid, dim3(256), lds, s, v, qr, part, nch, multi ? q_pos : (const int*)nullptr, nqt);
  if (c->ev_stop) RKV_HIP_CHECK(hipEventRecord(c->ev_stop, s));
  rkv_launch_merge(v, qr, part, nch, GEN_CHUNK, c->cur_k, c->cur_v, multi ? q_pos : nullptr, nqt, out, lse, s);
  return rkv_check_launch();
}

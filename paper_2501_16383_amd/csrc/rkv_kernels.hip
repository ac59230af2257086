// Write half (rotate, reorder, quantize, pack, sinks), calibration, and the exact views of the
// cache used by tests (dequantize, export, import).
#include "rkv_internal.h"
#include "rkv_quant.h"

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------

// Walsh-Hadamard butterflies (Eq. 10 without the 1/sqrt(2) factors) over PL values per lane times
// 2^XSTAGES lanes: element index = PL*lane + i, natural (Sylvester) order.
template <int PL, typename T>
__device__ inline void fwht_lanes(T (&x)[PL], int lane, int xstages) {
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
    T sgn = (lane & mask) ? (T)-1 : (T)1;
    asm volatile("" : "+v"(sgn));     // keep it a register operand so each butterfly is one FMA
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      T o = __shfl_xor(x[i], mask);
      x[i] = sgn * x[i] + o;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// init / reset
// ---------------------------------------------------------------------------------------------

__global__ void k_fill_zero(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (; i < n16; i += stride) p[i] = z;
}

__global__ void k_init_small(RkvView v, int tables) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int S = v.max_sinks > 0 ? v.max_sinks : 1;
  if (i < v.B * S) v.sink_pos[i] = -1;
  if (tables && i < v.E) {
    v.perm[i] = i;
    v.pinv[i] = i;
    v.gid[i] = i / v.qg;
  }
}

// RoPE angle table: rope[t][j] = (cos, sin)(t * theta^(-j/64)), evaluated in double.
__global__ void k_init_rope(RkvView v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= v.Tpad * 64) return;
  const int t = i >> 6, j = i & 63;
  const double freq = pow((double)v.theta, -(double)j / 64.0);
  double sn, cs;
  sincos((double)t * freq, &sn, &cs);
  v.rope[i] = make_float2((float)cs, (float)sn);
}

// B operand of v_mfma_f32_16x16x128_f8f6f4 holding H_128 (entries +-1 as FP4 E2M1: 0x2 / 0xA).
// Lane (n = lane & 15, q = lane >> 4) holds, in nibble e of dword v, input channel k = 32q + 8v + e
// of output channel 16*tile + n.  The decode kernel rotates the results of tiles p and p + 4 as a
// RoPE pair: channels 16p + n and 16p + n + 64 - or, with interleaved pairs (rope_style 1),
// tile p holds output channel 2 (16p + n) and tile p + 4 its odd neighbour.
__global__ void k_init_hop(uint32_t* hop, int rope_style) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // (tile, lane, v)
  if (i >= 8 * 64 * 4) return;
  const int vreg = i & 3, lane = (i >> 2) & 63, tile = i >> 8;
  const int n = lane & 15, q = lane >> 4;
  uint32_t w = 0;
  for (int e = 0; e < 8; ++e) {
    const int k = 32 * q + 8 * vreg + e, col = rope_style ? 2 * (16 * (tile & 3) + n) + (tile >> 2) : 16 * tile + n;
    w |= ((__popc(k & col) & 1) ? 0xAu : 0x2u) << (4 * e);
  }
  hop[i] = w;
}

int rkv_launch_init(rkv_cache* c, bool tables, hipStream_t s) {
  const size_t n16 = c->off_tables / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)c->base, n16);
  const RkvView& v = c->v;
  int S = v.max_sinks > 0 ? v.max_sinks : 1;
  int m = v.B * S > v.E ? v.B * S : v.E;
  hipLaunchKernelGGL(k_init_small, dim3((m + 255) / 256), dim3(256), 0, s, v, tables ? 1 : 0);
  if (tables) hipLaunchKernelGGL(k_init_rope, dim3((v.Tpad * 64 + 255) / 256), dim3(256), 0, s, v);
  if (tables) hipLaunchKernelGGL(k_init_hop, dim3(8), dim3(256), 0, s, v.hop, v.rope_style);
  if (tables) c->blocks_aligned = 1;
  return rkv_check_launch();
}

// ---------------------------------------------------------------------------------------------
// sinks: keep the original fp16 rows of flagged tokens (Sec. 4.3), first come first kept
// ---------------------------------------------------------------------------------------------

__global__ void __launch_bounds__(256) k_sinks(RkvView v, const __half* __restrict__ k, const __half* __restrict__ vv,
                                               const uint8_t* __restrict__ mask, int n_new) {
  __shared__ int s_count[256];
  __shared__ int s_tok[64];
  __shared__ int s_new;
  __shared__ float s_row[512];
  // n_new: rows per sequence in k, vv and mask; sequence b uses the first n_b of them
  const int b = blockIdx.x, tid = threadIdx.x;
  const int n_b = v.nnew ? v.nnew[b] : n_new;
  const int cnt0 = v.sink_cnt[b];
  const int room = v.max_sinks - cnt0;
  const int per = (n_b + 255) / 256;
  const int lo = min(tid * per, n_b), hi = min(lo + per, n_b);
  int mine = 0;
  for (int t = lo; t < hi; ++t) mine += mask[(size_t)b * n_new + t] != 0;
  s_count[tid] = mine;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int i = 0; i < 256; ++i) {
      int c = s_count[i];
      s_count[i] = run;
      run += c;
    }
    s_new = run < room ? run : (room > 0 ? room : 0);
  }
  __syncthreads();
  int slot = s_count[tid];
  for (int t = lo; t < hi && slot < room; ++t) {
    if (mask[(size_t)b * n_new + t] != 0) {
      s_tok[slot] = t;
      ++slot;
    }
  }
  __syncthreads();
  const int nn = s_new;
  for (int i = 0; i < nn; ++i) {
    const int t = s_tok[i];
    const size_t src = ((size_t)b * n_new + t) * v.E, dst = ((size_t)b * v.max_sinks + cnt0 + i) * v.E;
    // whole rows, 16 bytes per lane, every load of a round issued before its stores (rows are
    // 256-byte multiples and 16-byte aligned: E is a multiple of 128 halves)
    {
      const uint4* k4 = reinterpret_cast<const uint4*>(k + src);
      const uint4* v4 = reinterpret_cast<const uint4*>(vv + src);
      uint4* dk4 = reinterpret_cast<uint4*>(v.sink_k + dst);
      uint4* dv4 = reinterpret_cast<uint4*>(v.sink_v + dst);
      const int n16 = v.E / 8;
      for (int e0 = 0; e0 < n16; e0 += 4 * 256) {
        uint4 a[4], c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = e0 + u * 256 + tid;
          if (e < n16) {
            if (!v.keys_rotated) a[u] = k4[e];
            c[u] = v4[e];
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int e = e0 + u * 256 + tid;
          if (e < n16) {
            if (!v.keys_rotated) dk4[e] = a[u];
            dv4[e] = c[u];
          }
        }
      }
    }
    if (v.keys_rotated) {
      // the keys arrived rotated and reordered: undo the reorder, rotate again (H is its own
      // inverse), round to fp16 - group by group, butterflies in LDS (n <= 512 in this mode)
      for (int rg = 0; rg < v.NRG; ++rg) {
        const int gb = rg * v.n;
        for (int c = tid; c < v.n; c += 256) s_row[c] = __half2float(k[src + v.pinv[gb + c]]);
        __syncthreads();
        for (int h = 1; h < v.n; h <<= 1) {
          for (int j = tid; j < v.n / 2; j += 256) {
            const int lo = ((j / h) * 2 * h) + (j % h), hi = lo + h;
            const float a = s_row[lo], c2 = s_row[hi];
            s_row[lo] = a + c2;
            s_row[hi] = a - c2;
          }
          __syncthreads();
        }
        const float rs = rsqrtf((float)v.n);
        for (int c = tid; c < v.n; c += 256) v.sink_k[dst + gb + c] = __float2half_rn(s_row[c] * rs);
        __syncthreads();
      }
    }
    if (tid == 0) v.sink_pos[b * v.max_sinks + cnt0 + i] = rkv_len(v, b) + t;
  }
  if (tid == 0) v.sink_cnt[b] = cnt0 + nn;
}

// ---------------------------------------------------------------------------------------------
// quantize-append
//   One workgroup = (sequence, unit, tile of 16 token slots).  A unit is the smallest channel range
//   closed under both the rotation and the reorder: max(perm_span, n) channels.  Each wave takes one
//   token at a time: rotate in registers + lane exchanges (Sec. 4.2), scatter to reordered
//   positions in LDS (Sec. 4.1), reduce min/max per block of 128, Eq. 6-9, and OR the codes into LDS
//   images of the physical tile, which are then written with whole-dword stores.  With codes wider
//   than 2 bits the images take the low two bits; the upper two bits of 4-bit codes go to a second
//   pair of images (the planes have the same layout), the third bits of 3-bit codes to images of
//   their plane (one dword per pair of dwords of the low plane; a V dword of that plane also holds
//   the bits of the slab's other 16 tokens, which another workgroup may be writing: it is updated
//   with atomic operations on this tile's bits only).
// ---------------------------------------------------------------------------------------------

template <int PL>
__global__ void __launch_bounds__(256) k_append(RkvView v, const __half* __restrict__ kin, const __half* __restrict__ vin,
                                                int n_new, int tile0, int U) {
  extern __shared__ uint32_t smem[];
  float* zbuf = reinterpret_cast<float*>(smem);            // [4][U]
  uint32_t* imgK = smem + 4 * U;                            // [U]  (16 tokens x U codes)
  uint32_t* imgV = imgK + U;                                // [U]  (one dword per channel)
  const int hb = v.hb;
  uint32_t* imgKh = imgV + U;                               // 4-bit: [U], as imgK; 3-bit: [U / 2]
  uint32_t* imgVh = imgKh + (hb == 2 ? U : U / 2);          // 4-bit: [U], as imgV; 3-bit: [U], this tile's bits of the channel's dword
  const int himg = hb == 2 ? 2 * U : (hb == 1 ? U + U / 2 : 0);   // dwords of the two together
  const float qmax = (float)((4 << hb) - 1);
  const int blk_lanes = v.qg >> 3;                          // lanes (8 values each) of one quantization block
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tile = tile0 + blockIdx.x, unit = blockIdx.y, b = blockIdx.z;
  const int ubase = unit * U, n = v.n, g = v.g;
  const int rgs = U / n, rg0 = ubase / n;
  const int t_lo = v.len, t_hi = v.len + n_new;
  const float rs = rsqrtf((float)n);

  for (int i = tid; i < 2 * U + himg; i += 256) imgK[i] = 0;   // imgK, imgV and the high-bit images are adjacent
  __syncthreads();

  // old V dwords of a partly filled tile are fetched now and merged at the end
  uint32_t keep = 0;
  for (int m = 0; m < 16; ++m) {
    const int t = tile * 16 + m;
    if (!(t >= t_lo && t < t_hi)) keep |= 3u << rkv_v_shift(t & 31);
  }
  uint32_t oldv[4] = {0, 0, 0, 0}, oldv2[4] = {0, 0, 0, 0};
  if (keep && U <= 1024) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int idx = tid + 256 * k;
      if (idx < U) {
        const int r = idx / n, c = idx - r * n;
        const size_t a = rkv_v_slabbase(v, b, rg0 + r, tile >> 1) + rkv_v_off(g, c, (tile & 1) * 16);
        oldv[k] = v.vc[a];
        if (hb == 2) oldv2[k] = v.vh[a];
      }
    }
  }

  float* zw = zbuf + wave * U;
  const int m_first = max(0, t_lo - tile * 16), m_last = min(15, t_hi - 1 - tile * 16);
  for (int m0 = m_first; m0 <= m_last; m0 += 4) {
    const int m = m0 + wave;
    const int t = tile * 16 + m;
    const bool active = m <= m_last;
    const size_t row = ((size_t)b * n_new + (active ? t - t_lo : 0)) * v.E;
    if (active) {
      for (int r = 0; r < rgs; ++r) {
        float x[PL];
        const int cbase = ubase + r * n + PL * lane;
        load_halves<PL>(kin + row + cbase, x);
        fwht_lanes<PL>(x, lane, 6);
#pragma unroll
        for (int i = 0; i < PL; ++i) zw[v.pinv[cbase + i] - ubase] = x[i] * rs;
      }
    }
    __syncthreads();
    if (active) {
      for (int base = 0; base < U; base += 512) {
        const int pos = base + 8 * lane;
        const bool on = pos < U;
        // ---- keys: reordered positions pos..pos+7, block of 128 = 16 lanes
        float z[8];
        float mn = 3.0e38f, mx = -3.0e38f;
        if (on) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            z[i] = zw[pos + i];
            mn = fminf(mn, z[i]);
            mx = fmaxf(mx, z[i]);
          }
        }
        for (int s = 1; s < blk_lanes; s <<= 1) {
          mn = fminf(mn, __shfl_xor(mn, s));
          mx = fmaxf(mx, __shfl_xor(mx, s));
        }
        if (on) {
          float sc, zero, inv;
          quant_params(mn, mx, sc, zero, inv, v.meta8, qmax);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const uint32_t code = quant_code(z[i], inv, zero, qmax);
            const int cr = v.perm[ubase + pos + i] - ubase;      // rotated channel, unit-local
            const int r = cr / n, c = cr - r * n;
            int sh;
            const int off = rkv_k_off(g, m, c, sh);
            atomicOr(&imgK[r * 128 * g + off], (code & 3u) << sh);
            if (hb == 2) atomicOr(&imgKh[r * 128 * g + off], (code >> 2) << sh);
            else if (hb == 1) {
              int bit;
              const size_t hi_idx = rkv_h1_loc((size_t)(r * 128 * g + off), sh, bit);
              atomicOr(&imgKh[hi_idx], (code >> 2) << bit);
            }
          }
          if ((lane & (blk_lanes - 1)) == 0) rkv_store_meta(v, v.km, rkv_meta_index(v, b, t, (ubase + pos) / v.qg), sc, zero);
        }
        // ---- values: channels pos..pos+7 of the unit, block of 128 = one head
        float u[8];
        if (on) load_halves<8>(vin + row + ubase + pos, u);
        else {
#pragma unroll
          for (int i = 0; i < 8; ++i) u[i] = 0.f;
        }
        if (v.v_rotate) {
          fwht_lanes<8>(u, lane, 4);
#pragma unroll
          for (int i = 0; i < 8; ++i) u[i] *= 0.08838834764831845f;   // 1/sqrt(128)
        }
        mn = 3.0e38f; mx = -3.0e38f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          mn = fminf(mn, u[i]);
          mx = fmaxf(mx, u[i]);
        }
        for (int s = 1; s < blk_lanes; s <<= 1) {
          mn = fminf(mn, __shfl_xor(mn, s));
          mx = fmaxf(mx, __shfl_xor(mx, s));
        }
        if (on) {
          float sc, zero, inv;
          quant_params(mn, mx, sc, zero, inv, v.meta8, qmax);
          const int sh = rkv_v_shift(t & 31);
          int hbit = 0;                                     // 3-bit codes: the token's place in the third-bit dword of a channel
          rkv_h1_loc((size_t)(tile & 1), sh, hbit);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const uint32_t code = quant_code(u[i], inv, zero, qmax);
            atomicOr(&imgV[pos + i], (code & 3u) << sh);
            if (hb == 2) atomicOr(&imgVh[pos + i], (code >> 2) << sh);
            else if (hb == 1) atomicOr(&imgVh[pos + i], (code >> 2) << hbit);
          }
          if ((lane & (blk_lanes - 1)) == 0) rkv_store_meta(v, v.vm, rkv_meta_index(v, b, t, (ubase + pos) / v.qg), sc, zero);
        }
      }
    }
    __syncthreads();
  }

  // ---- write the images.  K: every 16-byte piece of a tile belongs to one token.
  const int tile_dw = 128 * g;
  for (int idx = tid; idx < U; idx += 256) {
    const int r = idx / tile_dw, off = idx - r * tile_dw;
    const int t = tile * 16 + rkv_k_tile_token(g, off);
    if (t >= t_lo && t < t_hi) {
      v.kc[rkv_k_tilebase(v, b, rg0 + r, tile) + off] = imgK[idx];
      if (hb == 2) v.kh[rkv_k_tilebase(v, b, rg0 + r, tile) + off] = imgKh[idx];
      else if (hb == 1 && !(idx & 1)) v.kh[(rkv_k_tilebase(v, b, rg0 + r, tile) + off) >> 1] = imgKh[idx >> 1];
    }
  }
  // third-bit places of this tile's tokens that this call writes (the same in every channel's dword)
  uint32_t clr = 0;
  if (hb == 1)
    for (int m = 0; m < 16; ++m) {
      const int t = tile * 16 + m;
      int bit;
      rkv_h1_loc((size_t)(tile & 1), rkv_v_shift(t & 31), bit);
      if (t >= t_lo && t < t_hi) clr |= 1u << bit;
    }
  // V: a dword holds 16 token slots of one channel; keep the slots of tokens not in this call.
  for (int idx = tid, k = 0; idx < U; idx += 256, ++k) {
    const int r = idx / n, c = idx - r * n;
    const size_t a = rkv_v_slabbase(v, b, rg0 + r, tile >> 1) + rkv_v_off(g, c, (tile & 1) * 16);
    uint32_t w = imgV[idx];
    if (keep) w |= (U <= 1024 ? oldv[k & 3] : v.vc[a]) & keep;
    v.vc[a] = w;
    if (hb == 2) {
      w = imgVh[idx];
      if (keep) w |= (U <= 1024 ? oldv2[k & 3] : v.vh[a]) & keep;
      v.vh[a] = w;
    } else if (hb == 1) {
      atomicAnd(&v.vh[a >> 1], ~clr);
      atomicOr(&v.vh[a >> 1], imgVh[idx]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// quantize-append, fast path for reorders that keep the 128-blocks of the rotated row
// (gid[c] == c/128): the quantization blocks are then the rotated blocks themselves, codes are
// stored by rotated channel, and the reorder indices are not needed at all.
//   One workgroup = (sequence, rotation group, slab of 32 token slots) so that every V dword
//   (16 tokens of one channel), every K tile and every metadata row it touches is written whole.
//   Wave w takes tokens 8w..8w+7 of the slab, one at a time: lane holds PL = n/64 consecutive
//   channels; rotation in registers + lane exchanges; min/max over the lanes of a block; Eq. 6-9.
// ---------------------------------------------------------------------------------------------

template <int PL>
__global__ void __launch_bounds__(256) k_append_fast(RkvView v, const __half* __restrict__ kin, const __half* __restrict__ vin,
                                                     int n_new, int slab0) {
  constexpr int G = PL / 2;                    // heads per rotation group
  constexpr int LPB = 128 / PL;                // lanes per 128-block
  __shared__ uint32_t imgK[2 * 128 * G];       // two K tiles
  __shared__ uint32_t imgV[4][64 * PL];        // per wave: partial V dwords of its 8 tokens, [i][lane]
  __shared__ uint32_t metaK[32 * G], metaV[32 * G];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int slab = slab0 + blockIdx.x, rg = blockIdx.y, b = blockIdx.z;
  const int n = 128 * G;
  const int t_lo = v.len, t_hi = v.len + n_new;
  const int ts = slab * 32;

  // slots of this slab that belong to tokens outside this call are kept
  uint32_t keep[2] = {0, 0};
  for (int tau = 0; tau < 32; ++tau) {
    const int t = ts + tau;
    if (!(t >= t_lo && t < t_hi)) keep[tau >> 4] |= 3u << rkv_v_shift(tau);
  }
  const size_t vbase = rkv_v_slabbase(v, b, rg, slab);
  uint32_t oldv[G];
#pragma unroll
  for (int k = 0; k < G; ++k) oldv[k] = 0;
  if (keep[0] | keep[1]) {
#pragma unroll
    for (int k = 0; k < G; ++k) oldv[k] = v.vc[vbase + tid + 256 * k];
  }
  for (int i = tid; i < 2 * 128 * G; i += 256) imgK[i] = 0;
  __syncthreads();

  const float rs = rsqrtf((float)n);
  const int blk = lane / LPB;                              // 128-block (= KV head) of this lane's channels
  const int kap0 = (PL * lane) & 127;                      // first channel inside the block
  uint32_t vword[PL];
#pragma unroll
  for (int i = 0; i < PL; ++i) vword[i] = 0;

  const int tau_first = max(0, t_lo - ts), tau_last = min(31, t_hi - 1 - ts);
  for (int k = 0; k < 8; ++k) {
    const int tau = 8 * wave + k;
    if (tau < tau_first || tau > tau_last) continue;       // wave-uniform
    const int t = ts + tau;
    const size_t row = ((size_t)b * n_new + (t - t_lo)) * v.E + (size_t)rg * n + PL * lane;
    // ---- keys
    float x[PL];
    load_halves<PL>(kin + row, x);
    fwht_lanes<PL>(x, lane, 6);
    float mn = 3.0e38f, mx = -3.0e38f;
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      x[i] *= rs;
      mn = fminf(mn, x[i]);
      mx = fmaxf(mx, x[i]);
    }
#pragma unroll
    for (int s = 1; s < LPB; s <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, s));
      mx = fmaxf(mx, __shfl_xor(mx, s));
    }
    {
      float sc, zero, inv;
      quant_params(mn, mx, sc, zero, inv, v.meta8);
      uint32_t part = 0;
      int off = 0;
#pragma unroll
      for (int i = 0; i < PL; ++i) {
        int sh;
        const int o = rkv_k_off(G, tau & 15, 128 * blk + kap0 + i, sh);
        if (i == 0) off = o;                               // the lane's channels share one dword
        part |= quant_code(x[i], inv, zero) << sh;
      }
      atomicOr(&imgK[(tau >> 4) * (128 * G) + off], part);
      if ((lane & (LPB - 1)) == 0) metaK[tau * G + blk] = rkv_pack_meta(sc, zero);
    }
    // ---- values
    float u[PL];
    load_halves<PL>(vin + row, u);
    if (v.v_rotate) {
      fwht_lanes<PL>(u, lane, PL == 8 ? 4 : (PL == 4 ? 5 : (PL == 2 ? 6 : 3)));
#pragma unroll
      for (int i = 0; i < PL; ++i) u[i] *= 0.08838834764831845f;
    }
    mn = 3.0e38f; mx = -3.0e38f;
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      mn = fminf(mn, u[i]);
      mx = fmaxf(mx, u[i]);
    }
#pragma unroll
    for (int s = 1; s < LPB; s <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, s));
      mx = fmaxf(mx, __shfl_xor(mx, s));
    }
    {
      float sc, zero, inv;
      quant_params(mn, mx, sc, zero, inv, v.meta8);
      const int sh = rkv_v_shift(tau);
#pragma unroll
      for (int i = 0; i < PL; ++i) vword[i] |= quant_code(u[i], inv, zero) << sh;
      if ((lane & (LPB - 1)) == 0) metaV[tau * G + blk] = rkv_pack_meta(sc, zero);
    }
  }
#pragma unroll
  for (int i = 0; i < PL; ++i) imgV[wave][i * 64 + lane] = vword[i];
  __syncthreads();

  // ---- K tiles: every 16-byte piece belongs to one token
#pragma unroll
  for (int k = 0; k < G; ++k) {
    const int idx = tid + 256 * k;                          // 0 .. 256G-1
    const int ti = idx / (128 * G), off = idx - ti * (128 * G);
    const int t = ts + ti * 16 + rkv_k_tile_token(G, off);
    if (t >= t_lo && t < t_hi) v.kc[rkv_k_tilebase(v, b, rg, 2 * slab + ti) + off] = imgK[idx];
  }
  // ---- V slab: dword idx = (((w*G + hh)*16 + nn)*2 + ct)*2 + d, channel c = 128hh + 32w + 16ct + nn;
  //      waves 2d and 2d+1 hold the two halves of its 16 token slots
#pragma unroll
  for (int k = 0; k < G; ++k) {
    const int idx = tid + 256 * k;
    const int d = idx & 1, ct = (idx >> 1) & 1, nn = (idx >> 2) & 15, rest = idx >> 6;
    const int hh = rest % G, w = rest / G;
    const int c = 128 * hh + 32 * w + 16 * ct + nn;
    const int ln = c / PL, i = c - ln * PL;
    uint32_t word = imgV[2 * d][i * 64 + ln] | imgV[2 * d + 1][i * 64 + ln];
    if (keep[d]) word |= oldv[k] & keep[d];
    if (keep[d] != 0xffffffffu) v.vc[vbase + idx] = word;
  }
  // ---- metadata rows of the tokens written
  for (int i = tid; i < 32 * G; i += 256) {
    const int tau = i / G;
    if (tau >= tau_first && tau <= tau_last) {
      const size_t mi = ((size_t)(b * v.NRG + rg) * v.Tpad + ts + tau) * G + (i - tau * G);
      rkv_store_meta_word(v, v.km, mi, metaK[i]);
      rkv_store_meta_word(v, v.vm, mi, metaV[i]);
    }
  }
}

int rkv_launch_sinks(rkv_cache* c, const __half* k, const __half* vv, const uint8_t* mask, int n_new, hipStream_t s) {
  const RkvView& v = c->v;
  hipLaunchKernelGGL(k_sinks, dim3(v.B), dim3(256), 0, s, v, k, vv, mask, n_new);
  return rkv_check_launch();
}

// Per-sequence lengths on the device: set_to >= 0 sets every length to it; set_to == -2 takes them
// from the staged per-sequence array (a truncation: retained sink rows at or behind the new end
// are dropped too - they were added in order of position); otherwise each length grows by `add`
// plus, while an append with per-sequence counts is in progress, by its count.
// Also rebuilds cstart (running count of 256-token chunks, see RkvView) - one workgroup; thread i
// owns a contiguous slice of the sequences.
__global__ void __launch_bounds__(256) k_lens(RkvView v, int* lens, int* cstart, int set_to, int add) {
  __shared__ int s_sum[256];
  const int tid = threadIdx.x;
  const int per = (v.B + 255) / 256, b0 = min(tid * per, v.B), b1 = min(b0 + per, v.B);
  int chunks = 0;
  for (int b = b0; b < b1; ++b) {
    const int len = set_to >= 0 ? set_to : (set_to == -2 ? v.nnew[b] : lens[b] + add + (v.nnew ? v.nnew[b] : 0));
    lens[b] = len;
    if (set_to == -2 && v.max_sinks > 0) {
      int c = v.sink_cnt[b];
      while (c > 0 && v.sink_pos[b * v.max_sinks + c - 1] >= len) --c;
      v.sink_cnt[b] = c;
    }
    chunks += (len + 255) >> 8;
  }
  s_sum[tid] = chunks;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int i = 0; i < 256; ++i) {
      const int c = s_sum[i];
      s_sum[i] = run;
      run += c;
    }
    cstart[v.B] = run;
  }
  __syncthreads();
  int run = s_sum[tid];
  for (int b = b0; b < b1; ++b) {
    cstart[b] = run;
    run += (lens[b] + 255) >> 8;
  }
}

int rkv_launch_lens(rkv_cache* c, int set_to, int add, hipStream_t s) {
  const RkvView& v = c->v;
  hipLaunchKernelGGL(k_lens, dim3(1), dim3(256), 0, s, v, c->dev_lens, c->dev_cstart, set_to, add);
  return rkv_check_launch();
}

int rkv_launch_append(rkv_cache* c, const __half* k, const __half* vv, int n_new, const uint8_t* mask, hipStream_t s) {
  const RkvView& v = c->v;
  if (mask && v.max_sinks > 0) hipLaunchKernelGGL(k_sinks, dim3(v.B), dim3(256), 0, s, v, k, vv, mask, n_new);
  if (rkv_append_mfma_supported(c)) return rkv_launch_append_mfma(c, k, vv, n_new, 0, s);
  if (c->blocks_aligned && !c->wide && (v.g == 2 || v.g == 4)) {
    const int slab0 = v.len >> 5, slab1 = (v.len + n_new - 1) >> 5;
    dim3 grid(slab1 - slab0 + 1, v.NRG, v.B);
    if (c->ev_start) RKV_HIP_CHECK(hipEventRecord(c->ev_start, s));
    if (v.g == 4) hipLaunchKernelGGL(k_append_fast<8>, grid, dim3(256), 0, s, v, k, vv, n_new, slab0);
    else hipLaunchKernelGGL(k_append_fast<4>, grid, dim3(256), 0, s, v, k, vv, n_new, slab0);
    if (c->ev_stop) RKV_HIP_CHECK(hipEventRecord(c->ev_stop, s));
    return rkv_check_launch();
  }
  const int U = v.span > v.n ? v.span : v.n;
  const int tile0 = v.len >> 4, tile1 = (v.len + n_new - 1) >> 4;
  dim3 grid(tile1 - tile0 + 1, v.E / U, v.B);
  const size_t lds = (size_t)6 * U * 4 + (v.hb == 2 ? (size_t)8 * U : v.hb == 1 ? (size_t)6 * U : 0);   // the kernel's images, see there
  void (*fn)(RkvView, const __half*, const __half*, int, int, int) = nullptr;
  switch (v.n / 64) {
    case 2: fn = k_append<2>; break;
    case 4: fn = k_append<4>; break;
    case 8: fn = k_append<8>; break;
    case 16: fn = k_append<16>; break;
    default: return RKV_EINVAL;
  }
  if (lds > 160 * 1024) return RKV_EINVAL;
  if (lds > 48 * 1024) RKV_HIP_CHECK(hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  if (c->ev_start) RKV_HIP_CHECK(hipEventRecord(c->ev_start, s));
  hipLaunchKernelGGL(fn, grid, dim3(256), lds, s, v, k, vv, n_new, tile0, U);
  if (c->ev_stop) RKV_HIP_CHECK(hipEventRecord(c->ev_stop, s));
  return rkv_check_launch();
}

// ---------------------------------------------------------------------------------------------
// dequantize (test support): Eq. 7, inverse reorder (through gid), inverse rotation
// ---------------------------------------------------------------------------------------------

template <int PL>
__global__ void __launch_bounds__(64) k_dequant(RkvView v, float* __restrict__ k_hat, float* __restrict__ v_hat) {
  const int rg = blockIdx.x, t = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int n = v.n;
  const size_t row = ((size_t)b * v.len + t) * v.E + (size_t)rg * n;
  if (k_hat) {
    float x[PL];
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      const int c = PL * lane + i;
      int sh;
      const uint32_t w = v.kc[rkv_k_dword(v, b, rg, t, c, sh)];
      float sc, zero;
      rkv_load_meta(v, v.km, rkv_meta_index(v, b, t, v.gid[rg * n + c]), sc, zero);
      x[i] = sc * ((float)(((w >> sh) & 3u) | rkv_khi_get(v, b, rg, t, c)) - zero);
    }
    fwht_lanes<PL>(x, lane, 6);
    const float rs = rsqrtf((float)n);
#pragma unroll
    for (int i = 0; i < PL; ++i) k_hat[row + PL * lane + i] = x[i] * rs;
  }
  if (v_hat) {
    for (int base = 0; base < n; base += 512) {
      const int c0 = base + 8 * lane;
      const bool on = c0 < n;
      float u[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        u[i] = 0.f;
        if (on) {
          int sh;
          const uint32_t w = v.vc[rkv_v_dword(v, b, rg, t, c0 + i, sh)];
          float sc, zero;
          rkv_load_meta(v, v.vm, rkv_meta_index(v, b, t, (rg * n + c0) / v.qg), sc, zero);
          u[i] = sc * ((float)(((w >> sh) & 3u) | rkv_vhi_get(v, b, rg, t, c0 + i)) - zero);
        }
      }
      if (v.v_rotate) {
        fwht_lanes<8>(u, lane, 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] *= 0.08838834764831845f;
      }
      if (on) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v_hat[row + c0 + i] = u[i];
      }
    }
  }
}

int rkv_launch_dequant(rkv_cache* c, float* k_hat, float* v_hat, hipStream_t s) {
  const RkvView& v = c->v;
  dim3 grid(v.NRG, v.len, v.B);
  switch (v.n / 64) {
    case 2: hipLaunchKernelGGL(k_dequant<2>, grid, dim3(64), 0, s, v, k_hat, v_hat); break;
    case 4: hipLaunchKernelGGL(k_dequant<4>, grid, dim3(64), 0, s, v, k_hat, v_hat); break;
    case 8: hipLaunchKernelGGL(k_dequant<8>, grid, dim3(64), 0, s, v, k_hat, v_hat); break;
    case 16: hipLaunchKernelGGL(k_dequant<16>, grid, dim3(64), 0, s, v, k_hat, v_hat); break;
    default: return RKV_EINVAL;
  }
  return rkv_check_launch();
}

// ---------------------------------------------------------------------------------------------
// export / import of the logical code array in canonical bytes (test support): four 2-bit codes
// per byte, or two wider codes per byte (a nibble each), first code in the lowest bits
// ---------------------------------------------------------------------------------------------

__global__ void k_export(RkvView v, uint8_t* kc, float* ks, float* kz, uint8_t* vc, float* vs, float* vz) {
  const int cpb = v.hb ? 2 : 4, fw = 8 / cpb;                 // codes per byte, bits of a byte each takes
  const size_t per_tok = v.E / cpb;
  const size_t total = (size_t)v.B * v.len * per_tok;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int j = idx % per_tok;
    const size_t bt = idx / per_tok;
    const int t = bt % v.len, b = bt / v.len;
    uint32_t kb = 0, vb = 0;
    for (int r = 0; r < cpb; ++r) {
      const int i = cpb * j + r;
      int sh;
      if (kc) {
        const int cr = v.perm[i];
        const uint32_t w = v.kc[rkv_k_dword(v, b, cr / v.n, t, cr % v.n, sh)];
        kb |= (((w >> sh) & 3u) | rkv_khi_get(v, b, cr / v.n, t, cr % v.n)) << (fw * r);
      }
      if (vc) {
        const uint32_t w = v.vc[rkv_v_dword(v, b, i / v.n, t, i % v.n, sh)];
        vb |= (((w >> sh) & 3u) | rkv_vhi_get(v, b, i / v.n, t, i % v.n)) << (fw * r);
      }
    }
    if (kc) kc[idx] = (uint8_t)kb;
    if (vc) vc[idx] = (uint8_t)vb;
    if (j < v.NG) {
      const size_t mi = rkv_meta_index(v, b, t, j), o = bt * v.NG + j;
      float sc, zero;
      rkv_load_meta(v, v.km, mi, sc, zero);
      if (ks) ks[o] = sc;
      if (kz) kz[o] = zero;
      rkv_load_meta(v, v.vm, mi, sc, zero);
      if (vs) vs[o] = sc;
      if (vz) vz[o] = zero;
    }
  }
}

int rkv_launch_export(rkv_cache* c, uint8_t* kc, float* ks, float* kz, uint8_t* vc, float* vs, float* vz, hipStream_t s) {
  const RkvView& v = c->v;
  const size_t total = (size_t)v.B * v.len * (v.E / (v.hb ? 2 : 4));
  size_t blocks = (total + 255) / 256;
  if (blocks > 65535) blocks = 65535;
  hipLaunchKernelGGL(k_export, dim3((unsigned)blocks), dim3(256), 0, s, v, kc, ks, kz, vc, vs, vz);
  return rkv_check_launch();
}

__global__ void k_import(RkvView v, int T, const uint8_t* kc, const float* ks, const float* kz, const uint8_t* vc,
                         const float* vs, const float* vz) {
  const int cpb = v.hb ? 2 : 4, fw = 8 / cpb;
  const uint32_t fmask = (1u << fw) - 1u;
  const size_t per_tok = v.E / cpb;
  const size_t total = (size_t)v.B * T * per_tok;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int j = idx % per_tok;
    const size_t bt = idx / per_tok;
    const int t = bt % T, b = bt / T;
    const uint32_t kb = kc[idx], vb = vc[idx];
    for (int r = 0; r < cpb; ++r) {
      const int i = cpb * j + r;
      int sh;
      const int cr = v.perm[i];
      const uint32_t kcode = (kb >> (fw * r)) & fmask, vcode = (vb >> (fw * r)) & fmask;
      size_t a = rkv_k_dword(v, b, cr / v.n, t, cr % v.n, sh);
      atomicOr(&v.kc[a], (kcode & 3u) << sh);
      if (v.hb == 2) atomicOr(&v.kh[a], (kcode >> 2) << sh);
      a = rkv_v_dword(v, b, i / v.n, t, i % v.n, sh);
      atomicOr(&v.vc[a], (vcode & 3u) << sh);
      if (v.hb == 2) atomicOr(&v.vh[a], (vcode >> 2) << sh);
      if (v.hb == 1) {
        int bit;
        a = rkv_h1_loc(rkv_k_dword(v, b, cr / v.n, t, cr % v.n, sh), sh, bit);
        atomicOr(&v.kh[a], (kcode >> 2) << bit);
        a = rkv_h1_loc(rkv_v_dword(v, b, i / v.n, t, i % v.n, sh), sh, bit);
        atomicOr(&v.vh[a], (vcode >> 2) << bit);
      }
    }
    if (j < v.NG) {
      const size_t mi = rkv_meta_index(v, b, t, j), o = bt * v.NG + j;
      rkv_store_meta(v, v.km, mi, ks[o], kz[o]);
      rkv_store_meta(v, v.vm, mi, vs[o], vz[o]);
    }
  }
}

int rkv_launch_import(rkv_cache* c, int T, const uint8_t* kc, const float* ks, const float* kz, const uint8_t* vc,
                      const float* vs, const float* vz, hipStream_t s) {
  const RkvView& v = c->v;
  // clear the code and metadata regions (they are contiguous from the start of the block up to the sink store)
  const size_t n16 = ((char*)v.sink_k - c->base) / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)c->base, n16);
  const size_t total = (size_t)v.B * T * (v.E / (v.hb ? 2 : 4));
  blocks = (total + 255) / 256;
  if (blocks > 65535) blocks = 65535;
  hipLaunchKernelGGL(k_import, dim3((unsigned)blocks), dim3(256), 0, s, v, T, kc, ks, kz, vc, vs, vz);
  return rkv_check_launch();
}

// ---------------------------------------------------------------------------------------------
// calibration (Alg. 1).  The rotation is linear, so the channel sums of the rotated keys are the
// rotation of the channel sums: sum first (float64), rotate once, rank-sort inside each span.
// ---------------------------------------------------------------------------------------------

__global__ void k_calib_sum(const __half* __restrict__ k, int n_tok, int E, double* __restrict__ sums) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= E) return;
  double acc = 0.0;
  for (int t = 0; t < n_tok; ++t) acc += (double)__half2float(k[(size_t)t * E + c]);
  sums[c] = acc;
}

__global__ void __launch_bounds__(256) k_calib_rotate(const double* __restrict__ sums, double* __restrict__ rot, int n) {
  extern __shared__ double sh[];
  const int rg = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < n; i += 256) sh[i] = sums[(size_t)rg * n + i];
  __syncthreads();
  for (int h = 1; h < n; h <<= 1) {
    for (int p = tid; p < n / 2; p += 256) {
      const int i = (p / h) * 2 * h + (p % h);
      const double a = sh[i], b = sh[i + h];
      sh[i] = a + b;
      sh[i + h] = a - b;
    }
    __syncthreads();
  }
  const double rs = 1.0 / sqrt((double)n);
  for (int i = tid; i < n; i += 256) rot[(size_t)rg * n + i] = sh[i] * rs;
}

__global__ void k_calib_rank(const double* __restrict__ rot, int E, int span, int* __restrict__ perm) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= E) return;
  const int base = (c / span) * span;
  const double x = rot[c];
  int rank = 0;
  for (int j = 0; j < span; ++j) {
    const double y = rot[base + j];
    rank += (y < x) || (y == x && base + j < c);
  }
  perm[base + rank] = c;
}

size_t rkv_calib_scratch_bytes(const rkv_config* cfg) { return (size_t)cfg->n_kv_heads * RKV_D * 8 * 2; }

int rkv_launch_calibrate(const rkv_config* cfg, const __half* k_cal, int n_tok, int* perm_out, void* scratch, hipStream_t s) {
  const int E = cfg->n_kv_heads * RKV_D, n = cfg->rot_heads * RKV_D;
  double* sums = (double*)scratch;
  double* rot = sums + E;
  hipLaunchKernelGGL(k_calib_sum, dim3((E + 255) / 256), dim3(256), 0, s, k_cal, n_tok, E, sums);
  hipLaunchKernelGGL(k_calib_rotate, dim3(E / n), dim3(256), (size_t)n * 8, s, sums, rot, n);
  hipLaunchKernelGGL(k_calib_rank, dim3((E + 255) / 256), dim3(256), 0, s, rot, E, cfg->perm_span, perm_out);
  return rkv_check_launch();
}

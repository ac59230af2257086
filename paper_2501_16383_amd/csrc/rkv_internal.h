// Internal declarations shared by the HIP translation units of librkv.
//
// Physical layout of one layer's cache (all inside the caller's block, 256-byte aligned parts).
// "Rotated channel" c is a channel index after the grouped-head Hadamard, before the reorder;
// "reordered position" i is its place after the reorder: reordered[i] = rotated[perm[i]].
// Codes are stored by ROTATED channel, so the read half needs no gather; the reorder survives as
// a table gid[] that says which quantization block (of 128 reordered positions) a rotated channel
// belongs to.  The canonical byte image of the logical code array is produced by rkv_export_codes.
//
//   K codes   [batch][rot group][Tpad/16 tiles] of 16 tokens x n codes.  Inside a tile, for
//             g = rot_heads >= 2: [block pair pr][q 0..3][token m 0..15][16 bytes], the 16 bytes
//             being [block-in-pair][dword d 0..1]; for g = 1: [q][m][dword d].  Rotated channel
//             128*blk + kap (kap = 32q + 8v + e) sits in dword d = v>>1 at bit 2*(2e + (v&1)).
//             One wave-wide 16-byte load therefore fetches 1 KiB contiguous and leaves in every
//             lane exactly the 2 x 32 codes it feeds to the FP4 matrix instruction.
//   K meta    [batch][rot group][Tpad][g] x (fp16 scale, fp16 zero); entry (rg, j) is the
//             quantization block G = rg*g + j of reordered positions [128G, 128G+128).
//   V codes   [batch][rot group][Tpad/32 slabs] of 32 tokens x n channels, token-minor:
//             [w 0..3][head-in-group hh][nn 0..15][ct 0..1][dword d 0..1]; channel
//             128*hh + 32w + 16ct + nn, token tau of the slab in dword d = tau>>4 at bit
//             2*(2*(tau&7) + ((tau>>3)&1)).
//   V meta    as K meta (block G = KV head).
//   sinks     fp16 rows [batch][max_sinks][E] for K and V, positions, counts.
//   tables    perm, inverse perm, gid (int32 [E] each), RoPE angles float2 [Tpad][64], the
//             Hadamard operand image of the matrix-core kernel.
//
// Codes wider than 2 bits and quantization groups smaller than 128 (Sec. 5.1, the settings of
// Tables tab:ablation and tab:quantgrani) keep all of the above for the low two bits of every code
// and add
//   K high, V high   4-bit codes: the upper two bits, in arrays laid out exactly as K codes and
//             V codes (same dword, same bit position), so that the matrix-core kernels read them
//             as a second plane; 3-bit codes: the third bit, one dword for each aligned pair of
//             dwords (2p, 2p + 1) of K codes / V codes (the 32 codes of one matrix operand), the
//             bit of the code at bit 2m of dword 2p + x sitting at bit 4 (m >> 1) + 2 x + (m & 1):
//             shifting the dword right by k = 0..3 and masking every fourth bit yields the four
//             operand dwords of FP4 nibbles, as the 2-bit unpacking does for the low bits;
//   K meta, V meta   128 / quant_group entries in place of each one (gid then counts blocks of
//             quant_group reordered positions).
// 3- and 4-bit codes in groups of 128 run on the matrix-core kernels (k_append_mfma<.., HB>,
// k_decode_mfma<.., HB>: the planes above the low two bits go through the same products); groups
// of 64 / 32 are read through the scores kernel of rkv_decode_row.hip and the matrix-core decode
// kernel's softmax and value phases (a reorder inside the rotation groups; any code width, either metadata
// format) and by the general kernel otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "../../include/rkv.h"

#define RKV_D 128
#define RKV_LDS_BYTES (160 * 1024)   // LDS of a compute unit
#define RKV_STAGE_SLOTS 4             // pinned host slots for per-sequence counts on their way to the device
#define RKV_PART_STRIDE 132   // floats per split-K partial: m, l, 2 pad, acc[128]
#define RKV_GEN_CHUNK 128     // tokens per split-K chunk of the general decode kernel
#define RKV_MFMA_CHUNK 256    // ... of the matrix-core decode kernel
#define RKV_ROW_CHUNK 64      // tokens per workgroup of the scores kernel for a reorder over the whole row

struct RkvView {
  uint32_t* kc;
  uint32_t* km;
  uint32_t* vc;
  uint32_t* vm;
  __half* sink_k;
  __half* sink_v;
  int* sink_pos;
  int* sink_cnt;
  int* perm;
  int* pinv;
  int* gid;
  float2* rope;
  uint32_t* hop;     // Hadamard B-operand image for the FP4 matrix instruction: [8 tiles][64 lanes][4 dwords]
  // Tables of the append kernel's variants (written by rkv_set_perm):
  uint32_t* xgsel;   // [rot group][wave 0..3][lane group q][head h]: the quantization blocks (2 bits each, element
                     // 4 ppl + rr) of the eight channels 128 h + 32 q + 8 (2 (wave & 1) + (wave >> 1)) + 4 ppl + rr
                     // that a lane of the append kernel's key role holds
  const uint2* xgid8; // [rot group][wave 0..3][lane group q][head h]: the same eight channels' quantization blocks of the
                     // whole row, one byte each (a reorder over the whole row: k_append_row_keys)
  int B, Hq, Hkv, g, n, E, NRG, NG, Tpad, max_sinks, len, span, rope_style, v_rotate, keys_rotated;
  const int* lens;   // per-sequence lengths [B] once the sequences differ in length, else null (all have `len` tokens)
  const int* cstart; // with `lens`: cstart[b] = 256-token chunks of the sequences before b, cstart[B] = all of them
  const int* nnew;   // during an append with per-sequence token counts: those counts [B], else null
  int meta8;         // 1: km / vm hold, per (token, rotation group), gm FP8 E4M3 scales followed by gm 8-bit zero-points (value + 128)
  uint32_t* kh;      // high bits of the codes (see the layout above), null with 2-bit codes
  uint32_t* vh;
  int qg;            // quantization group: 128, 64 or 32 channels
  int gm;            // metadata entries per (token, rotation group): g * 128 / qg
  int hb;            // bits per code above the low two: 0, 1 or 2
  float theta;
};

// length of sequence b
__device__ inline int rkv_len(const RkvView& v, int b) { return v.lens ? v.lens[b] : v.len; }

struct rkv_cache {
  rkv_config cfg;
  RkvView v;           // v.len: the length of the longest sequence
  int32_t* hlens;      // host mirror of the per-sequence lengths [batch]
  int32_t* stage;      // pinned host ring [RKV_STAGE_SLOTS][batch]: per-sequence counts on their way to dev_nnew
  hipEvent_t stage_ev[RKV_STAGE_SLOTS];   // recorded after the copy that reads a slot
  int stage_used[RKV_STAGE_SLOTS], stage_next;
  int* dev_lens;       // device copy (kept current once `ragged` is set) and staging for per-sequence token counts
  int* dev_nnew;
  int* dev_cstart;     // [batch + 1], see RkvView::cstart
  int ragged;          // 1 once sequences differ in length
  size_t bytes;
  char* base;
  size_t off_tables;      // everything before this offset is cleared by reset
  int blocks_aligned;     // 1 if the reorder keeps every rotated channel in its block of 128
  int wide;               // 1 with codes wider than 2 bits or groups smaller than 128: general kernels only
  int in_groups;          // 1 if the reorder keeps every rotated channel inside its rotation group (and rot_heads is 2 or 4)
  int decode_path;
  int n_cu;               // compute units of the device the cache lives on
  hipEvent_t ev_start, ev_stop;   // optional measurement hook around the main kernels
  const __half* cur_k;    // set for the duration of a decode call that attends the token being decoded
  const __half* cur_v;    // in full precision ([batch][n_kv_heads][128] fp16 each), else null
};

// offset (in dwords) of rotated channel c (within its rotation group) of token m inside a K tile
__host__ __device__ inline int rkv_k_off(int g, int m, int c, int& shift) {
  int blk = c >> 7, kap = c & 127;
  int q = kap >> 5, r5 = kap & 31, vv = r5 >> 3, e = r5 & 7, d = vv >> 1;
  shift = 2 * (2 * e + (vv & 1));
  if (g == 1) return (q * 16 + m) * 2 + d;
  return (((blk >> 1) * 4 + q) * 16 + m) * 4 + (blk & 1) * 2 + d;
}
__host__ __device__ inline size_t rkv_k_tilebase(const RkvView& v, int b, int rg, int tile) {
  return ((size_t)(b * v.NRG + rg) * (size_t)(v.Tpad >> 4) + tile) * (size_t)(128 * v.g);
}
__host__ __device__ inline size_t rkv_k_dword(const RkvView& v, int b, int rg, int t, int c, int& shift) {
  return rkv_k_tilebase(v, b, rg, t >> 4) + rkv_k_off(v.g, t & 15, c, shift);
}
// offset (in dwords) inside a K tile -> token m of the tile
__host__ __device__ inline int rkv_k_tile_token(int g, int off) { return g == 1 ? ((off >> 1) & 15) : ((off >> 2) & 15); }

__host__ __device__ inline int rkv_v_shift(int tau) { return 2 * (2 * (tau & 7) + ((tau >> 3) & 1)); }
// offset (in dwords) of channel c (within its rotation group), token tau inside a V slab
__host__ __device__ inline int rkv_v_off(int g, int c, int tau) {
  int hh = c >> 7, ch = c & 127;
  int w = ch >> 5, ct = (ch >> 4) & 1, nn = ch & 15, d = tau >> 4;
  return ((((w * g + hh) * 16 + nn) * 2 + ct) * 2 + d);
}
__host__ __device__ inline size_t rkv_v_slabbase(const RkvView& v, int b, int rg, int slab) {
  return ((size_t)(b * v.NRG + rg) * (size_t)(v.Tpad >> 5) + slab) * (size_t)(2 * v.n);
}
__host__ __device__ inline size_t rkv_v_dword(const RkvView& v, int b, int rg, int t, int c, int& shift) {
  shift = rkv_v_shift(t & 31);
  return rkv_v_slabbase(v, b, rg, t >> 5) + rkv_v_off(v.g, c, t & 31);
}

// meta entry of global quantization block G (0..E/qg) of token t
__host__ __device__ inline size_t rkv_meta_index(const RkvView& v, int b, int t, int G) {
  int rg = G / v.gm, j = G - rg * v.gm;
  return ((size_t)(b * v.NRG + rg) * (size_t)v.Tpad + t) * v.gm + j;
}
// Third bit of a 3-bit code (hb == 1): from the place of its low two bits (dword index and shift
// in K codes / V codes) to the dword index and bit in K high / V high
__host__ __device__ inline size_t rkv_h1_loc(size_t lo_index, int lo_shift, int& bit) {
  const int m = lo_shift >> 1;
  bit = 4 * (m >> 1) + 2 * (int)(lo_index & 1) + (m & 1);
  return lo_index >> 1;
}
// The bits above the low two of the code of (rotated) channel c of rotation group rg, token t,
// already shifted to their place in the code (0 with 2-bit codes)
__device__ inline uint32_t rkv_khi_get(const RkvView& v, int b, int rg, int t, int c) {
  if (v.hb == 0) return 0u;
  int sh;
  if (v.hb == 2) {
    const uint32_t w = v.kh[rkv_k_dword(v, b, rg, t, c, sh)];
    return ((w >> sh) & 3u) << 2;
  }
  int bit;
  const uint32_t w = v.kh[rkv_h1_loc(rkv_k_dword(v, b, rg, t, c, sh), sh, bit)];
  return ((w >> bit) & 1u) << 2;
}
__device__ inline uint32_t rkv_vhi_get(const RkvView& v, int b, int rg, int t, int c) {
  if (v.hb == 0) return 0u;
  int sh;
  if (v.hb == 2) {
    const uint32_t w = v.vh[rkv_v_dword(v, b, rg, t, c, sh)];
    return ((w >> sh) & 3u) << 2;
  }
  int bit;
  const uint32_t w = v.vh[rkv_h1_loc(rkv_v_dword(v, b, rg, t, c, sh), sh, bit)];
  return ((w >> bit) & 1u) << 2;
}

__device__ inline uint32_t rkv_pack_meta(float scale, float zero) {
  __half2 h = __halves2half2(__float2half_rn(scale), __float2half_rn(zero));
  return *reinterpret_cast<uint32_t*>(&h);
}
__device__ inline void rkv_unpack_meta(uint32_t u, float& scale, float& zero) {
  __half2 h = *reinterpret_cast<__half2*>(&u);
  scale = __low2float(h);
  zero = __high2float(h);
}

// FP8 E4M3 (1-4-3, bias 7, subnormals m * 2^-9, largest number 448) written out from the format's
// definition; x must be one of its non-negative numbers.
__device__ inline uint32_t rkv_e4m3_encode(float x) {
  if (x < 0.015625f) return (uint32_t)(x * 512.0f);                    // subnormal (or 0)
  const uint32_t b = __float_as_uint(x);
  return ((((b >> 23) & 0xffu) - 120u) << 3) | ((b >> 20) & 7u);
}
__device__ inline float rkv_e4m3_decode(uint32_t byte) {
  const uint32_t e = (byte >> 3) & 15u, m = byte & 7u;
  if (e == 0) return (float)m * 0.001953125f;
  return __uint_as_float(((e + 120u) << 23) | (m << 20));
}
// smallest E4M3 number >= x (x >= 0), at most 448
__device__ inline float rkv_e4m3_round_up(float x) {
  if (!(x < 448.0f)) return 448.0f;
  if (x < 0.015625f) return ceilf(x * 512.0f) * 0.001953125f;          // multiples of 2^-9 (2^-6 itself is the first normal)
  return __uint_as_float((__float_as_uint(x) + 0x000fffffu) & 0xfff00000u);   // three mantissa bits, carry into the exponent
}
// Entry idx (rkv_meta_index) of a metadata array in the cache's format.  The 8-bit format keeps,
// for each (token, rotation group), the gm scale bytes first and the gm zero-point bytes after them
// (the matrix-core decode kernel converts either kind four at a time); a zero-point z in -128..127
// is stored as the unsigned byte z + 128.
__device__ inline void rkv_load_meta(const RkvView& v, const uint32_t* m, size_t idx, float& scale, float& zero) {
  if (v.meta8) {
    const uint8_t* p = reinterpret_cast<const uint8_t*>(m) + 2 * (idx - idx % v.gm) + idx % v.gm;
    scale = rkv_e4m3_decode(p[0]);
    zero = (float)p[v.gm] - 128.0f;
  } else {
    rkv_unpack_meta(m[idx], scale, zero);
  }
}
__device__ inline void rkv_store_meta(const RkvView& v, uint32_t* m, size_t idx, float scale, float zero) {
  if (v.meta8) {
    uint8_t* p = reinterpret_cast<uint8_t*>(m) + 2 * (idx - idx % v.gm) + idx % v.gm;
    p[0] = (uint8_t)rkv_e4m3_encode(scale);
    p[v.gm] = (uint8_t)((int)zero + 128);
  } else {
    m[idx] = rkv_pack_meta(scale, zero);
  }
}
// the same from a staged fp16 pair (scale and zero are exact in fp16 in either format)
__device__ inline void rkv_store_meta_word(const RkvView& v, uint32_t* m, size_t idx, uint32_t word) {
  if (v.meta8) {
    float s, z;
    rkv_unpack_meta(word, s, z);
    rkv_store_meta(v, m, idx, s, z);
  } else {
    m[idx] = word;
  }
}

// Streaming accesses: data that is read or written once per launch (new keys and values, the
// cache during decode) is marked non-temporal so that it does not displace anything in the caches;
// measured on this chip, a plain read stream reaches 7.2 TB/s that way against 6.4 TB/s without.
typedef unsigned int rkv_u4v __attribute__((ext_vector_type(4)));
typedef unsigned int rkv_u2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 rkv_ld_stream(const uint4* p) {
  const rkv_u4v t = __builtin_nontemporal_load(reinterpret_cast<const rkv_u4v*>(p));
  return make_uint4(t[0], t[1], t[2], t[3]);
}
__device__ __forceinline__ uint2 rkv_ld_stream(const uint2* p) {
  const rkv_u2v t = __builtin_nontemporal_load(reinterpret_cast<const rkv_u2v*>(p));
  return make_uint2(t[0], t[1]);
}
__device__ __forceinline__ void rkv_st_stream(uint32_t* p, uint32_t x) { __builtin_nontemporal_store(x, p); }

// Several query tokens per sequence in one step: the kernels then run on a view whose Hq counts
// "virtual" query heads, nq per real one.  Virtual head hv of KV head kvh = hv / rep' (rep' = virtual
// heads per KV head) is query token qi = (hv % rep') / rep of real head kvh * rep + (hv % rep') % rep,
// where rep = rep' / nq.  Tensors are [batch][nq][real heads][...].
struct RkvVHead { int qi, h; };
__device__ inline RkvVHead rkv_virtual_head(const RkvView& v, int hv, int nq) {
  const int repv = v.Hq / v.Hkv, rep = repv / nq;
  const int kvh = hv / repv, vr = hv - kvh * repv;
  RkvVHead r;
  r.qi = vr / rep;
  r.h = kvh * rep + (vr - r.qi * rep);
  return r;
}

// bytes at the start of the decode scratch block that hold the prepared queries: the natural
// layout once, the matrix-core kernel's lane-ordered layout four times (see k_prep_q)
inline size_t rkv_query_scratch_bytes(size_t batch, size_t n_q_heads) {
  return (batch * n_q_heads * RKV_D * 4 * 5 + 255) & ~(size_t)255;
}

// kernels' host launchers (defined in the .hip files)
int rkv_launch_init(rkv_cache* c, bool tables, hipStream_t s);
int rkv_launch_set_perm_tables(rkv_cache* c, hipStream_t s);
int rkv_launch_append(rkv_cache* c, const __half* k, const __half* v, int n_new, const uint8_t* mask, hipStream_t s);
bool rkv_append_mfma_supported(const rkv_cache* c);
int rkv_launch_append_mfma(rkv_cache* c, const __half* k, const __half* v, int n_new, int max_slabs, hipStream_t s);
int rkv_launch_sinks(rkv_cache* c, const __half* k, const __half* v, const uint8_t* mask, int n_new, hipStream_t s);
int rkv_launch_lens(rkv_cache* c, int set_to, int add, hipStream_t s);
int rkv_launch_dequant(rkv_cache* c, float* k_hat, float* v_hat, hipStream_t s);
int rkv_launch_export(rkv_cache* c, uint8_t* kc, float* ks, float* kz, uint8_t* vc, float* vs, float* vz, hipStream_t s);
int rkv_launch_import(rkv_cache* c, int T, const uint8_t* kc, const float* ks, const float* kz, const uint8_t* vc,
                      const float* vs, const float* vz, hipStream_t s);
int rkv_launch_decode_general(rkv_cache* c, const __half* q, const int* q_pos, int n_queries, float* out, float* lse, void* scratch,
                              hipStream_t s);
int rkv_launch_decode_mfma(rkv_cache* c, const __half* q, const int* q_pos, int nq, float* out, float* lse, void* scratch,
                           bool q_prepared, hipStream_t s);
int rkv_mfma_share(int heads_per_kv_head);
// a reorder over the whole token row (rkv_decode_row.hip): its scores kernel and the buffer it fills
bool rkv_row_supported(const rkv_cache* c);
bool rkv_scores_local(const rkv_cache* c);   // groups of 32 inside the heads: scores from the same kernel
bool rkv_scores_path(const rkv_cache* c);    // either of the two
int rkv_append_mfma_variant(const rkv_cache* c);   // RKV_KERNEL_* of the matrix-core append kernel a cache takes
size_t rkv_row_scores_bytes(int batch, int n_q_heads, int max_tokens);
int rkv_launch_scores_row(const rkv_cache* c, const RkvView& v, const float* qr, float* sc, hipStream_t s);
bool rkv_scores_multi_ok(const rkv_cache* c, int n_queries);   // several query tokens per step on that route
size_t rkv_partial_bytes(int batch, int n_q_heads, int Tpad);
int rkv_launch_step_mfma(rkv_cache* c, const __half* k, const __half* v, const __half* q, const int* q_pos, float* qr, int share,
                         hipStream_t s);
bool rkv_mfma_supported(const rkv_cache* c);
int rkv_mfma_variant(const rkv_cache* c);   // RKV_KERNEL_MFMA, _MFMA_CROSS or _MFMA_SUB (if rkv_mfma_supported)
void rkv_launch_prep_q(const RkvView& v, const __half* q, const int* q_pos, int cur, float* qr, int share, int nq,
                       hipStream_t s);
void rkv_launch_merge(const RkvView& v, const float* qr, const float* part, int nch, int chunk_tokens, const __half* k_cur,
                      const __half* v_cur, const int* q_lim, int nq, float* out, float* lse, hipStream_t s);
int rkv_launch_calibrate(const rkv_config* cfg, const __half* k_cal, int n_tok, int* perm_out, void* scratch, hipStream_t s);
int rkv_launch_fold_rotation(const rkv_config* cfg, const float* w, int rows, const int* perm, float* out, hipStream_t s);
int rkv_launch_select_sinks(const __half* x, int batch, int n_tok, int width, int k, int32_t* idx_out, uint8_t* mask_out,
                            float* scratch, hipStream_t s);
size_t rkv_decode_scratch_bytes(const rkv_config* cfg);
size_t rkv_calib_scratch_bytes(const rkv_config* cfg);

#define RKV_HIP_CHECK(expr)                    \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) return RKV_EHIP;     \
  } while (0)

inline int rkv_check_launch() { return hipPeekAtLastError() == hipSuccess ? RKV_OK : RKV_EHIP; }

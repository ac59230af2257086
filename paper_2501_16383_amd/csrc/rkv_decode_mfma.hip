// Read half, matrix-core kernel for gfx950.
//
// The inverse rotation of the keys is a dense contraction with a +-1 matrix, and 2-bit codes are
// exactly representable in FP4 (E2M1: a nibble holding the integer c in its two low bits is the
// value c/2), so the per-head Hadamard H_128 of the raw codes runs on
// v_mfma_f32_16x16x128_f8f6f4 with exact small-integer results in fp32.  The rest is linear in
// those results:
//     k^[head a][j] = (1/sqrt(n)) * sum_blk H_g[a][blk] * scale_blk * (H_128 c_blk - 128 zero_blk e_0)[j]
// (H_n = H_g (x) H_128 for the grouped-head rotation of Sec. 4.2; Eq. 7 folded in).  The sum over
// the blocks is a second, tiny matrix product on v_mfma_f32_4x4x4_16b_f16 (16 independent 4x4x4
// products per instruction): rows = the token's fp16 scales signed by a row of H_g, columns = the
// blocks' results, which are exact in fp16; the zero-point term is one more such product.  The
// vector ALU does RoPE and the dot with the query (Eq. 5).  p.V runs on the same instruction with the codes as the FP4
// operand and the softmax weights p_t * scale_t as the other: each weight is scaled by a power of
// two per (head, chunk) to a 24-bit integer and split into six base-16 digits, which FP8 (E4M3)
// holds exactly.  All products are then small half-integers of similar size, so the instruction's
// internal accumulation is exact (with weights of mixed magnitude in one dot product it is not:
// small terms are cut ~2^-14 below the largest); zero-points enter as one scalar per head.
//
// One workgroup = (sequence, rotation group, chunk of 256 tokens), 4 waves.
//   phase K  wave w: tokens 64w..64w+63 in tiles of 16.  A = codes [16 tokens x 128], B = H_128 tile
//            [128 x 16 channels]; lane (n, q) of the result holds channel 16*tile + n of tokens
//            4q..4q+3.  Scores are reduced over the 16 channel lanes with DPP and go to LDS.
//   phase S  wave a: softmax statistics of head a over the chunk, weights -> FP8 digits in LDS.
//   phase V  wave w: channels 32w..32w+31 of every head; A = weight digits [16 x (4 heads x 32
//            tokens)], block-diagonal over heads, B = codes [(4 heads x 32 tokens) x 16 channels].
// Covers: reorder that keeps 128-blocks, rot_heads 2 or 4, codes of 2 to 4 bits in groups of 128;
// both RoPE pairings (the Hadamard operand tiles are built so that tiles p and p + 4 yield the two
// channels of a pair).  With GQA (or several query tokens per step) a workgroup serves two of the query heads
// that share a KV head: unpacking, rotation and RoPE of the keys are done once for them, the
// softmax and value phases once per query head.  Everything else takes the general kernel.
#include "rkv_internal.h"
#include <cstdlib>
#include <hip/hip_ext.h>

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

#ifndef MF_TILES
#define MF_TILES 4         // 16-token tiles per wave
#endif
#define MF_CH (64 * MF_TILES)   // tokens per workgroup (4 waves)
static_assert(MF_CH == 256, "the per-sequence chunk table (k_lens) counts chunks of 256 tokens");
static_assert(MF_CH == RKV_MFMA_CHUNK, "the work-space size of a call is worked out from RKV_MFMA_CHUNK");
#ifndef MF_ACC
#define MF_ACC 16         // score accumulators per lane and pass of the key phase
#endif
#ifndef MF_OCC_HI
#define MF_OCC_HI 2        // the same for the variants that hold a second plane of codes of four heads (three would spill)
#endif
#ifndef MF_OCC
#define MF_OCC 3           // workgroups per compute unit the register budget is set for
#endif

__device__ __forceinline__ v4f mfma_fp4(const v8i& a, const v8i& b, const v4f& c) {
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 4, 0, 0, 0, 0);
}
__device__ __forceinline__ v4f mfma_fp8_fp4(const v8i& a, const v8i& b, const v4f& c) {
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 4, 0, 0, 0, 0);
}

__device__ __forceinline__ v4h as_v4h(uint32_t a, uint32_t b) {
  union { uint32_t u[2]; v4h h; } c;
  c.u[0] = a;
  c.u[1] = b;
  return c.h;
}
// two floats that are exactly representable in fp16 -> packed pair
__device__ __forceinline__ uint32_t pk_f16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
// 16 independent 4x4x4 products: block = lane / 4, A row / B column = lane % 4, result column = lane % 4
__device__ __forceinline__ v4f mfma_4x4x4(const v4h& a, const v4h& b, const v4f& c) {
  return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 0, 0, 0);
}

// two dwords of 2-bit codes -> four dwords of FP4 nibbles (value = code / 2)
__device__ __forceinline__ v8i unpack_fp4(uint32_t d0, uint32_t d1) {
  v8i r;
  r[0] = (int)(d0 & 0x33333333u);
  r[1] = (int)((d0 >> 2) & 0x33333333u);
  r[2] = (int)(d1 & 0x33333333u);
  r[3] = (int)((d1 >> 2) & 0x33333333u);
  r[4] = r[5] = r[6] = r[7] = 0;
  return r;
}

// one dword of third bits (3-bit codes; bit 4j + k belongs to nibble j of operand dword k) -> four
// dwords of FP4 nibbles (value = bit / 2)
__device__ __forceinline__ v8i unpack_fp4_bits(uint32_t h) {
  v8i r;
  r[0] = (int)(h & 0x11111111u);
  r[1] = (int)((h >> 1) & 0x11111111u);
  r[2] = (int)((h >> 2) & 0x11111111u);
  r[3] = (int)((h >> 3) & 0x11111111u);
  r[4] = r[5] = r[6] = r[7] = 0;
  return r;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
#define DPP_ROW_MIRROR 0x140
#define DPP_ROW_HALF_MIRROR 0x141
#define DPP_QUAD_MIRROR 0x1B      // quad_perm [3,2,1,0]
#define DPP_QUAD_SWAP 0xB1        // quad_perm [1,0,3,2]

// Sum NV values over the 16 lanes of a row; lane n ends with the total of value n (NV = 16) or of
// value n & 7 (NV = 8).
// The first two steps of the sixteen-value case, written out: a step's lanes of the upper half keep
// the upper values and those of the lower half the lower ones, which a DPP addition does in one
// instruction per half when it is told to write only that half's banks of four lanes (the other
// lanes keep what the destination holds) - two instructions per result where a select of what to
// keep, a select of what to send and the addition take three.  The compiler does not look into
// the text for the two idle cycles a DPP operand needs after a vector write of it, and it does not
// know of them for the results either: hence the waits at both ends, and the order inside (every
// register is read two or more instructions after it was written).
__device__ __forceinline__ void row_transpose_reduce_16_to_4(const float (&v)[16], float (&k4)[4]) {
  float a0, a1, a2, a3, a4, a5, a6, a7;
  asm("s_nop 1\n\t"
      "v_add_f32_dpp %4, %12, %12 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %5, %13, %13 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %6, %14, %14 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %7, %15, %15 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %8, %16, %16 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %9, %17, %17 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %10, %18, %18 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %11, %19, %19 row_mirror row_mask:0xf bank_mask:0x3\n\t"
      "v_add_f32_dpp %4, %20, %20 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %5, %21, %21 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %6, %22, %22 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %7, %23, %23 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %8, %24, %24 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %9, %25, %25 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %10, %26, %26 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %11, %27, %27 row_mirror row_mask:0xf bank_mask:0xc\n\t"
      "v_add_f32_dpp %0, %4, %4 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
      "v_add_f32_dpp %1, %5, %5 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
      "v_add_f32_dpp %2, %6, %6 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
      "v_add_f32_dpp %3, %7, %7 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
      "v_add_f32_dpp %0, %8, %8 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
      "v_add_f32_dpp %1, %9, %9 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
      "v_add_f32_dpp %2, %10, %10 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
      "v_add_f32_dpp %3, %11, %11 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
      "s_nop 1"
      : "=&v"(k4[0]), "=&v"(k4[1]), "=&v"(k4[2]), "=&v"(k4[3]), "=&v"(a0), "=&v"(a1), "=&v"(a2), "=&v"(a3), "=&v"(a4), "=&v"(a5),
        "=&v"(a6), "=&v"(a7)
      : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]), "v"(v[8]), "v"(v[9]), "v"(v[10]),
        "v"(v[11]), "v"(v[12]), "v"(v[13]), "v"(v[14]), "v"(v[15]));
}

template <int NV>
__device__ __forceinline__ float row_transpose_reduce(float (&v)[NV], int n) {
  float k4[4];
  if constexpr (NV == 16) {
    row_transpose_reduce_16_to_4(v, k4);
  } else {
  float k8[8];
  if constexpr (NV == 16) {
    const bool hi = (n & 8) != 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float keep = hi ? v[i + 8] : v[i], send = hi ? v[i] : v[i + 8];
      k8[i] = keep + dpp_f<DPP_ROW_MIRROR>(send);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) k8[i] = v[i] + dpp_f<DPP_ROW_MIRROR>(v[i]);
  }
  {
    const bool hi = (n & 4) != 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float keep = hi ? k8[i + 4] : k8[i], send = hi ? k8[i] : k8[i + 4];
      k4[i] = keep + dpp_f<DPP_ROW_HALF_MIRROR>(send);
    }
  }
  }
  float k2[2];
  {
    const bool hi = (n & 2) != 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float keep = hi ? k4[i + 2] : k4[i], send = hi ? k4[i] : k4[i + 2];
      k2[i] = keep + dpp_f<DPP_QUAD_MIRROR>(send);
    }
  }
  const bool hi = (n & 1) != 0;
  const float keep = hi ? k2[1] : k2[0], send = hi ? k2[0] : k2[1];
  return keep + dpp_f<DPP_QUAD_SWAP>(send);
}

// All-lanes reduction over the 64 lanes of a wave: 4 DPP steps inside each row of 16, then the
// four row results through scalar registers.
template <bool IS_MAX>
__device__ __forceinline__ float wave_allreduce(float x) {
  auto op = [](float a, float b) { return IS_MAX ? fmaxf(a, b) : a + b; };
  x = op(x, dpp_f<DPP_QUAD_SWAP>(x));
  x = op(x, dpp_f<0x4E>(x));                 // quad_perm [2,3,0,1]
  x = op(x, dpp_f<DPP_ROW_HALF_MIRROR>(x));
  x = op(x, dpp_f<DPP_ROW_MIRROR>(x));
  const int xi = __float_as_int(x);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(xi, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(xi, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(xi, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(xi, 48));
  return op(op(r0, r1), op(r2, r3));
}

// MULTI: several query tokens per sequence.  v.Hq then counts virtual heads (nq per real head, see
// rkv_virtual_head) and virtual head hv only attends tokens at positions <= q_lim[b][query token of hv].
// META8: scales in FP8 E4M3 and zero-points in 8 bits (rkv_load_meta describes the layout); they
// are widened to the fp16 operands of the small matrix products right after loading.
// HB = 2: 4-bit codes, c = c_lo + 4 c_hi.  The plane of the upper two bits has the layout of the lower
// one.  HB = 1: 3-bit codes, the plane of third bits holds one dword per operand (half the size).
// Key phase: it goes through the same unpacking (nibble = c_hi / 2) and meets a copy of the
// Hadamard operand with entries +-4 in place of +-1, accumulating onto the low plane's products,
// so that the big products yield H_128 (c / 2) as before.  Value phase: it accumulates separately
// and is folded in, times 4, once per chunk.  Sums stay exact: |H_128 (c / 2)| <= 960 < 1024.
// SUB = 2 or 4 (with PRE): quantization groups of 64 or 32 channels, reorder inside the heads.  The
// scores come from k_scores_row2 (a key phase of SUB masked passes over the sub-blocks was the
// first design and measured slower); here every value head has SUB (scale, zero-point) pairs per
// token, so the softmax phase makes SUB sets of weight digits and a wave of the value phase takes
// the set of the sub-block its 32 channels lie in.  (HB composes with SUB and PRE: the value phase's plane of
// upper bits does not depend on where the scores and the weights come from.)
// ALU: measurement only.  The same kernel with the cache stream - K codes, K metadata, V codes,
// V metadata - replaced by values made up in registers (from the lane number and a kernel
// argument, so that nothing folds at compile time): what the arithmetic alone costs when no byte
// of the cache has to arrive.  The results mean nothing.
// PRE: the scores of the compressed stream come from a buffer [sequence][query head][token slot]
// (-infinity at retained sink tokens) in place of the key phase - a reorder over the whole token
// row, whose scores k_scores_row computes; qt then points to that buffer.  Softmax, values and
// partial results as in the plain kernel.
template <int G, int REP, bool MULTI, bool META8, int HB, int SUB = 0, bool ALU = false, bool PRE = false>
__global__ void __launch_bounds__(256, (HB && G == 4) ? MF_OCC_HI : MF_OCC) k_decode_mfma(RkvView v, const float* __restrict__ qt,
                                                                       float* __restrict__ part, int nch,
                                                                       const int* __restrict__ q_lim, int nq, int ns, uint32_t inv_ns, uint32_t inv_nrg) {
  constexpr bool HI = HB != 0;
  constexpr int NH = G * REP;                    // query heads served by this workgroup: REP per KV head
  constexpr int RP = (MF_ACC / (G * REP) < 4) ? MF_ACC / (G * REP) : 4;   // tokens (of a lane's four) per pass of the key phase: MF_ACC score accumulators at most
  __shared__ float s_sc[NH][MF_CH];
  // Weight digits of phase S for the matrix products of phase V.  The operand [16 rows = 4 heads x
  // 4 digits][128 = 4 heads x 32 tokens] is block-diagonal over the heads, so only the 32 token
  // bytes of each row are kept, [slab][digit set][row][token], followed by one 16-byte piece of
  // zeros that the lanes holding the operand's empty parts read instead.
  constexpr int SA_ZERO = 16 * 32, SA_SET = SA_ZERO + 16;
  constexpr int NS = SUB ? SUB : 1;              // sub-blocks of a value head (groups of 64 / 32): weights per sub-block
  constexpr size_t SA_BYTES = (size_t)NS * (MF_CH / 32) * 2 * SA_SET;
  __shared__ __attribute__((aligned(16))) uint8_t s_A_raw[SA_BYTES];
  uint8_t (*const s_A)[MF_CH / 32][2][SA_SET] = reinterpret_cast<uint8_t (*)[MF_CH / 32][2][SA_SET]>(s_A_raw);
  __shared__ float s_m[4], s_l[4], s_zs[NS][4], s_wsc[NS][4];
  __shared__ int s_sink[64];
  __shared__ uint4 s_H[8][64];                   // Hadamard operand tiles
  __shared__ float2 s_step[64];                  // RoPE rotation by 16 positions, per channel pair
  __shared__ float2 s_step1[REP > 1 ? 64 : 1];   // ... by one position (several query heads per KV head)
  __shared__ int s_lim[MULTI ? NH : 1];          // last position each served query head may attend
  constexpr int QV = REP == 1 ? 4 : 1;            // query versions held (positions pos - r); with REP > 1 only r = 0
  __shared__ uint4 s_q[QV][4][NH / 2][16];        // [r][p][f / 4][n] x 4 floats f % 4, f = (KV head * REP + query head of it) * 2 + (lo, hi)
  // Metadata of the chunk's keys and values (plain variants): fetched once, at the start, token by
  // token, and kept in LDS - a tile's worth held in registers a whole tile ahead of its use costs
  // 16 registers, which is the difference between three and four workgroups per compute unit
  // They are stored there in the form their users take: per token the scales of the group's blocks
  // as packed fp16 pairs (s_ks: the A operand of the small matrix products, up to signs), for the
  // values (scale, zero-point) per head (s_vm) - whatever the storage format was.  The keys'
  // zero-points never reach the key phase: H_128 of a constant block is 128 z e_0, so they only
  // touch channel 0 of every head, k^[a][0] -= (2 / sqrt(n)) * 64 * Z_a(t) with
  // Z_a(t) = sum_blk H_g[a][blk] * scale_blk * zero_blk, and channel 0 is one half of RoPE pair 0,
  // whose angle at token t is t itself.  Their share of the score of (token t, query head h),
  //     - 64 * Z_a(t) * (cos(t) * q~[h][pair 0, first half] + sin(t) * q~[h][pair 0, second half]),
  // is worked out once per token when the metadata are staged and put where the key phase adds
  // its sum (s_sc).
  constexpr bool LM = SUB == 0;
  constexpr int MWL = META8 ? G / 2 : G;             // metadata dwords per token and rotation group as stored
  constexpr int GP = G / 2;                          // packed pairs per token
  __shared__ __attribute__((aligned(16))) uint32_t s_ks[LM ? MF_CH * GP : 1], s_vm[LM ? MF_CH * G : 1];
  static_assert(SUB == 0 || PRE, "groups of 64 / 32 run on precomputed scores");
  static_assert(!ALU || (!META8 && HB == 0 && !MULTI), "the arithmetic-only measurement exists for the plain 2-bit variants");
  static_assert(!PRE || !ALU, "precomputed scores: no arithmetic-only measurement");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, q = lane >> 4;
  // Wave priority: the few instructions before the first barrier, and the short softmax and
  // value phases at the end, go ahead of the key phases of the compute unit's other workgroups
  // (which are dense vector work and fill every gap): a young wave otherwise waits behind them for
  // each of its instructions, and its workgroup's place on the compute unit idles meanwhile.
  __builtin_amdgcn_s_setprio(3);
  // The arguments the first microsecond needs, asked for in one go (left to itself the compiler
  // fetches each where it is first used, one scalar round trip after the other)
  asm volatile("" ::"s"(v.kc), "s"(v.km), "s"(v.vc), "s"(v.vm), "s"(v.rope), "s"(v.hop), "s"(v.sink_pos), "s"(v.sink_cnt), "s"(v.lens),
               "s"(qt), "s"(v.Tpad), "s"(v.NRG), "s"(v.B), "s"(v.len), "s"(v.max_sinks), "s"(nch), "s"(ns), "s"(inv_ns), "s"(inv_nrg));
  // row (n & 3) of H_g as fp16 sign masks for the packed scale pairs (blocks 0,1) and (2,3);
  // rows >= G are zero
  const int hrow = n & 3;
  const uint32_t keep_row = hrow < G ? 0xffffffffu : 0u;
  const uint32_t sm01 = ((__popc(hrow & 1) & 1) ? 0x80000000u : 0u);
  const uint32_t sm23 = ((__popc(hrow & 2) & 1) ? 0x00008000u : 0u) | ((__popc(hrow & 3) & 1) ? 0x80000000u : 0u);

  // Of the `rep` query heads that share a KV head (GQA) one workgroup serves REP, so that unpacking,
  // rotation and RoPE of the keys are done once for them; if rep > REP the workgroups of the other
  // query-head groups re-read the same chunk.
  // With per-sequence lengths the grid has no sequence dimension: the chunks of all sequences are
  // numbered consecutively (cstart[b] = chunks of the sequences before b), rounded up to 8 in all,
  // so that no workgroup is launched for chunks a shorter sequence does not have.
  // (ns = query-head groups of a KV head = rep / REP; the quotients below are taken with the
  // reciprocals the host passes - inv = ceil(2^32 / d), 0 for d = 1 -: a scalar integer division
  // is some thirty dependent instructions, several of them on the vector pipe that the compute
  // unit's other workgroups keep busy, and there were five of them before the first request)
  const int rep = ns * REP;
  int rg = blockIdx.y;
  int rrg, chunk, b;
  if (v.lens) {
    const int tot8 = gridDim.x / ns;
    rrg = blockIdx.x / tot8;
    const int w = blockIdx.x - rrg * tot8;
    if (w >= v.cstart[v.B]) return;
    int lo = 0, hi = v.B;                        // the last sequence whose first chunk is <= w and that has chunks
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (v.cstart[mid] <= w) lo = mid;
      else hi = mid;
    }
    b = lo;
    chunk = w - v.cstart[b];
  } else {
    // One grid dimension.  Workgroups go to the chip's eight compute dies (each with an L2 of its
    // own) in turn, so id % 8 names the die: a die takes every eighth (sequence, rotation group)
    // and runs all of its chunks, and for each chunk the workgroups of all query-head groups one
    // after the other.  What those workgroups share - the prepared queries, the sink list, and
    // with GQA the chunk's codes themselves - is then fetched into one L2 once.
    // (grid: x = 8 * nch * ns, y = eighths of the (sequence, rotation group) pairs; x runs fastest)
    const int xcd = blockIdx.x & 7, rem = blockIdx.x >> 3;
    chunk = inv_ns ? (int)__umulhi((uint32_t)rem, inv_ns) : rem;
    rrg = rem - chunk * ns;
    const int br = blockIdx.y * 8 + xcd;
    if (br >= v.B * v.NRG) return;
    b = inv_nrg ? (int)__umulhi((uint32_t)br, inv_nrg) : br;
    rg = br - b * v.NRG;
  }
  const int len = rkv_len(v, b);
  if (chunk * MF_CH >= len) return;
  const int t0 = chunk * MF_CH;

  // Everything the workgroup needs before its first tile is requested here, back to back, and put
  // in LDS further down, once - a request that is waited for before the next one goes out costs a
  // round trip to L2 or memory each, and the workgroup's place on the compute unit idles meanwhile
  // (six such round trips were a quarter of a workgroup's life).
  //  - Hadamard operand tiles (the key phase reads two of them per step)
  const uint4 ld_h0 = reinterpret_cast<const uint4*>(v.hop)[tid], ld_h1 = reinterpret_cast<const uint4*>(v.hop)[tid + 256];
  //  - queries of this rotation group, already RoPE'd, scaled and laid out as s_q by k_prep_q
  constexpr int Q16 = QV * 16 * 4 * 2 * NH / 4;          // 16-byte pieces in all
  constexpr int QN = (Q16 + 255) / 256;                  // per thread
  const uint4* q_src = reinterpret_cast<const uint4*>(qt + (((size_t)b * v.NRG + rg) * ns + rrg) * (4 * 16 * 4 * 2 * NH));
  uint4 ld_q[QN];
#pragma unroll
  for (int i = 0; i < QN; ++i) ld_q[i] = tid + 256 * i < Q16 ? q_src[tid + 256 * i] : make_uint4(0, 0, 0, 0);
  //  - RoPE angles are kept for the first of a lane's four tokens only.  With one query head per KV
  //    head they rotate all four keys and the query comes rotated back by 0..3 positions to make up
  //    for it (k_prep_q); with several (REP > 1: the extra query copies would not fit the register
  //    budget) the other three tokens follow by rotating one position at a time (table row 1).  The
  //    next tile follows by rotating 16 positions (table row 16; used once per tile, read from LDS)
  const float2 ld_step = v.rope[(REP == 1 ? 16 : 12) * 64 + (tid & 63)];
  //    (the one-position rotation: table row 1, kept in LDS as well - eight registers less where they are scarce)
  float2 ld_step1 = make_float2(0.f, 0.f);
  if constexpr (REP > 1) ld_step1 = v.rope[64 + (tid & 63)];
  //  - the sink list: positions unconditionally (the store holds max_sinks of them, unused ones -1), masked by the count below
  const int ld_cnt = v.max_sinks > 0 ? v.sink_cnt[b] : 0;
  const int ld_spos = (v.max_sinks > 0 && (tid & 63) < v.max_sinks) ? v.sink_pos[b * v.max_sinks + (tid & 63)] : -1;
  //  - (plain variants) the metadata of token t0 + tid of keys and values, its RoPE angle for channel
  //    pair 0 and the queries' entries for that pair: staged below
  uint32_t ld_mk[4] = {0, 0, 0, 0}, ld_mv[4] = {0, 0, 0, 0};
  float2 ld_cs0 = make_float2(0.f, 0.f);
  float4 ld_q0[LM ? NH / 2 : 1];
  if constexpr (LM) {
    const size_t mi = ((size_t)(b * v.NRG + rg) * v.Tpad + t0 + tid) * MWL;
    auto fetch = [&](const uint32_t* g, uint32_t (&d)[4]) {
      if constexpr (ALU) return;
      if constexpr (MWL == 4) {
        const uint4 u = rkv_ld_stream(reinterpret_cast<const uint4*>(g));
        d[0] = u.x; d[1] = u.y; d[2] = u.z; d[3] = u.w;
      } else if constexpr (MWL == 2) {
        const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(g));
        d[0] = u.x; d[1] = u.y;
      } else {
        d[0] = *g;
      }
    };
    fetch(v.km + mi, ld_mk);
    fetch(v.vm + mi, ld_mv);
    ld_cs0 = v.rope[(size_t)(t0 + tid) * 64];
    // entry (r = 0, p = 0, n = 0) of the prepared queries: floats f % 4 of piece f / 4, f = 2 * head + half
#pragma unroll
    for (int i = 0; i < NH / 2; ++i) ld_q0[i] = reinterpret_cast<const float4*>(q_src)[i * 16];
  }
  //  - the RoPE angles of this lane's first token and the first key tile: in the key phase below
  int ld_lim = 0;
  if constexpr (MULTI) {
    // served head a * REP + rri is virtual head rrg * REP + rri of its KV head: query token (that / heads per token)
    ld_lim = q_lim[b * nq + (rrg * REP + (tid < NH ? tid : 0) % REP) / (rep / nq)];
  }

  const int cnt = ld_cnt;
  {
    if constexpr (PRE) {
      // thread = token of the chunk: its scores from the buffer, its value metadata to LDS (with
      // groups of 64 / 32 the softmax phase fetches the sub-blocks' metadata itself)
      uint32_t dv[G];
      if constexpr (LM && META8) {
        // G scale bytes, then G zero-point bytes -> (scale, zero-point) fp16 pairs, the form the softmax phase takes
        const uint8_t* vm8 = reinterpret_cast<const uint8_t*>(v.vm) + ((size_t)(b * v.NRG + rg) * v.Tpad + t0 + tid) * (2 * G);
        uint32_t sw, zw;
        if constexpr (G == 4) {
          const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(vm8));
          sw = u.x; zw = u.y;
        } else {
          sw = *reinterpret_cast<const uint32_t*>(vm8);
          zw = sw >> 16;
        }
        dv[0] = rkv_pack_meta(__builtin_amdgcn_cvt_f32_fp8((int)sw, 0), (float)(zw & 0xffu) - 128.0f);
        dv[1] = rkv_pack_meta(__builtin_amdgcn_cvt_f32_fp8((int)sw, 1), (float)((zw >> 8) & 0xffu) - 128.0f);
        if constexpr (G == 4) {
          dv[2] = rkv_pack_meta(__builtin_amdgcn_cvt_f32_fp8((int)sw, 2), (float)((zw >> 16) & 0xffu) - 128.0f);
          dv[3] = rkv_pack_meta(__builtin_amdgcn_cvt_f32_fp8((int)sw, 3), (float)(zw >> 24) - 128.0f);
        }
      } else if constexpr (LM) {
        const size_t mi = ((size_t)(b * v.NRG + rg) * v.Tpad + t0 + tid) * G;
        if constexpr (G == 4) {
          const uint4 u = rkv_ld_stream(reinterpret_cast<const uint4*>(v.vm + mi));
          dv[0] = u.x; dv[1] = u.y; dv[2] = u.z; dv[3] = u.w;
        } else {
          const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(v.vm + mi));
          dv[0] = u.x; dv[1] = u.y;
        }
      }
      float pre[NH];
#pragma unroll
      for (int a = 0; a < G; ++a)
#pragma unroll
        for (int rri = 0; rri < REP; ++rri) {
          const int qh = (rg * G + a) * rep + rrg * REP + rri;
          bool seen = t0 + tid < len;
          // (several query tokens: virtual head rrg * REP + rri of its KV head belongs to query token (that / heads per token))
          if constexpr (MULTI) seen = seen && t0 + tid <= q_lim[b * nq + (rrg * REP + rri) / (rep / nq)];
          pre[a * REP + rri] = seen ? qt[((size_t)b * v.Hq + qh) * v.Tpad + t0 + tid] : -INFINITY;
        }
      uint4* a4 = reinterpret_cast<uint4*>(s_A_raw);
      for (int i = tid; i < (int)(SA_BYTES / 16); i += 256) a4[i] = make_uint4(0, 0, 0, 0);
      if (tid < 64) s_sink[tid] = tid < cnt ? ld_spos : -1;
      if constexpr (LM) {
#pragma unroll
        for (int i = 0; i < G; ++i) s_vm[tid * G + i] = dv[i];
      }
#pragma unroll
      for (int a = 0; a < NH; ++a) s_sc[a][tid] = pre[a];
      __syncthreads();
    } else {
    // ------------------------------------------------------------------ phase K
    {
      const int tw = t0 + wave * (16 * MF_TILES);
      float cs_c[4], cs_s[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const float2 cs = v.rope[(size_t)(tw + 4 * q) * 64 + 16 * p + n];
        cs_c[p] = cs.x;
        cs_s[p] = cs.y;
      }
      const uint4* ktiles = reinterpret_cast<const uint4*>(v.kc + rkv_k_tilebase(v, b, rg, tw >> 4));
      // the plane above the low two bits: 16 bytes per lane and pair of blocks (HB = 2) or 8 (HB = 1)
      const uint32_t* khtiles = HI ? v.kh + (rkv_k_tilebase(v, b, rg, tw >> 4) >> (HB == 1 ? 1 : 0)) : nullptr;
      const uint32_t* kmeta = v.km + ((size_t)(b * v.NRG + rg) * v.Tpad + tw) * (META8 ? G / 2 : G);

      uint4 cw[G / 2], cwh[HI ? G / 2 : 1];
      constexpr int MW = META8 ? G / 2 : G;              // metadata dwords per token and rotation group
      uint32_t mw[4][MW];
      auto load_tile = [&](int ti) {
        if constexpr (ALU) {                                 // made-up codes
          const uint32_t x = (uint32_t)lane * 2654435761u ^ (uint32_t)(nq + ti);
#pragma unroll
          for (int pr = 0; pr < G / 2; ++pr) cw[pr] = make_uint4(x, x * 3u, x * 5u, x * 7u + pr);
        }
#pragma unroll
        for (int pr = 0; pr < G / 2; ++pr) if constexpr (!ALU) cw[pr] = rkv_ld_stream(ktiles + (size_t)ti * (32 * G) + pr * 64 + lane);
        if constexpr (HI) {
#pragma unroll
          for (int pr = 0; pr < G / 2; ++pr) {
            const size_t li = (size_t)ti * (32 * G) + pr * 64 + lane;
            if constexpr (HB == 2) {
              cwh[pr] = rkv_ld_stream(reinterpret_cast<const uint4*>(khtiles) + li);
            } else {
              const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(khtiles) + li);
              cwh[pr] = make_uint4(u.x, u.y, 0, 0);
            }
          }
        }
        if constexpr (LM) {
          // (plain variants: the chunk's metadata are in LDS)
        } else if constexpr (META8) {
          // the lane's four tokens are consecutive: 4 x 2G bytes in one piece
          const uint4* mp = reinterpret_cast<const uint4*>(kmeta + (size_t)(ti * 16 + 4 * q) * MW);
          const uint4 u0 = rkv_ld_stream(mp);
          if constexpr (G == 4) {
            const uint4 u1 = rkv_ld_stream(mp + 1);
            mw[0][0] = u0.x; mw[0][1] = u0.y; mw[1][0] = u0.z; mw[1][1] = u0.w;
            mw[2][0] = u1.x; mw[2][1] = u1.y; mw[3][0] = u1.z; mw[3][1] = u1.w;
          } else {
            mw[0][0] = u0.x; mw[1][0] = u0.y; mw[2][0] = u0.z; mw[3][0] = u0.w;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t* mp = kmeta + (size_t)(ti * 16 + 4 * q + r) * G;
            if constexpr (G == 4) {
              const uint4 u = rkv_ld_stream(reinterpret_cast<const uint4*>(mp));
              mw[r][0] = u.x; mw[r][1] = u.y; mw[r][2] = u.z; mw[r][3] = u.w;
            } else {
              const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(mp));
              mw[r][0] = u.x; mw[r][1] = u.y;
            }
          }
        }
      };
      load_tile(0);
      // (the requests are all out: what came back goes to LDS)
      {
        uint4* a4 = reinterpret_cast<uint4*>(s_A_raw);
        for (int i = tid; i < (int)(SA_BYTES / 16); i += 256) a4[i] = make_uint4(0, 0, 0, 0);
      }
      (&s_H[0][0])[tid] = ld_h0;
      (&s_H[0][0])[tid + 256] = ld_h1;
    #pragma unroll
      for (int i = 0; i < QN; ++i)
      if (tid + 256 * i < Q16) (&s_q[0][0][0][0])[tid + 256 * i] = ld_q[i];
      if (tid < 64) {
        s_step[tid] = ld_step;
        if constexpr (REP > 1) s_step1[tid] = ld_step1;
        s_sink[tid] = tid < cnt ? ld_spos : -1;              // complete after the barrier that precedes the key phase
      }
      if constexpr (!LM) {                                   // every wave clears its own 64 score slots
    #pragma unroll
        for (int a = 0; a < NH; ++a) s_sc[a][wave * 64 + lane] = -INFINITY;
      }
      if constexpr (MULTI) {
        if (tid < NH) s_lim[tid] = min(ld_lim, len - 1);
      }
      if constexpr (LM) {                              // thread = token of the chunk (inside the padded allocation)
        // a token's metadata as stored -> packed fp16 pairs (s01, s23) and (z01, z23)
        auto pairs = [&](const uint32_t* src, uint32_t (&sp)[2], uint32_t (&zp)[2]) {
          sp[1] = zp[1] = 0;
          if constexpr (ALU) {                               // scale 1, zero-point 0
            sp[0] = sp[1] = 0x3C003C00u + (uint32_t)(nq - 1);
            zp[0] = zp[1] = 0;
          } else if constexpr (META8) {
            // G scale bytes, then G zero-point bytes.  FP8 -> fp32 -> fp16 is exact; a zero-point byte
            // u = z + 128 under the high byte 0x64 is the fp16 number 1024 + u
            const uint32_t d0 = src[0], dz = G == 4 ? src[1] : src[0] >> 16;
            const v2h off = {(_Float16)1152.0f, (_Float16)1152.0f};
            const auto f01 = __builtin_amdgcn_cvt_pk_f32_fp8((int)d0, false);
            sp[0] = pk_f16(f01[0], f01[1]);
            zp[0] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(v2h, __builtin_amdgcn_perm(0x64646464u, dz, 0x04010400u)) - off);
            if constexpr (G == 4) {
              const auto f23 = __builtin_amdgcn_cvt_pk_f32_fp8((int)d0, true);
              sp[1] = pk_f16(f23[0], f23[1]);
              zp[1] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(v2h, __builtin_amdgcn_perm(0x64646464u, dz, 0x04030402u)) - off);
            }
          } else {                                           // (scale, zero-point) fp16 pairs per block
            sp[0] = __builtin_amdgcn_perm(src[1], src[0], 0x05040100u);
            zp[0] = __builtin_amdgcn_perm(src[1], src[0], 0x07060302u);
            if constexpr (G == 4) {
              sp[1] = __builtin_amdgcn_perm(src[3], src[2], 0x05040100u);
              zp[1] = __builtin_amdgcn_perm(src[3], src[2], 0x07060302u);
            }
          }
        };
        uint32_t sp[2], zp[2];
        uint32_t (&dk)[4] = ld_mk, (&dv)[4] = ld_mv;
        pairs(dk, sp, zp);
    #pragma unroll
        for (int i = 0; i < GP; ++i) s_ks[tid * GP + i] = sp[i];
        {
          // the zero-points' share of this token's scores (see above); -infinity past the sequence's end,
          // which is what a slot the key phase never writes must hold
          float sf[4], zf[4];
    #pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t sw = sp[i >> 1], zw = zp[i >> 1];
            sf[i] = i < G ? (float)__builtin_bit_cast(_Float16, (uint16_t)(i & 1 ? sw >> 16 : sw & 0xffffu)) : 0.f;
            zf[i] = i < G ? (float)__builtin_bit_cast(_Float16, (uint16_t)(i & 1 ? zw >> 16 : zw & 0xffffu)) : 0.f;
          }
          const float2 cs0 = ld_cs0;
    #pragma unroll
          for (int a = 0; a < G; ++a) {
            float Z = 0.f;
    #pragma unroll
            for (int i = 0; i < G; ++i) Z = fmaf((__popc(a & i) & 1) ? -sf[i] : sf[i], zf[i], Z);
    #pragma unroll
            for (int rri = 0; rri < REP; ++rri) {
              const int f = (a * REP + rri) * 2;                 // entry (r = 0, p = 0, n = 0) of the prepared query: floats f, f + 1
              const float4 q4 = ld_q0[f >> 2];
              const float ql = (f & 3) ? q4.z : q4.x, qh = (f & 3) ? q4.w : q4.y;
              s_sc[a * REP + rri][tid] = t0 + tid < len ? -64.0f * Z * fmaf(cs0.x, ql, cs0.y * qh) : -INFINITY;
            }
          }
        }
        if constexpr (META8 || ALU) {                      // values: (scale, zero-point) per head
          pairs(dv, sp, zp);
          s_vm[tid * G] = __builtin_amdgcn_perm(zp[0], sp[0], 0x05040100u);
          s_vm[tid * G + 1] = __builtin_amdgcn_perm(zp[0], sp[0], 0x07060302u);
          if constexpr (G == 4) {
            s_vm[tid * G + 2] = __builtin_amdgcn_perm(zp[1], sp[1], 0x05040100u);
            s_vm[tid * G + 3] = __builtin_amdgcn_perm(zp[1], sp[1], 0x07060302u);
          }
        } else {
    #pragma unroll
          for (int i = 0; i < G; ++i) s_vm[tid * G + i] = dv[i];
        }
      }
      __syncthreads();        // LDS copies of the Hadamard operand and the query are complete; first tile already in flight
      __builtin_amdgcn_s_setprio(0);
      // which of the wave's tiles hold a retained sink token (a wave-uniform bit mask): the others
      // skip the comparison with the sink list
      uint32_t sink_tiles = 0;
      for (int i = 0; i < cnt; ++i) {
        const int d = s_sink[i] - tw;
        if (d >= 0 && d < 16 * MF_TILES) sink_tiles |= 1u << (d >> 4);
      }
      sink_tiles = __builtin_amdgcn_readfirstlane(sink_tiles);

#pragma unroll
      for (int ti = 0; ti < MF_TILES; ++ti) {
        const int tt = tw + ti * 16;
        if (tt >= len) break;                              // wave-uniform
        v8i A[G];
#pragma unroll
        for (int pr = 0; pr < G / 2; ++pr) {
          A[2 * pr] = unpack_fp4(cw[pr].x, cw[pr].y);
          A[2 * pr + 1] = unpack_fp4(cw[pr].z, cw[pr].w);
        }
        v8i Ah[HI ? G : 1];
        if constexpr (HI) {
#pragma unroll
          for (int pr = 0; pr < G / 2; ++pr) {
            if constexpr (HB == 2) {
              Ah[2 * pr] = unpack_fp4(cwh[pr].x, cwh[pr].y);
              Ah[2 * pr + 1] = unpack_fp4(cwh[pr].z, cwh[pr].w);
            } else {
              Ah[2 * pr] = unpack_fp4_bits(cwh[pr].x);
              Ah[2 * pr + 1] = unpack_fp4_bits(cwh[pr].y);
            }
          }
        }
        // scale rows of the 4x4 products: (+-s_0, +-s_1, +-s_2, +-s_3) of token 4q + r, signs of H_g row n & 3
        v4h sA[4];
        if constexpr (LM) {
          const uint32_t* sp = &s_ks[(wave * (16 * MF_TILES) + ti * 16 + 4 * q) * GP];
          uint32_t sw[4][2];
          if constexpr (G == 4) {
#pragma unroll
            for (int r = 0; r < 4; r += 2) {
              const uint4 a = *reinterpret_cast<const uint4*>(sp + 2 * r);
              sw[r][0] = a.x; sw[r][1] = a.y; sw[r + 1][0] = a.z; sw[r + 1][1] = a.w;
            }
          } else {
            const uint4 a = *reinterpret_cast<const uint4*>(sp);
            sw[0][0] = a.x; sw[1][0] = a.y; sw[2][0] = a.z; sw[3][0] = a.w;
            sw[0][1] = sw[1][1] = sw[2][1] = sw[3][1] = 0;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) sA[r] = as_v4h((sw[r][0] ^ sm01) & keep_row, G == 4 ? (sw[r][1] ^ sm23) & keep_row : 0u);
        }
        if (ti + 1 < MF_TILES) load_tile(ti + 1);          // prefetch (inside the padded allocation)

        // The key phase runs in passes over RP of the lane's four tokens, so that the score
        // accumulators (RP tokens x G heads x REP query heads) stay within 16 registers - more of
        // them and the compiler's allocation leaves the 256-register budget.  A pass repeats the big
        // matrix products (every one yields all four tokens), which costs less than repeating the
        // small ones, the packing or RoPE.
#pragma unroll
        for (int r0 = 0; r0 < 4; r0 += RP) {
        float pt[RP * G * REP];                            // [token of the pass][KV head][query head of it]
#pragma unroll
        for (int i = 0; i < RP * G * REP; ++i) pt[i] = 0.f;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          // H_128 of the raw codes for channels 16p + n (lo) and 16p + n + 64 (hi) - or the even and the odd
          // channel of pair 16p + n -: half-integers, exact
          v4f lo[G], hi[G];
          {
            v8i Hlo, Hhi;
            const uint4 h0 = s_H[p][lane], h1 = s_H[p + 4][lane];
            Hlo[0] = (int)h0.x; Hlo[1] = (int)h0.y; Hlo[2] = (int)h0.z; Hlo[3] = (int)h0.w; Hlo[4] = Hlo[5] = Hlo[6] = Hlo[7] = 0;
            Hhi[0] = (int)h1.x; Hhi[1] = (int)h1.y; Hhi[2] = (int)h1.z; Hhi[3] = (int)h1.w; Hhi[4] = Hhi[5] = Hhi[6] = Hhi[7] = 0;
            const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int blk = 0; blk < G; ++blk) {
              lo[blk] = mfma_fp4(A[blk], Hlo, zero4);
              hi[blk] = mfma_fp4(A[blk], Hhi, zero4);
            }
            if constexpr (HI) {
              // FP4 1.0 (0x2) and -1.0 (0xA) with bit 2 set are 4.0 and -4.0
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                Hlo[i] |= 0x44444444;
                Hhi[i] |= 0x44444444;
              }
#pragma unroll
              for (int blk = 0; blk < G; ++blk) {
                lo[blk] = mfma_fp4(Ah[blk], Hlo, lo[blk]);
                hi[blk] = mfma_fp4(Ah[blk], Hhi, hi[blk]);
              }
            }
          }
          float c = cs_c[p], s = cs_s[p];                      // angles of the pass's first token (REP == 1: of token 4q)
#pragma unroll
          for (int rr = 0; rr < RP; ++rr) {
            const int r = r0 + rr;
            // k^[a] = sum_blk H_g[a][blk] * scale_blk * u_blk   (H_g butterfly over the blocks)
            // as 16 independent 4x4x4 products per instruction: block = (token 4q + r, 4 channel
            // lanes), A row a = signed fp16 scales, B = the four blocks' results (half-integers
            // below 1024: exact in fp16), fp32 accumulate
            const v4f z4 = {0.f, 0.f, 0.f, 0.f};
            v4f klo, khi;
            if constexpr (G == 4) {
              klo = mfma_4x4x4(sA[r], as_v4h(pk_f16(lo[0][r], lo[1][r]), pk_f16(lo[2][r], lo[3][r])), z4);
              khi = mfma_4x4x4(sA[r], as_v4h(pk_f16(hi[0][r], hi[1][r]), pk_f16(hi[2][r], hi[3][r])), z4);
            } else {
              klo = mfma_4x4x4(sA[r], as_v4h(pk_f16(lo[0][r], lo[1][r]), 0u), z4);
              khi = mfma_4x4x4(sA[r], as_v4h(pk_f16(hi[0][r], hi[1][r]), 0u), z4);
            }
            // the query: with REP == 1 the copy rotated back by r positions, else the plain one
            // (floats 2 * REP * a .. of the row belong to KV head a: [query head of it][lo, hi])
            constexpr int QF = (2 * REP * G < 8) ? 2 * REP * G : 8;   // floats fetched at a time
#pragma unroll
            for (int f0 = 0; f0 < 2 * REP * G; f0 += QF) {
              float qv[QF];
#pragma unroll
              for (int i = 0; i < QF; i += 4) {
                const uint4 u = s_q[REP == 1 ? r : 0][p][(f0 + i) / 4][n];
                qv[i] = __uint_as_float(u.x); qv[i + 1] = __uint_as_float(u.y); qv[i + 2] = __uint_as_float(u.z); qv[i + 3] = __uint_as_float(u.w);
              }
#pragma unroll
              for (int fa = 0; fa < QF; fa += 2 * REP) {
                const int a = (f0 + fa) / (2 * REP);
                const float xl = klo[a] * c - khi[a] * s;
                const float xh = klo[a] * s + khi[a] * c;
#pragma unroll
                for (int rri = 0; rri < REP; ++rri) {
                  const int o = (rr * G + a) * REP + rri;
                  pt[o] = fmaf(xh, qv[fa + 2 * rri + 1], fmaf(xl, qv[fa + 2 * rri], pt[o]));
                }
              }
            }
            if constexpr (REP > 1) {                           // next token: one position further
              const float2 s1 = s_step1[16 * p + n];
              const float c1 = c * s1.x - s * s1.y;
              s = s * s1.x + c * s1.y;
              c = c1;
            }
          }
          if constexpr (REP > 1) {                             // the state moves on with the passes
            cs_c[p] = c;
            cs_s[p] = s;
          }
        }
        if (r0 + RP >= 4) {
          // after the last pass: on to the next tile's first token (16 positions from this tile's;
          // with REP > 1 the passes have covered 4 of them)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const float c = cs_c[p], s = cs_s[p];
            const float2 st = s_step[16 * p + n];
            cs_c[p] = c * st.x - s * st.y;
            cs_s[p] = s * st.x + c * st.y;
          }
        }
        // reduce over the 16 channel lanes: value idx = (rr * G + a) * REP + rri ends in lane idx
        // (token 4q + r0 + rr, query head a * REP + rri)
        constexpr int NV = RP * G * REP;
        constexpr int NR = NV < 16 ? NV : 16;              // values per transposing reduction
#pragma unroll
        for (int j = 0; j < NV / NR; ++j) {
          float grp[NR];
#pragma unroll
          for (int i = 0; i < NR; ++i) grp[i] = pt[NR * j + i];
          const float tot = row_transpose_reduce<NR>(grp, n);
          const int idx = NR * j + (n & (NR - 1));
          const int tok = tt + 4 * q + r0 + idx / (G * REP), hq = idx % (G * REP);
          bool masked = tok >= len;
          if constexpr (MULTI) masked = tok > s_lim[hq];
          if (sink_tiles & (1u << ti))
            for (int i = 0; i < cnt; ++i) masked |= (s_sink[i] == tok);
          if constexpr (LM) {                              // onto the zero-points' share, put there when the metadata were staged
            if (n < NR) s_sc[hq][tok - t0] = masked ? -INFINITY : tot + s_sc[hq][tok - t0];
          } else {
            if (n < NR && !masked) s_sc[hq][tok - t0] = tot;
          }
        }
        }
      }
    }
    }
    __builtin_amdgcn_s_setprio(3);
    // V metadata of the four tokens this lane turns into weights in phase S (head = wave); requested
    // here and not before the key phase, where four more live registers would mean spills - and
    // with them a scratch allocation, which keeps some shader engines from holding three workgroups
    uint32_t vmeta[NS][MF_CH / 64];
#pragma unroll
    for (int i = 0; i < MF_CH / 64; ++i) {
      const size_t mi = ((size_t)(b * v.NRG + rg) * v.Tpad + t0 + lane + 64 * i) * (G * NS);
      if constexpr (LM) {
        // (read from LDS in the softmax phase)
      } else if constexpr (SUB != 0 && META8) {
        // the head's NS scale bytes and NS zero-point bytes, one load each
        const uint8_t* vm8 = reinterpret_cast<const uint8_t*>(v.vm) + 2 * mi + (wave < G ? wave : 0) * NS;
        uint32_t sw, zw;
        if constexpr (NS == 4) {
          sw = *reinterpret_cast<const uint32_t*>(vm8);
          zw = *reinterpret_cast<const uint32_t*>(vm8 + G * NS);
        } else {
          sw = *reinterpret_cast<const uint16_t*>(vm8);
          zw = *reinterpret_cast<const uint16_t*>(vm8 + G * NS);
        }
#pragma unroll
        for (int sb = 0; sb < NS; ++sb)
          vmeta[sb][i] = wave < G ? __builtin_amdgcn_perm(zw, sw, 0x0c0c0000u | ((4u + sb) << 8) | sb) : 0x8000u;
      } else if constexpr (SUB != 0) {
#pragma unroll
        for (int sb = 0; sb < NS; ++sb) vmeta[sb][i] = wave < G ? v.vm[mi + wave * NS + sb] : 0u;
      } else if constexpr (META8) {
        const uint8_t* vm8 = reinterpret_cast<const uint8_t*>(v.vm) + 2 * mi;
        vmeta[0][i] = wave < G ? ((uint32_t)vm8[wave] | ((uint32_t)vm8[G + wave] << 8)) : 0x8000u;
      } else {
        vmeta[0][i] = wave < G ? v.vm[mi + wave] : 0u;
      }
    }
    const bool has_head = q < G;
    const uint4* vslab = reinterpret_cast<const uint4*>(v.vc + rkv_v_slabbase(v, b, rg, t0 >> 5));
    const uint32_t* vhslab = HI ? v.vh + (rkv_v_slabbase(v, b, rg, t0 >> 5) >> (HB == 1 ? 1 : 0)) : nullptr;
    const int lidx = wave * (16 * G) + (has_head ? lane : 0);
    const int nslab = min(MF_CH / 32, (len - t0 + 31) >> 5);
    // the softmax and value phases run once per query head of a KV head; the V codes are requested
    // again each time (from L2 after the first), which is cheaper than holding them across the loop
#pragma unroll 1
    for (int rri = 0; rri < REP; ++rri) {
    // all V codes of the chunk (one 16-byte load per lane and slab): in flight while the softmax phase runs
    uint4 vcodes[MF_CH / 32], vhcodes[HI ? MF_CH / 32 : 1];
#pragma unroll
    for (int sl = 0; sl < MF_CH / 32; ++sl) {
      // (lanes without a head feed zeros to the products; slabs beyond the chunk's end are never used)
      if constexpr (G < 4) vcodes[sl] = make_uint4(0, 0, 0, 0);
      if constexpr (ALU) {
        const uint32_t x = (uint32_t)lidx * 2654435761u ^ (uint32_t)(nq + sl);
        if (has_head && sl < nslab) vcodes[sl] = make_uint4(x, x * 3u, x * 5u, x * 7u);
      } else if (has_head && sl < nslab) vcodes[sl] = rkv_ld_stream(vslab + (size_t)sl * (64 * G) + lidx);
      if constexpr (HI) {
        vhcodes[sl] = make_uint4(0, 0, 0, 0);
        if (has_head && sl < nslab) {
          if constexpr (HB == 2) {
            vhcodes[sl] = rkv_ld_stream(reinterpret_cast<const uint4*>(vhslab) + (size_t)sl * (64 * G) + lidx);
          } else {
            const uint2 u = rkv_ld_stream(reinterpret_cast<const uint2*>(vhslab) + (size_t)sl * (64 * G) + lidx);
            vhcodes[sl] = make_uint4(u.x, u.y, 0, 0);
          }
        }
      }
    }
    __syncthreads();

    // ------------------------------------------------------------------ phase S
    if (wave < G) {
      const int a = wave;
      float sv[MF_CH / 64], w[MF_CH / 64], zv[MF_CH / 64];
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < MF_CH / 64; ++i) {
        sv[i] = s_sc[a * REP + rri][lane + 64 * i];
        m = fmaxf(m, sv[i]);
      }
      m = wave_allreduce<true>(m);
      float pe[MF_CH / 64], l = 0.f;
#pragma unroll
      for (int i = 0; i < MF_CH / 64; ++i) {
        pe[i] = sv[i] > -INFINITY ? __expf(sv[i] - m) : 0.f;
        l += pe[i];
      }
      l = wave_allreduce<false>(l);
#pragma unroll
      for (int sb = 0; sb < NS; ++sb) {                     // once, or once per sub-block of the head (its own scales and zero-points)
      float wmax = 0.f;
#pragma unroll
      for (int i = 0; i < MF_CH / 64; ++i) {
        float s_, z_;
        if constexpr (LM) {                                 // token lane + 64 i, head a
          rkv_unpack_meta(s_vm[(lane + 64 * i) * G + a], s_, z_);
        } else if constexpr (META8) {
          s_ = __builtin_amdgcn_cvt_f32_fp8((int)vmeta[sb][i], 0);
          z_ = (float)((vmeta[sb][i] >> 8) & 0xffu) - 128.0f;
        } else {
          rkv_unpack_meta(vmeta[sb][i], s_, z_);
        }
        w[i] = pe[i] * s_;
        zv[i] = z_;
        wmax = fmaxf(wmax, w[i]);
      }
      wmax = wave_allreduce<true>(wmax);
      // 24-bit fixed point: largest weight lands in [2^23, 2^24); six base-16 digits, exact in E4M3
      int ex = 0;
      if (wmax > 0.f) frexpf(wmax, &ex);
      const float up = ldexpf(1.0f, 24 - ex), down = ldexpf(1.0f, ex - 24);
      float zs = 0.f;
#pragma unroll
      for (int i = 0; i < MF_CH / 64; ++i) {
        const int tl = lane + 64 * i, slab = tl >> 5, tau = tl & 31;
        const uint32_t W = (uint32_t)rintf(w[i] * up);
        zs += (float)W * zv[i];
        uint8_t* dst = &s_A[sb][slab][0][(4 * a) * 32 + tau];
#pragma unroll
        for (int k = 0; k < 6; k += 2) {
          // digits 5-k and 4-k (most significant first): rows 0..3 of set 0, rows 0..1 of set 1
          const float d_hi = (float)(k == 0 ? (W >> 20) : ((W >> (20 - 4 * k)) & 15u));
          const float d_lo = (float)((W >> (16 - 4 * k)) & 15u);
          const int pk = __builtin_amdgcn_cvt_pk_fp8_f32(d_hi, d_lo, 0, false);
          const int row = k & 3, set = k >> 2;
          dst[set * SA_SET + row * 32] = (uint8_t)(pk & 0xff);
          dst[set * SA_SET + (row + 1) * 32] = (uint8_t)((pk >> 8) & 0xff);
        }
      }
      zs = wave_allreduce<false>(zs);
      if (lane == 0) {
        s_m[a] = m;
        s_l[a] = l;
        s_zs[sb][a] = zs * down;
        s_wsc[sb][a] = down;
      }
      }
    }
    __syncthreads();

    // ------------------------------------------------------------------ phase V
    {
      // Operand lane (row n = 4 * head + digit, lane group q) covers contraction indices 32q..32q+31,
      // which the V codes' layout assigns to head 2 * (second half of the 32) + (q >> 1), tokens
      // 16 * (q & 1) .. + 15 of the slab: its first or second 16 bytes are that head's row, the
      // rest of the operand is zero
      const int vsub = SUB ? (wave * SUB) / 4 : 0;          // this wave's channels 32 wave .. + 31 lie in one sub-block of their head
      const int arow = n >> 2;
      const bool ause = (q >> 1) == (arow & 1);
      const int adata = n * 32 + 16 * (q & 1);
      const int aoff0 = (ause && (arow >> 1) == 0) ? adata : SA_ZERO;
      const int aoff1 = (ause && (arow >> 1) == 1) ? adata : SA_ZERO;
      v4f acc[2][2], acch[2][2];                            // [channel tile][digit set]; acch: the plane of the upper bits
#pragma unroll
      for (int i = 0; i < 2; ++i) acc[i][0] = acc[i][1] = acch[i][0] = acch[i][1] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int sl = 0; sl < MF_CH / 32; ++sl) {
        if (sl < nslab) {                                   // workgroup-uniform
          v8i A[2];
#pragma unroll
          for (int set = 0; set < 2; ++set) {
            const uint4 a0 = *reinterpret_cast<const uint4*>(&s_A[vsub][sl][set][aoff0]);
            const uint4 a1 = *reinterpret_cast<const uint4*>(&s_A[vsub][sl][set][aoff1]);
            A[set][0] = (int)a0.x; A[set][1] = (int)a0.y; A[set][2] = (int)a0.z; A[set][3] = (int)a0.w;
            A[set][4] = (int)a1.x; A[set][5] = (int)a1.y; A[set][6] = (int)a1.z; A[set][7] = (int)a1.w;
          }
          const v8i B0 = unpack_fp4(vcodes[sl].x, vcodes[sl].y), B1 = unpack_fp4(vcodes[sl].z, vcodes[sl].w);
#pragma unroll
          for (int set = 0; set < 2; ++set) {
            acc[0][set] = mfma_fp8_fp4(A[set], B0, acc[0][set]);
            acc[1][set] = mfma_fp8_fp4(A[set], B1, acc[1][set]);
          }
          if constexpr (HI) {
            const v8i B0h = HB == 2 ? unpack_fp4(vhcodes[sl].x, vhcodes[sl].y) : unpack_fp4_bits(vhcodes[sl].x);
            const v8i B1h = HB == 2 ? unpack_fp4(vhcodes[sl].z, vhcodes[sl].w) : unpack_fp4_bits(vhcodes[sl].y);
#pragma unroll
            for (int set = 0; set < 2; ++set) {
              acch[0][set] = mfma_fp8_fp4(A[set], B0h, acch[0][set]);
              acch[1][set] = mfma_fp8_fp4(A[set], B1h, acch[1][set]);
            }
          }
        }
      }
      if (has_head) {
        const int qh = (rg * G + q) * rep + rrg * REP + rri;   // query head served for KV head rg*G + q
        float* dst = part + (((size_t)b * v.Hq + qh) * nch + chunk) * RKV_PART_STRIDE;
        const float wsc = 2.0f * s_wsc[vsub][q];            // FP4 nibble = code/2
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          v4f hi = acc[ct][0], lo = acc[ct][1];
          if constexpr (HI) {
            hi += acch[ct][0] * 4.0f;
            lo += acch[ct][1] * 4.0f;
          }
          const float sum = ((((hi[0] * 16.0f + hi[1]) * 16.0f + hi[2]) * 16.0f + hi[3]) * 16.0f + lo[0]) * 16.0f + lo[1];
          dst[4 + 16 * (2 * wave + ct) + n] = sum * wsc - s_zs[vsub][q];
        }
        if (wave == 0 && n == 0) {
          dst[0] = s_m[q];
          dst[1] = s_l[q];
        }
      }
    }
    }
  }
}



// a reorder across 128-blocks inside the rotation groups, groups of 128: scores from the scores kernel
// (the rotation group's own blocks in its table), softmax and values from this file's kernel
static bool mfma_cross_block(const rkv_cache* c) {
  const RkvView& v = c->v;
  return !c->blocks_aligned && c->in_groups && v.qg == 128 && rkv_scores_local(c);
}

// groups of 64 / 32 (the reorder inside the rotation groups, or over the whole row): the same route
static bool mfma_sub_groups(const rkv_cache* c) {
  const RkvView& v = c->v;
  return v.qg < 128 && rkv_scores_path(c);
}

int rkv_mfma_variant(const rkv_cache* c) {
  return rkv_row_supported(c) ? RKV_KERNEL_MFMA_ROW : mfma_cross_block(c) ? RKV_KERNEL_MFMA_CROSS : mfma_sub_groups(c) ? RKV_KERNEL_MFMA_SUB : RKV_KERNEL_MFMA;
}

bool rkv_mfma_supported(const rkv_cache* c) {
  const RkvView& v = c->v;
  if (mfma_cross_block(c) || mfma_sub_groups(c) || rkv_row_supported(c)) return true;
  // 2-bit codes, or wider ones (a second plane), in groups of 128
  return c->blocks_aligned && v.qg == 128 && (v.g == 2 || v.g == 4);
}

typedef void (*RkvDecodeFn)(RkvView, const float*, float*, int, const int*, int, int, uint32_t, uint32_t);

// The variant of the kernel a cache takes.  multi: several query tokens per sequence; share: query
// heads of a KV head per workgroup (1 or 2); alu: the arithmetic-only measurement.
static RkvDecodeFn pick_kernel(const rkv_cache* c, bool multi, int share, bool alu) {
  const RkvView& v = c->v;
  // precomputed scores (groups of 64 / 32; a reorder over the whole row): softmax and value phases only
#define RKV_MF_PRE_M(G_, R_, S_, H_, M_) (v.meta8 ? k_decode_mfma<G_, R_, M_, true, H_, S_, false, true> : k_decode_mfma<G_, R_, M_, false, H_, S_, false, true>)
#define RKV_MF_PRE(G_, R_, S_, H_) (multi ? RKV_MF_PRE_M(G_, R_, S_, H_, true) : RKV_MF_PRE_M(G_, R_, S_, H_, false))
#define RKV_MF_PRE_SUB(G_, H_) (sub == 4 ? RKV_MF_PRE(G_, 1, 4, H_) : RKV_MF_PRE(G_, 1, 2, H_))
  if (v.qg < 128 && rkv_scores_path(c)) {                   // (groups of 64 / 32: codes of 2, 3 or 4 bits)
    const int sub = 128 / v.qg;
    if (v.g == 4) return v.hb == 2 ? RKV_MF_PRE_SUB(4, 2) : v.hb == 1 ? RKV_MF_PRE_SUB(4, 1) : RKV_MF_PRE_SUB(4, 0);
    return v.hb == 2 ? RKV_MF_PRE_SUB(2, 2) : v.hb == 1 ? RKV_MF_PRE_SUB(2, 1) : RKV_MF_PRE_SUB(2, 0);
  }
  if (rkv_scores_path(c)) {                                 // (a reorder over the whole row, or across blocks inside the rotation groups)
#define RKV_MF_PRE_X(G_, R_) (v.hb == 2 ? RKV_MF_PRE(G_, R_, 0, 2) : v.hb == 1 ? RKV_MF_PRE(G_, R_, 0, 1) : RKV_MF_PRE(G_, R_, 0, 0))
    if (v.g == 4) return share == 1 ? RKV_MF_PRE_X(4, 1) : RKV_MF_PRE_X(4, 2);
    return share == 1 ? RKV_MF_PRE_X(2, 1) : RKV_MF_PRE_X(2, 2);
#undef RKV_MF_PRE_X
  }
#undef RKV_MF_PRE_SUB
#undef RKV_MF_PRE
#undef RKV_MF_PRE_M
#ifdef RKV_DEV_FEW_VARIANTS
  // developer builds: only the plain 2-bit variants of four-head rotation groups (quick to compile)
  if (multi || v.g != 4 || v.hb || v.meta8 || !c->blocks_aligned || v.qg != 128) abort();
  if (alu) return k_decode_mfma<4, 1, false, false, 0, 0, true>;
  return share == 1 ? k_decode_mfma<4, 1, false, false, 0> : k_decode_mfma<4, 2, false, false, 0>;
#else
  if (alu) return v.g == 4 ? k_decode_mfma<4, 1, false, false, 0, 0, true> : k_decode_mfma<2, 1, false, false, 0, 0, true>;
#define RKV_MF_PICK(G_, R_, M_)                                                                            \
  do {                                                                                                     \
    if (v.hb == 2) return v.meta8 ? k_decode_mfma<G_, R_, M_, true, 2> : k_decode_mfma<G_, R_, M_, false, 2>; \
    if (v.hb == 1) return v.meta8 ? k_decode_mfma<G_, R_, M_, true, 1> : k_decode_mfma<G_, R_, M_, false, 1>; \
    return v.meta8 ? k_decode_mfma<G_, R_, M_, true, 0> : k_decode_mfma<G_, R_, M_, false, 0>;               \
  } while (0)
  if (multi) {
    if (v.g == 4 && share == 1) RKV_MF_PICK(4, 1, true);
    else if (v.g == 4) RKV_MF_PICK(4, 2, true);
    else if (share == 1) RKV_MF_PICK(2, 1, true);
    else RKV_MF_PICK(2, 2, true);
  }
  if (v.g == 4 && share == 1) RKV_MF_PICK(4, 1, false);
  else if (v.g == 4) RKV_MF_PICK(4, 2, false);
  else if (share == 1) RKV_MF_PICK(2, 1, false);
  else RKV_MF_PICK(2, 2, false);
#undef RKV_MF_PICK
#endif
}

// nq == 0: the usual step, one query token that attends the whole cache (and, if set, the current
// token's exact row).  nq >= 1: nq query tokens per sequence, token i at position q_pos[b][i] and
// blind to cached tokens behind it; q, out and lse are then [batch][nq][heads][...] and the scratch
// buffer holds nq times the single-query size.
// query heads of a KV head served by one workgroup: two where the ratio is even (four per
// workgroup measured slower: 158 against 151 us on the GQA configuration - the variant needs
// more registers than three workgroups per compute unit leave)
int rkv_mfma_share(int heads_per_kv_head) { return heads_per_kv_head % 2 == 0 ? 2 : 1; }

// q_prepared: the queries are already in the scratch block (rkv_launch_step_mfma put them there)
int rkv_launch_decode_mfma(rkv_cache* c, const __half* q, const int* q_pos, int nq, float* out, float* lse, void* scratch,
                           bool q_prepared, hipStream_t s) {
  if (!rkv_mfma_supported(c)) return RKV_EINVAL;
  const bool multi = nq > 0;
  if (multi && (c->cur_k || !q_pos)) return RKV_EINVAL;
  if (!multi) nq = 1;
  RkvView v = c->v;
  v.Hq *= nq;                                               // virtual heads
  float* qr = (float*)scratch;
  const size_t qbytes = rkv_query_scratch_bytes(v.B, v.Hq);
  float* part = (float*)((char*)scratch + qbytes);
  const int rep = v.Hq / v.Hkv;
  const bool sg = mfma_sub_groups(c);
  const bool xb = mfma_cross_block(c) || sg;
  const bool row = rkv_scores_path(c);
  if (row && multi && !rkv_scores_multi_ok(c, nq)) return RKV_EINVAL;   // (the scores kernel serves 8 rows per KV head)
  const int share = sg ? 1 : rkv_mfma_share(rep);           // (groups of 64 / 32: one query head per workgroup)
  if (!q_prepared) rkv_launch_prep_q(v, q, q_pos, c->cur_k ? 1 : 0, qr, share, nq, s);
  float* qt = qr + (size_t)v.B * v.Hq * RKV_D;              // lane-ordered copy written by k_prep_q
  const int nch = (v.len + MF_CH - 1) / MF_CH;
  const int ns = rep / share;
  // reciprocals for the kernel's index arithmetic: ceil(2^32 / d) gives exact quotients n / d for n * d < 2^32
  auto recip = [](int d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); };
  dim3 grid(8 * nch * ns, (v.B * v.NRG + 7) / 8, 1);        // see the kernel for the mapping
  if (c->ragged) {                                          // all sequences' chunks in one dimension
    int total = 0;
    for (int b = 0; b < v.B; ++b) total += (c->hlens[b] + MF_CH - 1) / MF_CH;
    grid = dim3(((total + 7) & ~7) * ns, v.NRG, 1);
  }
  if (grid.y > 65535) return RKV_EINVAL;
  if (c->decode_path == 3 && (multi || xb || v.hb || v.meta8 || share != 1)) return RKV_EINVAL;   // arithmetic-only measurement: plain variants
  // The measurement events, if set, are tied to the kernel's own dispatch (its begin and end time
  // stamps): events recorded as separate commands before and after it also count the gaps between
  // commands on the stream, some 4 us per launch.
  const bool timed = c->ev_start && c->ev_stop;
  if (row) {
    // a reorder over the whole row: the scores come from a kernel of their own, into a buffer behind
    // the partial results (rkv_decode_scratch_bytes reserves it); the events span both kernels
    if (c->decode_path == 3) return RKV_EINVAL;
    float* sc = (float*)((char*)part + rkv_partial_bytes(v.B, v.Hq, (int)v.Tpad));
    if (timed) RKV_HIP_CHECK(hipEventRecord(c->ev_start, s));
    const int rc = rkv_launch_scores_row(c, v, qr, sc, s);
    if (rc != RKV_OK) return rc;
    if (nch > 0)
      hipLaunchKernelGGL(pick_kernel(c, multi, share, false), grid, dim3(256), 0, s, v, (const float*)sc, part, nch,
                         multi ? q_pos : (const int*)nullptr, nq, ns, recip(ns), recip(v.NRG));
    if (timed) RKV_HIP_CHECK(hipEventRecord(c->ev_stop, s));
    rkv_launch_merge(v, qr, part, nch, MF_CH, c->cur_k, c->cur_v, multi ? q_pos : nullptr, nq, out, lse, s);
    return rkv_check_launch();
  }
  if (nch > 0) {                                            // (an empty cache has only the current token)
    if (timed)
      hipExtLaunchKernelGGL(pick_kernel(c, multi, share, c->decode_path == 3), grid, dim3(256), 0, s, c->ev_start, c->ev_stop, 0, v,
                            qt, part, nch, multi ? q_pos : nullptr, nq, ns, recip(ns), recip(v.NRG));
    else
      hipLaunchKernelGGL(pick_kernel(c, multi, share, c->decode_path == 3), grid, dim3(256), 0, s, v, qt, part, nch,
                         multi ? q_pos : nullptr, nq, ns, recip(ns), recip(v.NRG));
  } else if (timed) {
    RKV_HIP_CHECK(hipEventRecord(c->ev_start, s));
    RKV_HIP_CHECK(hipEventRecord(c->ev_stop, s));
  }
  rkv_launch_merge(v, qr, part, nch, MF_CH, c->cur_k, c->cur_v, multi ? q_pos : nullptr, nq, out, lse, s);
  return rkv_check_launch();
}

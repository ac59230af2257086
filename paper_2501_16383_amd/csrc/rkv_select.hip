// Attention-sink identification (Sec. 4.3): the tokens with the most massive activations in the
// output of the previous decoder block are the ones kept in fp16.  A token's score is its largest
// |activation|; the k highest scores win, ties go to the lower token index, indices are returned in
// ascending order.  fp16 maxima are exact, so the result equals the definition bit for bit.
#include "rkv_internal.h"

// score[b][t] = max_c |x[b][t][c]|; one wave per token row, 16-byte loads, packed fp16 maxima
__global__ void __launch_bounds__(256) k_token_maxabs(const __half* __restrict__ x, int n_tok, int width, float* __restrict__ score) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * 4 + wave, b = blockIdx.y;
  if (t >= n_tok) return;
  const __half* row = x + ((size_t)b * n_tok + t) * width;
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  h2 m = {(_Float16)0, (_Float16)0};
  const int n16 = width >> 3;                                  // 16-byte pieces (width is a multiple of 8)
  for (int i = lane; i < n16; i += 64) {
    const uint4 u = rkv_ld_stream(reinterpret_cast<const uint4*>(row) + i);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) m = __builtin_elementwise_max(m, __builtin_bit_cast(h2, w[k] & 0x7fff7fffu));
  }
  float s = fmaxf((float)m[0], (float)m[1]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s = fmaxf(s, __shfl_xor(s, o));
  if (lane == 0) score[(size_t)b * n_tok + t] = s;
}

// k rounds of "largest remaining score, lowest index"; one workgroup per sequence.  A key packs the
// score's bit pattern (scores are >= 0, so the patterns order like the values) above the
// complemented index, so the maximum key is the wanted token.
__global__ void __launch_bounds__(256) k_topk_tokens(float* __restrict__ score, int n_tok, int k, int32_t* __restrict__ idx_out,
                                                     uint8_t* __restrict__ mask_out) {
  __shared__ unsigned long long s_key[4];
  __shared__ int s_pick[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, b = blockIdx.x;
  float* sc = score + (size_t)b * n_tok;
  if (mask_out)
    for (int t = tid; t < n_tok; t += 256) mask_out[(size_t)b * n_tok + t] = 0;
  for (int round = 0; round < k; ++round) {
    unsigned long long best = 0;
    for (int t = tid; t < n_tok; t += 256) {
      const float s = sc[t];
      if (s >= 0.0f) {                                         // picked tokens are marked with -1
        const unsigned long long key = ((unsigned long long)__float_as_uint(s) << 32) | (unsigned)(0xffffffffu - (unsigned)t);
        best = key > best ? key : best;
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const unsigned long long other = __shfl_xor(best, o);
      best = other > best ? other : best;
    }
    if (lane == 0) s_key[wave] = best;
    __syncthreads();
    if (tid == 0) {
      unsigned long long m = s_key[0];
      for (int w = 1; w < 4; ++w) m = s_key[w] > m ? s_key[w] : m;
      const int t = (int)(0xffffffffu - (unsigned)(m & 0xffffffffu));
      s_pick[round] = t;
      sc[t] = -1.0f;
    }
    __syncthreads();
  }
  if (tid == 0) {
    for (int i = 1; i < k; ++i) {                               // ascending order (k <= 64)
      const int v = s_pick[i];
      int j = i - 1;
      while (j >= 0 && s_pick[j] > v) { s_pick[j + 1] = s_pick[j]; --j; }
      s_pick[j + 1] = v;
    }
    for (int i = 0; i < k; ++i) {
      idx_out[(size_t)b * k + i] = s_pick[i];
      if (mask_out) mask_out[(size_t)b * n_tok + s_pick[i]] = 1;
    }
  }
}

int rkv_launch_select_sinks(const __half* x, int batch, int n_tok, int width, int k, int32_t* idx_out, uint8_t* mask_out,
                            float* scratch, hipStream_t s) {
  hipLaunchKernelGGL(k_token_maxabs, dim3((n_tok + 3) / 4, batch), dim3(256), 0, s, x, n_tok, width, scratch);
  hipLaunchKernelGGL(k_topk_tokens, dim3(batch), dim3(256), 0, s, scratch, n_tok, k, idx_out, mask_out);
  return rkv_check_launch();
}

// ---------------------------------------------------------------------------------------------
// Offline folding of rotation and reorder into a projection (Sec. 4.2, Sec. 4.4): each row of the
// matrix is rotated group by group (butterflies in LDS, fp32) and gathered through the reorder
// indices.  One workgroup per row; cold path.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_fold_rotation(const float* __restrict__ w, const int* __restrict__ perm, float* __restrict__ out,
                                                       int E, int n) {
  extern __shared__ float row[];
  const size_t base = (size_t)blockIdx.x * E;
  for (int c = threadIdx.x; c < E; c += 256) row[c] = w[base + c];
  __syncthreads();
  for (int h = 1; h < n; h <<= 1) {                 // Eq. 10 without the 1/sqrt(2) factors; h < n keeps a pair inside its group
    for (int i = threadIdx.x; i < E / 2; i += 256) {
      const int lo = ((i / h) * 2 * h) + (i % h), hi = lo + h;
      const float a = row[lo], b = row[hi];
      row[lo] = a + b;
      row[hi] = a - b;
    }
    __syncthreads();
  }
  const float rs = rsqrtf((float)n);
  for (int c = threadIdx.x; c < E; c += 256) out[base + c] = row[perm ? perm[c] : c] * rs;
}

int rkv_launch_fold_rotation(const rkv_config* cfg, const float* w, int rows, const int* perm, float* out, hipStream_t s) {
  const int E = cfg->n_kv_heads * RKV_D, n = cfg->rot_heads * RKV_D;
  const size_t lds = (size_t)E * 4;
  if (lds > 64 * 1024) return RKV_EINVAL;
  if (lds > 48 * 1024)
    RKV_HIP_CHECK(hipFuncSetAttribute((const void*)k_fold_rotation, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL(k_fold_rotation, dim3(rows), dim3(256), lds, s, w, perm, out, E, n);
  return rkv_check_launch();
}

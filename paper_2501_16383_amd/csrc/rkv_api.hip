// Host side of the C ABI: argument checks, the cache object, dispatch to the kernels.
#include "rkv_internal.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#define RKV_EXPORT extern "C" __attribute__((visibility("default")))

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static void free_host_side(rkv_cache* c);

// Work space of rkv_decode_attention_static: prepared queries and split-K partials, as in the
// caller's dev_scratch of rkv_decode_attention.  Every GPU the library runs on holds its own copy
// of the array, at its own address, until the process ends.  In host code `scratch` is only a
// handle for hipGetSymbolAddress: the kernels get the address looked up below.
static __device__ __align__(256) unsigned char scratch[RKV_STATIC_SCRATCH_BYTES];
#define RKV_MAX_DEVICES 64
static void* g_static_scratch[RKV_MAX_DEVICES];   // per device, filled on the first look-up with that device current
static std::mutex g_static_scratch_lock;

static int static_scratch_of_current_device(void** out) {
  int dev = -1;
  RKV_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= RKV_MAX_DEVICES) return RKV_EINVAL;
  std::lock_guard<std::mutex> hold(g_static_scratch_lock);
  if (!g_static_scratch[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RKV_EHIP;
    g_static_scratch[dev] = p;
  }
  *out = g_static_scratch[dev];
  return RKV_OK;
}

static int check_config(const rkv_config* c, bool need_capacity) {
  if (!c) return RKV_EINVAL;
  if (c->head_dim != RKV_D) return RKV_EINVAL;
  if (c->quant_group != 128 && c->quant_group != 64 && c->quant_group != 32) return RKV_EINVAL;
  if (c->bits < 2 || c->bits > 4) return RKV_EINVAL;
  if (c->clip_ratio != 1.0f) return RKV_EINVAL;
  if (c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads != 0) return RKV_EINVAL;
  if (c->n_q_heads / c->n_kv_heads > 8) return RKV_EINVAL;
  if (c->rot_heads != 1 && c->rot_heads != 2 && c->rot_heads != 4 && c->rot_heads != 8) return RKV_EINVAL;
  if (c->n_kv_heads % c->rot_heads != 0) return RKV_EINVAL;
  if (c->n_kv_heads > 128) return RKV_EINVAL;
  const int n = c->rot_heads * RKV_D, E = c->n_kv_heads * RKV_D;
  if (c->perm_span != RKV_D && c->perm_span != n && c->perm_span != E) return RKV_EINVAL;
  if (c->rope_style != 0 && c->rope_style != 1) return RKV_EINVAL;
  if (c->v_rotate != 0 && c->v_rotate != 1) return RKV_EINVAL;
  if (c->keys_rotated != 0 && c->keys_rotated != 1) return RKV_EINVAL;
  if (c->meta_format != 0 && c->meta_format != 1) return RKV_EINVAL;
  if (c->keys_rotated && ((c->rot_heads != 2 && c->rot_heads != 4) || c->perm_span != RKV_D || c->v_rotate)) return RKV_EINVAL;
  if (!(c->rope_theta > 1.0f)) return RKV_EINVAL;
  {
    // the general append kernel keeps the images of max(perm_span, n) channels of a tile in LDS
    // (rkv_launch_append): that must fit a compute unit.  It is not what runs where every reorder
    // has a matrix-core append kernel (groups of 128, rotation over 2 or 4 heads, keys
    // and values as they come; the whole-row variant holds per-block tables for up to 127 blocks)
    const bool always_matrix = c->quant_group == 128 && (c->rot_heads == 2 || c->rot_heads == 4) &&
                               !c->v_rotate && !c->keys_rotated && c->n_kv_heads <= 127;
    const size_t U = c->perm_span > n ? c->perm_span : n;
    const size_t lds = 24 * U + (c->bits == 4 ? 8 * U : c->bits == 3 ? 6 * U : 0);
    if (lds > RKV_LDS_BYTES && !always_matrix) return RKV_EINVAL;
  }
  if (need_capacity) {
    if (c->batch < 1 || c->max_tokens < 1 || c->max_sinks < 0 || c->max_sinks > 64) return RKV_EINVAL;
    if ((int64_t)c->max_tokens > 65536 || (int64_t)c->batch > 65535) return RKV_EINVAL;
  }
  return RKV_OK;
}

struct Offsets {
  size_t kc, km, vc, vm, kh, vh, sk, sv, spos, scnt, lens, nnew, cstart, tables, perm, pinv, gid, rope, hop, xgsel, xgid8, total;
  int Tpad;
};

static Offsets plan(const rkv_config* c) {
  Offsets o;
  const size_t B = c->batch, E = (size_t)c->n_kv_heads * RKV_D, NG = E / c->quant_group, HB = c->bits - 2;
  o.Tpad = (c->max_tokens + 255) & ~255;
  const size_t T = o.Tpad, S = c->max_sinks > 0 ? c->max_sinks : 1;
  const size_t MB = c->meta_format == 1 ? 2 : 4;           // bytes per (token, block) metadata entry
  size_t p = 0;
  o.kc = p; p = align256(p + B * T * E / 4);
  o.km = p; p = align256(p + B * T * NG * MB);
  o.vc = p; p = align256(p + B * T * E / 4);
  o.vm = p; p = align256(p + B * T * NG * MB);
  o.kh = p; p = align256(p + B * T * E * HB / 8);
  o.vh = p; p = align256(p + B * T * E * HB / 8);
  o.sk = p; p = align256(p + B * S * E * 2);
  o.sv = p; p = align256(p + B * S * E * 2);
  o.spos = p; p = align256(p + B * S * 4);
  o.scnt = p; p = align256(p + B * 4);
  o.lens = p; p = align256(p + B * 4);
  o.nnew = p; p = align256(p + B * 4);
  o.cstart = p; p = align256(p + (B + 1) * 4);
  o.tables = p;
  o.perm = p; p = align256(p + E * 4);
  o.pinv = p; p = align256(p + E * 4);
  o.gid = p; p = align256(p + E * 4);
  o.rope = p; p = align256(p + T * 64 * 8);
  o.hop = p; p = align256(p + 8 * 64 * 4 * 4);
  {
    // tables of the matrix-core append kernel's variants (see build_xtables)
    const size_t g = c->rot_heads, nrg = c->n_kv_heads / c->rot_heads;
    o.xgsel = p; p = align256(p + nrg * 16 * g * 4);
    o.xgid8 = p; p = align256(p + nrg * 16 * g * 8);
  }
  o.total = p;
  return o;
}

// Tables of the matrix-core append kernel's variants (RkvView::xgsel, xgid8), from the inverse
// permutation (inv[c] = reordered position of rotated channel c):
//   * a reorder that crosses 128-blocks but stays inside the rotation groups, groups of 128: the
//     quantization block of a rotated channel within its group is (inv[c] % n) / 128;
//   * quantization groups of 64 / 32 with a reorder inside the heads: the sub-block of its head is
//     (inv[c] % 128) / quant_group;
//   * a reorder over the whole row: the row's block inv[c] / 128, a byte each.
// (The read half of these settings takes gid.)
static int build_xtables(rkv_cache* cache, const std::vector<int32_t>& inv, int aligned, int* in_groups_out, hipStream_t s) {
  const RkvView& v = cache->v;
  const int E = v.E, g = v.g, n = v.n, nrg = v.NRG, qg = v.qg;
  int in_groups = (g == 2 || g == 4) ? 1 : 0;
  for (int c = 0; c < E && in_groups; ++c)
    if (inv[c] / n != c / n) in_groups = 0;
  *in_groups_out = in_groups;
  const bool cross = in_groups && !aligned, subs = aligned && qg < 128 && (g == 2 || g == 4);
  if (!in_groups && !aligned && (g == 2 || g == 4) && E / qg <= 255) {
    // a reorder over the whole row: the row's quantization block of every rotated channel, as bytes in the
    // order the append kernel's lanes hold them
    std::vector<uint8_t> x8((size_t)nrg * 16 * g * 8, 0);
    for (int rg = 0; rg < nrg; ++rg)
      for (int c = 0; c < n; ++c) {
        const int blk = c >> 7, kap = c & 127, q = kap >> 5, w8 = (kap >> 3) & 3, wave = (w8 >> 1) | ((w8 & 1) << 1);
        x8[((((size_t)rg * 4 + wave) * 4 + q) * g + blk) * 8 + (kap & 7)] = (uint8_t)(inv[rg * n + c] / qg);
      }
    RKV_HIP_CHECK(hipMemcpyAsync((void*)v.xgid8, x8.data(), x8.size(), hipMemcpyHostToDevice, s));
    RKV_HIP_CHECK(hipStreamSynchronize(s));
    return RKV_OK;
  }
  if (!cross && !subs) return RKV_OK;
  std::vector<uint32_t> xgsel((size_t)nrg * 16 * g, 0u);
  for (int rg = 0; rg < nrg; ++rg) {
    for (int c = 0; c < n; ++c) {                            // rotated channel of the group
      const int blk = c >> 7, kap = c & 127, q = kap >> 5;
      const int pos = inv[rg * n + c] - rg * n;              // reordered position within the group
      const int pass = subs ? (pos & 127) / qg : pos / qg;
      // per (wave, lane group, rotated block) 2 bits for each of a lane's 8 channels: the quantization
      // block within the group, or the sub-block within the head (4 bits each for a reorder across blocks
      // with groups of 64 / 32: any of the group's g * 128 / quant_group <= 16 blocks)
      const int gb = (cross && qg < 128) ? 4 : 2;
      const int w8 = (kap >> 3) & 3, wave = (w8 >> 1) | ((w8 & 1) << 1);     // 2 (wave & 1) + (wave >> 1) = w8
      xgsel[(((size_t)rg * 4 + wave) * 4 + q) * g + blk] |= (uint32_t)pass << (gb * (kap & 7));
    }
  }
  RKV_HIP_CHECK(hipMemcpyAsync(v.xgsel, xgsel.data(), xgsel.size() * 4, hipMemcpyHostToDevice, s));
  RKV_HIP_CHECK(hipStreamSynchronize(s));                    // the vectors go out of scope
  return RKV_OK;
}

RKV_EXPORT int rkv_query_sizes(const rkv_config* cfg, size_t* cache_bytes, size_t* scratch_bytes) {
  int rc = check_config(cfg, true);
  if (rc != RKV_OK) return rc;
  if (cache_bytes) *cache_bytes = plan(cfg).total;
  if (scratch_bytes) {
    size_t a = rkv_decode_scratch_bytes(cfg), b = rkv_calib_scratch_bytes(cfg);
    *scratch_bytes = a > b ? a : b;
  }
  return RKV_OK;
}

RKV_EXPORT int rkv_cache_create(const rkv_config* cfg, void* dev_mem, size_t bytes, void* stream, rkv_cache** out) {
  if (!out) return RKV_EINVAL;
  *out = nullptr;
  int rc = check_config(cfg, true);
  if (rc != RKV_OK) return rc;
  if (!dev_mem || ((uintptr_t)dev_mem & 255) != 0) return RKV_EINVAL;
  Offsets o = plan(cfg);
  if (bytes < o.total) return RKV_EINVAL;
  rkv_cache* c = new (std::nothrow) rkv_cache();
  if (!c) return RKV_EINVAL;
  c->cfg = *cfg;
  c->bytes = o.total;
  c->base = (char*)dev_mem;
  c->off_tables = o.tables;
  c->blocks_aligned = 1;
  c->decode_path = 0;
  c->ev_start = c->ev_stop = nullptr;
  c->cur_k = c->cur_v = nullptr;
  c->ragged = 0;
  c->hlens = new (std::nothrow) int32_t[cfg->batch]();
  c->stage = nullptr;
  c->stage_next = 0;
  for (int i = 0; i < RKV_STAGE_SLOTS; ++i) {
    c->stage_ev[i] = nullptr;
    c->stage_used[i] = 0;
  }
  if (!c->hlens) {
    free_host_side(c);
    return RKV_EINVAL;
  }
  if (hipHostMalloc((void**)&c->stage, (size_t)RKV_STAGE_SLOTS * cfg->batch * 4, hipHostMallocDefault) != hipSuccess) {
    c->stage = nullptr;
    free_host_side(c);
    return RKV_EHIP;
  }
  for (int i = 0; i < RKV_STAGE_SLOTS; ++i)
    if (hipEventCreateWithFlags(&c->stage_ev[i], hipEventDisableTiming) != hipSuccess) {
      c->stage_ev[i] = nullptr;
      free_host_side(c);
      return RKV_EHIP;
    }
  c->dev_lens = (int*)(c->base + o.lens);
  c->dev_nnew = (int*)(c->base + o.nnew);
  c->dev_cstart = (int*)(c->base + o.cstart);
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus < 1) {
      free_host_side(c);
      return RKV_EHIP;
    }
    c->n_cu = cus;
  }
  RkvView& v = c->v;
  v.kc = (uint32_t*)(c->base + o.kc);
  v.km = (uint32_t*)(c->base + o.km);
  v.vc = (uint32_t*)(c->base + o.vc);
  v.vm = (uint32_t*)(c->base + o.vm);
  v.hb = cfg->bits - 2;
  v.kh = v.hb ? (uint32_t*)(c->base + o.kh) : nullptr;
  v.vh = v.hb ? (uint32_t*)(c->base + o.vh) : nullptr;
  v.qg = cfg->quant_group;
  v.gm = cfg->rot_heads * (128 / cfg->quant_group);
  c->wide = (cfg->bits != 2 || cfg->quant_group != 128) ? 1 : 0;
  v.sink_k = (__half*)(c->base + o.sk);
  v.sink_v = (__half*)(c->base + o.sv);
  v.sink_pos = (int*)(c->base + o.spos);
  v.sink_cnt = (int*)(c->base + o.scnt);
  v.perm = (int*)(c->base + o.perm);
  v.pinv = (int*)(c->base + o.pinv);
  v.gid = (int*)(c->base + o.gid);
  v.rope = (float2*)(c->base + o.rope);
  v.hop = (uint32_t*)(c->base + o.hop);
  v.xgsel = (uint32_t*)(c->base + o.xgsel);
  v.xgid8 = (const uint2*)(c->base + o.xgid8);
  c->in_groups = 0;
  v.B = cfg->batch;
  v.Hq = cfg->n_q_heads;
  v.Hkv = cfg->n_kv_heads;
  v.g = cfg->rot_heads;
  v.n = cfg->rot_heads * RKV_D;
  v.E = cfg->n_kv_heads * RKV_D;
  v.NRG = cfg->n_kv_heads / cfg->rot_heads;
  v.NG = v.E / cfg->quant_group;
  v.Tpad = o.Tpad;
  v.max_sinks = cfg->max_sinks;
  v.len = 0;
  v.span = cfg->perm_span;
  v.rope_style = cfg->rope_style;
  v.v_rotate = cfg->v_rotate;
  v.keys_rotated = cfg->keys_rotated;
  v.meta8 = cfg->meta_format == 1;
  v.lens = nullptr;
  v.cstart = nullptr;
  v.nnew = nullptr;
  v.theta = cfg->rope_theta;
  {
    void* unused = nullptr;                                  // set-up: this device's address of the static work space
    rc = static_scratch_of_current_device(&unused);
    if (rc != RKV_OK) {
      free_host_side(c);
      return rc;
    }
  }
  rc = rkv_launch_init(c, true, (hipStream_t)stream);
  if (rc == RKV_OK && cfg->quant_group < 128) {            // the identity reorder's tables for groups of 64 / 32
    std::vector<int32_t> ident(v.E);
    for (int i = 0; i < v.E; ++i) ident[i] = i;
    rc = build_xtables(c, ident, 1, &c->in_groups, (hipStream_t)stream);
  }
  if (rc != RKV_OK) {
    free_host_side(c);
    return rc;
  }
  *out = c;
  return RKV_OK;
}

// Per-sequence counts that a call takes from host memory go to the device through a slot of the
// cache's own pinned ring, so that the caller's array is done with when the call returns whatever
// the runtime does with pageable memory.  A slot is reused only after the copy that last read it
// has completed (its event).
static int stage_counts(rkv_cache* c, const int32_t* host_vals, hipStream_t s) {
  const int slot = c->stage_next;
  c->stage_next = (slot + 1) % RKV_STAGE_SLOTS;
  if (c->stage_used[slot]) RKV_HIP_CHECK(hipEventSynchronize(c->stage_ev[slot]));
  int32_t* dst = c->stage + (size_t)slot * c->v.B;
  memcpy(dst, host_vals, (size_t)c->v.B * 4);
  RKV_HIP_CHECK(hipMemcpyAsync(c->dev_nnew, dst, (size_t)c->v.B * 4, hipMemcpyHostToDevice, s));
  RKV_HIP_CHECK(hipEventRecord(c->stage_ev[slot], s));
  c->stage_used[slot] = 1;
  return RKV_OK;
}

static void free_host_side(rkv_cache* c) {
  if (!c) return;
  delete[] c->hlens;
  if (c->stage) (void)hipHostFree(c->stage);
  for (int i = 0; i < RKV_STAGE_SLOTS; ++i)
    if (c->stage_ev[i]) (void)hipEventDestroy(c->stage_ev[i]);
  delete c;
}

RKV_EXPORT void rkv_cache_destroy(rkv_cache* cache) { free_host_side(cache); }

RKV_EXPORT int rkv_cache_reset(rkv_cache* cache, void* stream) {
  if (!cache) return RKV_EINVAL;
  cache->v.len = 0;
  cache->v.lens = nullptr;
  cache->v.cstart = nullptr;
  cache->ragged = 0;
  for (int b = 0; b < cache->v.B; ++b) cache->hlens[b] = 0;
  return rkv_launch_init(cache, false, (hipStream_t)stream);
}

RKV_EXPORT int rkv_cache_length(const rkv_cache* cache) { return cache ? cache->v.len : RKV_EINVAL; }

RKV_EXPORT int rkv_cache_lengths(const rkv_cache* cache, int32_t* host_lengths) {
  if (!cache || !host_lengths) return RKV_EINVAL;
  for (int b = 0; b < cache->v.B; ++b) host_lengths[b] = cache->hlens[b];
  return RKV_OK;
}

RKV_EXPORT int rkv_cache_truncate(rkv_cache* cache, const int32_t* host_new_lengths, void* stream) {
  if (!cache || !host_new_lengths) return RKV_EINVAL;
  const int B = cache->v.B;
  int lo = host_new_lengths[0], hi = lo;
  for (int b = 0; b < B; ++b) {
    const int nl = host_new_lengths[b];
    if (nl < 0 || nl > cache->hlens[b]) return RKV_EINVAL;
    lo = nl < lo ? nl : lo;
    hi = nl > hi ? nl : hi;
  }
  if (lo != hi && !cache->ragged && !rkv_append_mfma_supported(cache)) return RKV_EINVAL;   // would need per-sequence lengths
  hipStream_t s = (hipStream_t)stream;
  {
    const int rc = stage_counts(cache, host_new_lengths, s);
    if (rc != RKV_OK) return rc;
  }
  cache->v.nnew = cache->dev_nnew;
  const int rc = rkv_launch_lens(cache, -2, 0, s);
  cache->v.nnew = nullptr;
  if (rc != RKV_OK) return rc;
  for (int b = 0; b < B; ++b) cache->hlens[b] = host_new_lengths[b];
  cache->v.len = hi;
  if (lo != hi && !cache->ragged) {
    cache->ragged = 1;
    cache->v.lens = cache->dev_lens;
    cache->v.cstart = cache->dev_cstart;
  }
  return RKV_OK;
}

RKV_EXPORT int rkv_set_decode_path(rkv_cache* cache, int32_t path) {
  if (!cache || path < 0 || path > 3) return RKV_EINVAL;
  cache->decode_path = path;
  return RKV_OK;
}

RKV_EXPORT int rkv_decode_kernel_of(const rkv_cache* cache, int32_t n_queries) {
  if (!cache || n_queries < 0 || n_queries > RKV_MAX_QUERIES) return RKV_EINVAL;
  const int kind = rkv_mfma_supported(cache) ? rkv_mfma_variant(cache) : RKV_KERNEL_GENERAL;
  if (n_queries > 0) {
    // several query tokens per step: the plain matrix-core kernel; else the configuration's variant or the
    // general kernel, which serve up to 8 (query token, query head) pairs per KV head
    if (kind == RKV_KERNEL_MFMA && cache->decode_path != 1) return kind;
    // (the variants that take their scores from the scores kernel: up to 8 rows per KV head there too)
    if (kind != RKV_KERNEL_GENERAL && kind != RKV_KERNEL_MFMA && cache->decode_path != 1 && rkv_scores_multi_ok(cache, n_queries)) return kind;
    if (cache->decode_path >= 2) return RKV_EINVAL;
    return (cache->v.Hq / cache->v.Hkv) * n_queries <= 8 ? RKV_KERNEL_GENERAL : RKV_EINVAL;
  }
  if (cache->decode_path == 1) return RKV_KERNEL_GENERAL;
  if (cache->decode_path >= 2 && kind == RKV_KERNEL_GENERAL) return RKV_EINVAL;
  return kind;
}

RKV_EXPORT int rkv_append_kernel_of(const rkv_cache* cache) {
  if (!cache) return RKV_EINVAL;
  const RkvView& v = cache->v;
  if (rkv_append_mfma_supported(cache)) return rkv_append_mfma_variant(cache);
  if (cache->blocks_aligned && !cache->wide && (v.g == 2 || v.g == 4)) return RKV_KERNEL_SHUFFLE;
  return RKV_KERNEL_GENERAL;
}

RKV_EXPORT int rkv_set_profile_events(rkv_cache* cache, void* ev_start, void* ev_stop) {
  if (!cache || ((ev_start == nullptr) != (ev_stop == nullptr))) return RKV_EINVAL;
  cache->ev_start = (hipEvent_t)ev_start;
  cache->ev_stop = (hipEvent_t)ev_stop;
  return RKV_OK;
}

RKV_EXPORT int rkv_set_perm(rkv_cache* cache, const int32_t* dev_perm, void* stream) {
  if (!cache || !dev_perm) return RKV_EINVAL;
  if (cache->v.len != 0) return RKV_ESTATE;
  const int E = cache->v.E, span = cache->v.span;
  std::vector<int32_t> p(E), inv(E, -1), gid(E);
  hipStream_t s = (hipStream_t)stream;
  RKV_HIP_CHECK(hipMemcpyAsync(p.data(), dev_perm, (size_t)E * 4, hipMemcpyDeviceToHost, s));
  RKV_HIP_CHECK(hipStreamSynchronize(s));
  for (int i = 0; i < E; ++i) {
    int c = p[i];
    if (c < 0 || c >= E || inv[c] != -1) return RKV_EPERM;
    if (c / span != i / span) return RKV_EPERM;
    inv[c] = i;
  }
  int aligned = 1;
  for (int c = 0; c < E; ++c) {
    gid[c] = inv[c] / cache->cfg.quant_group;
    if (inv[c] / 128 != c / 128) aligned = 0;
  }
  RKV_HIP_CHECK(hipMemcpyAsync(cache->v.perm, p.data(), (size_t)E * 4, hipMemcpyHostToDevice, s));
  RKV_HIP_CHECK(hipMemcpyAsync(cache->v.pinv, inv.data(), (size_t)E * 4, hipMemcpyHostToDevice, s));
  RKV_HIP_CHECK(hipMemcpyAsync(cache->v.gid, gid.data(), (size_t)E * 4, hipMemcpyHostToDevice, s));
  int in_groups = 0;
  {
    const int rc = build_xtables(cache, inv, aligned, &in_groups, s);
    if (rc != RKV_OK) return rc;
  }
  RKV_HIP_CHECK(hipStreamSynchronize(s));
  cache->blocks_aligned = aligned;
  cache->in_groups = in_groups;
  return RKV_OK;
}

RKV_EXPORT int rkv_calibrate_perm(const rkv_config* cfg, const void* dev_k_cal, int32_t n_tok, int32_t* dev_perm_out,
                                  void* dev_scratch, void* stream) {
  int rc = check_config(cfg, false);
  if (rc != RKV_OK) return rc;
  if (!dev_k_cal || !dev_perm_out || !dev_scratch || n_tok < 1) return RKV_EINVAL;
  return rkv_launch_calibrate(cfg, (const __half*)dev_k_cal, n_tok, dev_perm_out, dev_scratch, (hipStream_t)stream);
}

RKV_EXPORT int rkv_fold_rotation(const rkv_config* cfg, const float* dev_w, int32_t rows, const int32_t* dev_perm,
                                 float* dev_w_out, void* stream) {
  if (!cfg || !dev_w || !dev_w_out || rows < 1) return RKV_EINVAL;
  if (cfg->head_dim != RKV_D || cfg->n_kv_heads < 1 || cfg->n_kv_heads > 128) return RKV_EINVAL;
  if (cfg->rot_heads != 1 && cfg->rot_heads != 2 && cfg->rot_heads != 4 && cfg->rot_heads != 8) return RKV_EINVAL;
  if (cfg->n_kv_heads % cfg->rot_heads != 0) return RKV_EINVAL;
  return rkv_launch_fold_rotation(cfg, dev_w, rows, dev_perm, dev_w_out, (hipStream_t)stream);
}

RKV_EXPORT int rkv_select_sinks(const void* dev_x, int32_t batch, int32_t n_tok, int32_t width, int32_t k, int32_t* dev_idx_out,
                                uint8_t* dev_mask_out, void* dev_scratch, void* stream) {
  if (!dev_x || !dev_idx_out || !dev_scratch) return RKV_EINVAL;
  if (batch < 1 || n_tok < 1 || width < 8 || (width & 7) || k < 1 || k > 64 || k > n_tok) return RKV_EINVAL;
  return rkv_launch_select_sinks((const __half*)dev_x, batch, n_tok, width, k, dev_idx_out, dev_mask_out, (float*)dev_scratch,
                                 (hipStream_t)stream);
}

RKV_EXPORT int rkv_quantize_append(rkv_cache* cache, const void* dev_k, const void* dev_v, int32_t n_new,
                                   const uint8_t* dev_sink_mask, void* stream) {
  if (!cache || n_new < 0) return RKV_EINVAL;
  if (n_new == 0) return RKV_OK;                      // nothing to read: the pointers may be null
  if (!dev_k || !dev_v) return RKV_EINVAL;
  if ((int64_t)cache->v.len + n_new > cache->cfg.max_tokens) return RKV_ECAPACITY;   // v.len: the longest sequence
  if (cache->ragged && !rkv_append_mfma_supported(cache)) return RKV_EINVAL;
  int rc = rkv_launch_append(cache, (const __half*)dev_k, (const __half*)dev_v, n_new, dev_sink_mask, (hipStream_t)stream);
  if (rc == RKV_OK && cache->ragged) rc = rkv_launch_lens(cache, -1, n_new, (hipStream_t)stream);
  if (rc == RKV_OK) {
    cache->v.len += n_new;
    for (int b = 0; b < cache->v.B; ++b) cache->hlens[b] += n_new;
  }
  return rc;
}

RKV_EXPORT int rkv_quantize_append_ragged(rkv_cache* cache, const void* dev_k, const void* dev_v, int32_t n_new_max,
                                          const int32_t* host_n_new, const uint8_t* dev_sink_mask, void* stream) {
  if (!cache || !host_n_new || n_new_max < 0) return RKV_EINVAL;
  const int B = cache->v.B;
  int hi = 0, lo = n_new_max, new_max = 0, max_slabs = 0;
  for (int b = 0; b < B; ++b) {
    const int nb = host_n_new[b], lb = cache->hlens[b];
    if (nb < 0 || nb > n_new_max) return RKV_EINVAL;
    if ((int64_t)lb + nb > cache->cfg.max_tokens) return RKV_ECAPACITY;
    hi = nb > hi ? nb : hi;
    lo = nb < lo ? nb : lo;
    new_max = lb + nb > new_max ? lb + nb : new_max;
    if (nb > 0) {
      const int slabs = ((lb + nb - 1) >> 5) - (lb >> 5) + 1;
      max_slabs = slabs > max_slabs ? slabs : max_slabs;
    }
  }
  if (hi == 0) return RKV_OK;
  if (!dev_k || !dev_v) return RKV_EINVAL;
  // every sequence appends the same number of rows, packed as the uniform call expects them
  if (lo == hi && hi == n_new_max) return rkv_quantize_append(cache, dev_k, dev_v, n_new_max, dev_sink_mask, stream);
  if (!rkv_append_mfma_supported(cache)) return RKV_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  int rc = RKV_OK;
  if (!cache->ragged) {
    rc = rkv_launch_lens(cache, cache->v.len, 0, s);          // device lengths start from the common length
    if (rc != RKV_OK) return rc;
    cache->ragged = 1;
    cache->v.lens = cache->dev_lens;
    cache->v.cstart = cache->dev_cstart;
  }
  rc = stage_counts(cache, host_n_new, s);
  if (rc != RKV_OK) return rc;
  cache->v.nnew = cache->dev_nnew;
  if (dev_sink_mask && cache->v.max_sinks > 0)
    rc = rkv_launch_sinks(cache, (const __half*)dev_k, (const __half*)dev_v, dev_sink_mask, n_new_max, s);
  if (rc == RKV_OK) rc = rkv_launch_append_mfma(cache, (const __half*)dev_k, (const __half*)dev_v, n_new_max, max_slabs, s);
  if (rc == RKV_OK) rc = rkv_launch_lens(cache, -1, 0, s);      // lengths += the staged counts
  cache->v.nnew = nullptr;
  if (rc == RKV_OK) {
    for (int b = 0; b < B; ++b) cache->hlens[b] += host_n_new[b];
    cache->v.len = new_max;
  }
  return rc;
}

RKV_EXPORT int rkv_decode_attention_with_current(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos,
                                                 const void* dev_k_cur, const void* dev_v_cur, float* dev_out,
                                                 float* dev_lse, void* dev_scratch, void* stream) {
  if (!cache || !dev_k_cur || !dev_v_cur) return RKV_EINVAL;
  cache->cur_k = (const __half*)dev_k_cur;
  cache->cur_v = (const __half*)dev_v_cur;
  const int rc = rkv_decode_attention(cache, dev_q, dev_q_pos, dev_out, dev_lse, dev_scratch, stream);
  cache->cur_k = cache->cur_v = nullptr;
  return rc;
}

RKV_EXPORT int rkv_decode_attention(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos, float* dev_out,
                                    float* dev_lse, void* dev_scratch, void* stream) {
  if (!cache || !dev_q || !dev_out || !dev_scratch) return RKV_EINVAL;
  if (cache->v.len < 1 && !cache->cur_k) return RKV_ESTATE;
  if (cache->ragged && !cache->cur_k)
    for (int b = 0; b < cache->v.B; ++b)
      if (cache->hlens[b] < 1) return RKV_ESTATE;           // a sequence with nothing to attend
  bool fast = rkv_mfma_supported(cache);
  if (cache->decode_path >= 2 && !fast) return RKV_EINVAL;
  if (cache->decode_path == 1) fast = false;
  if (fast)
    return rkv_launch_decode_mfma(cache, (const __half*)dev_q, dev_q_pos, 0, dev_out, dev_lse, dev_scratch, false,
                                  (hipStream_t)stream);
  return rkv_launch_decode_general(cache, (const __half*)dev_q, dev_q_pos, 0, dev_out, dev_lse, dev_scratch, (hipStream_t)stream);
}

RKV_EXPORT int rkv_decode_attention_static(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos, float* dev_out,
                                           float* dev_lse, void* stream) {
  if (!cache) return RKV_EINVAL;
  // what this call's kernels write: the prepared queries, then one partial per (sequence, query
  // head, chunk of the cache's current length) - chunks of the kernel that will run
  const bool fast = rkv_mfma_supported(cache) && cache->decode_path != 1;
  const size_t chunk = fast ? RKV_MFMA_CHUNK : RKV_GEN_CHUNK;
  const size_t nch = ((size_t)cache->v.len + chunk - 1) / chunk;
  size_t need = rkv_query_scratch_bytes(cache->v.B, cache->v.Hq) +
                (size_t)cache->v.B * cache->v.Hq * nch * RKV_PART_STRIDE * 4 + 256;
  // (a reorder over the whole row: the scores buffer sits behind the partial results of the cache's capacity)
  if (fast && rkv_scores_path(cache))
    need = rkv_query_scratch_bytes(cache->v.B, cache->v.Hq) + rkv_partial_bytes(cache->v.B, cache->v.Hq, cache->v.Tpad) +
           rkv_row_scores_bytes(cache->v.B, cache->v.Hq, cache->cfg.max_tokens) + 256;
  if (need > RKV_STATIC_SCRATCH_BYTES) return RKV_ESCRATCH;
  void* ptr = nullptr;
  const int rc = static_scratch_of_current_device(&ptr);
  if (rc != RKV_OK) return rc;
  return rkv_decode_attention(cache, dev_q, dev_q_pos, dev_out, dev_lse, ptr, stream);
}

RKV_EXPORT int rkv_decode_step(rkv_cache* cache, const void* dev_k, const void* dev_v, const void* dev_q, const int32_t* dev_q_pos,
                               float* dev_out, float* dev_lse, void* dev_scratch, void* stream) {
  if (!cache || !dev_k || !dev_v || !dev_q || !dev_out || !dev_scratch) return RKV_EINVAL;
  if ((int64_t)cache->v.len + 1 > cache->cfg.max_tokens) return RKV_ECAPACITY;
  const bool fused = rkv_append_mfma_supported(cache) && rkv_append_mfma_variant(cache) != RKV_KERNEL_MFMA_ROW &&
                     rkv_mfma_supported(cache) && cache->decode_path != 1;
  if (!fused) {   // the same two calls, one after the other
    const int rc = rkv_quantize_append(cache, dev_k, dev_v, 1, nullptr, stream);
    return rc != RKV_OK ? rc : rkv_decode_attention(cache, dev_q, dev_q_pos, dev_out, dev_lse, dev_scratch, stream);
  }
  hipStream_t s = (hipStream_t)stream;
  // (the sub-group variant of the decode kernel takes one query head per workgroup)
  const int share = rkv_mfma_variant(cache) == RKV_KERNEL_MFMA_SUB ? 1 : rkv_mfma_share(cache->v.Hq / cache->v.Hkv);
  int rc = rkv_launch_step_mfma(cache, (const __half*)dev_k, (const __half*)dev_v, (const __half*)dev_q, dev_q_pos,
                                (float*)dev_scratch, share, s);
  if (rc == RKV_OK && cache->ragged) rc = rkv_launch_lens(cache, -1, 1, s);
  if (rc != RKV_OK) return rc;
  cache->v.len += 1;
  for (int b = 0; b < cache->v.B; ++b) cache->hlens[b] += 1;
  return rkv_launch_decode_mfma(cache, (const __half*)dev_q, dev_q_pos, 0, dev_out, dev_lse, dev_scratch, true, s);
}

RKV_EXPORT int rkv_decode_attention_multi(rkv_cache* cache, const void* dev_q, const int32_t* dev_q_pos, int32_t n_queries,
                                          float* dev_out, float* dev_lse, void* dev_scratch, void* stream) {
  if (!cache || !dev_q || !dev_q_pos || !dev_out || !dev_scratch) return RKV_EINVAL;
  if (n_queries < 1 || n_queries > RKV_MAX_QUERIES) return RKV_EINVAL;
  if (cache->v.len < 1) return RKV_ESTATE;
  if (cache->ragged)
    for (int b = 0; b < cache->v.B; ++b)
      if (cache->hlens[b] < 1) return RKV_ESTATE;
  const int kind = rkv_decode_kernel_of(cache, n_queries);
  if (kind < 0) return kind;
  if (kind == RKV_KERNEL_GENERAL)
    return rkv_launch_decode_general(cache, (const __half*)dev_q, dev_q_pos, n_queries, dev_out, dev_lse, dev_scratch,
                                     (hipStream_t)stream);
  return rkv_launch_decode_mfma(cache, (const __half*)dev_q, dev_q_pos, n_queries, dev_out, dev_lse, dev_scratch, false,
                                (hipStream_t)stream);
}

RKV_EXPORT int rkv_dequantize(rkv_cache* cache, float* dev_k_hat, float* dev_v_hat, void* stream) {
  if (!cache) return RKV_EINVAL;
  if (cache->v.len < 1) return RKV_ESTATE;
  return rkv_launch_dequant(cache, dev_k_hat, dev_v_hat, (hipStream_t)stream);
}

RKV_EXPORT int rkv_export_codes(rkv_cache* cache, uint8_t* dev_k_codes, float* dev_k_scale, float* dev_k_zero,
                                uint8_t* dev_v_codes, float* dev_v_scale, float* dev_v_zero, void* stream) {
  if (!cache) return RKV_EINVAL;
  if (cache->v.len < 1) return RKV_ESTATE;
  return rkv_launch_export(cache, dev_k_codes, dev_k_scale, dev_k_zero, dev_v_codes, dev_v_scale, dev_v_zero,
                           (hipStream_t)stream);
}

RKV_EXPORT int rkv_import_codes(rkv_cache* cache, int32_t n_tokens, const uint8_t* dev_k_codes, const float* dev_k_scale,
                                const float* dev_k_zero, const uint8_t* dev_v_codes, const float* dev_v_scale,
                                const float* dev_v_zero, void* stream) {
  if (!cache || !dev_k_codes || !dev_k_scale || !dev_k_zero || !dev_v_codes || !dev_v_scale || !dev_v_zero) return RKV_EINVAL;
  if (n_tokens < 1) return RKV_EINVAL;
  if (n_tokens > cache->cfg.max_tokens) return RKV_ECAPACITY;
  if (cache->ragged) return RKV_ESTATE;                       // the import gives every sequence the same length: reset first
  int rc = rkv_launch_import(cache, n_tokens, dev_k_codes, dev_k_scale, dev_k_zero, dev_v_codes, dev_v_scale, dev_v_zero,
                             (hipStream_t)stream);
  if (rc == RKV_OK) {
    cache->v.len = n_tokens;
    for (int b = 0; b < cache->v.B; ++b) cache->hlens[b] = n_tokens;
  }
  return rc;
}

RKV_EXPORT int rkv_export_sinks(rkv_cache* cache, int32_t* dev_count, int32_t* dev_pos, void* dev_k, void* dev_v,
                                void* stream) {
  if (!cache) return RKV_EINVAL;
  const RkvView& v = cache->v;
  hipStream_t s = (hipStream_t)stream;
  const size_t S = v.max_sinks;
  if (dev_count) RKV_HIP_CHECK(hipMemcpyAsync(dev_count, v.sink_cnt, (size_t)v.B * 4, hipMemcpyDeviceToDevice, s));
  if (S == 0) return RKV_OK;
  if (dev_pos) RKV_HIP_CHECK(hipMemcpyAsync(dev_pos, v.sink_pos, (size_t)v.B * S * 4, hipMemcpyDeviceToDevice, s));
  if (dev_k) RKV_HIP_CHECK(hipMemcpyAsync(dev_k, v.sink_k, (size_t)v.B * S * v.E * 2, hipMemcpyDeviceToDevice, s));
  if (dev_v) RKV_HIP_CHECK(hipMemcpyAsync(dev_v, v.sink_v, (size_t)v.B * S * v.E * 2, hipMemcpyDeviceToDevice, s));
  return RKV_OK;
}

RKV_EXPORT int rkv_layout_locate(const rkv_config* cfg, int32_t is_v, int32_t b, int32_t t, int32_t c, size_t* word_index,
                                 int32_t* bit_shift, size_t* n_words) {
  int rc = check_config(cfg, true);
  if (rc != RKV_OK) return rc;
  if (!word_index || !bit_shift) return RKV_EINVAL;
  Offsets o = plan(cfg);
  RkvView v{};
  v.g = cfg->rot_heads;
  v.n = cfg->rot_heads * RKV_D;
  v.E = cfg->n_kv_heads * RKV_D;
  v.NRG = cfg->n_kv_heads / cfg->rot_heads;
  v.Tpad = o.Tpad;
  if (b < 0 || b >= cfg->batch || t < 0 || t >= o.Tpad || c < 0 || c >= v.E) return RKV_EINVAL;
  int sh = 0;
  const int rg = c / v.n, cc = c % v.n;
  *word_index = is_v ? rkv_v_dword(v, b, rg, t, cc, sh) : rkv_k_dword(v, b, rg, t, cc, sh);
  *bit_shift = sh;
  if (n_words) *n_words = (size_t)cfg->batch * o.Tpad * v.E / 16;
  return RKV_OK;
}

RKV_EXPORT const char* rkv_strerror(int code) {
  switch (code) {
    case RKV_OK: return "ok";
    case RKV_EINVAL: return "invalid argument or unsupported configuration";
    case RKV_ECAPACITY: return "cache capacity exceeded";
    case RKV_EPERM: return "reorder indices are not a permutation closed under perm_span";
    case RKV_EHIP: return "HIP runtime error";
    case RKV_ESTATE: return "call not valid in the cache's current state";
    case RKV_ESCRATCH: return "the library's built-in work space is too small for this cache (pass a work space of your own: rkv_decode_attention)";
    default: return "unknown error";
  }
}

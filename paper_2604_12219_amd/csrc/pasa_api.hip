// C ABI of the PASA forward (see include/pasa.h): argument validation, workspace carving, launches.
// Nothing here allocates, frees or synchronises.
#include "pasa.h"
#include "pasa_kernels.hpp"

#include <math.h>

#include <atomic>
#include <mutex>

// Scratch of pasa_sparse_attn_fwd_static, the entry point that allocates nothing: the attention workspace
// (statistics tiles, group matrices, unit sums) lives in this array instead of a caller's buffer.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; the device address it yields is kept per device and is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[PASA_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxChunks = 8192;   // chunks of 32 key blocks per head (262,144 key blocks)
constexpr int kMaxGroups = 65535;  // first-order groups per head
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

int check_shape(const pasa_shape_t* s) {
  if (!s) return PASA_EINVAL;
  if (s->B < 1 || s->H < 1 || s->n < 1) return PASA_EINVAL;
  if ((int64_t)s->B * s->H > 65535) return PASA_EUNSUPPORTED;
  if (s->d != 64 && s->d != 128) return PASA_EUNSUPPORTED;
  if (s->block != 64 && s->block != 128) return PASA_EUNSUPPORTED;
  if (!(s->scale >= 0.f) || isinf(s->scale)) return PASA_EINVAL;
  if (s->stride_n < s->d || s->stride_h < 1 || s->stride_b < 1) return PASA_EINVAL;
  if ((s->stride_n % 8) || (s->stride_h % 8) || (s->stride_b % 8)) return PASA_EALIGN;
  if ((int64_t)s->n * s->stride_n * 2 >= ((int64_t)1 << 32)) return PASA_EUNSUPPORTED;  // 32-bit byte offsets inside a head
  return PASA_OK;
}

int num_blocks(const pasa_shape_t* s) { return (s->n + s->block - 1) / s->block; }

int check_group(int group, int nb) {
  if (group < 0) return PASA_EINVAL;
  if (group == 0 || group >= nb) return PASA_OK;
  if (group % 32 == 0) return PASA_OK;
  if (group < 32 && (group & (group - 1)) == 0) return PASA_OK;
  return PASA_EUNSUPPORTED;
}

float effective_scale(const pasa_shape_t* s) { return s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->d); }

struct AttnWorkspace {
  size_t st, hg, partial, kbar, part_o, part_ml, queue, bitmap, total;
  int n_groups, unit, n_units, n_chunks, n_slices;
};

// Number of key-range slices of the sparse kernel.  K and V of one head should fit the 4 MB L2 of an
// XCD slice by slice; there are 8 XCDs, so slices come in multiples of 8.
int choose_slices(const pasa_shape_t* s) {
  if (s->kv_slices >= 1) return s->kv_slices;
  // kv_slices == 0: no slicing.  Slicing removes most of the fabric traffic, but the extra partial
  // results and the merge pass cost more than that buys while the kernel is not yet limited by the
  // fabric; callers can switch it on per shape.
  return 1;
}

int check_slices(const pasa_shape_t* s) {
  if (s->kv_slices < 0) return PASA_EINVAL;
  if (s->kv_slices <= 1) return PASA_OK;
  if (s->kv_slices % 8 != 0 || s->kv_slices > (num_blocks(s) + 31) / 32) return PASA_EUNSUPPORTED;
  return PASA_OK;
}

AttnWorkspace carve_attn(const pasa_shape_t* s) {
  AttnWorkspace w{};
  const int nb = num_blocks(s);
  const size_t bh = (size_t)s->B * s->H;
  w.n_chunks = (nb + 31) / 32;
  w.n_slices = choose_slices(s);
  size_t off = 0;
  if (w.n_slices > 1) {
    w.part_o = off; off = align_up(off + bh * w.n_slices * s->n * s->d * 4);
    w.part_ml = off; off = align_up(off + bh * w.n_slices * s->n * 2 * 4);
    w.queue = off; off = align_up(off + 8 * 4);
  }
  // room for a selection bitmap built from index lists (callers that pass no bitmap of their own)
  w.bitmap = off; off = align_up(off + bh * nb * (size_t)w.n_chunks * 4);
  if (s->group > 0) {
    const int group = s->group >= nb ? nb : s->group;
    w.n_groups = (nb + group - 1) / group;
    // Blocks summed by one workgroup of the statistics kernel: a whole group, at most 32 blocks -- fewer (a power of
    // two that divides the group) while that leaves the device short of workgroups, at the price of more unit sums.
    w.unit = group < 32 ? group : 32;
    while (w.unit > 8 && (int64_t)bh * ((nb + w.unit - 1) / w.unit) < 1024) w.unit /= 2;
    w.n_units = (nb + w.unit - 1) / w.unit;
    w.st = off; off = align_up(off + bh * w.n_chunks * 64 * s->d * 2);
    w.hg = off; off = align_up(off + bh * w.n_groups * s->d * s->d * 2);
    w.partial = off; off = align_up(off + bh * w.n_units * s->d * s->d * 4);
    w.kbar = off; off = align_up(off + bh * nb * s->d * 4);  // block-mean keys as split bf16 pairs, for pasa_block_score_with_stats
  }
  w.total = off;
  return w;
}

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until looked up
std::mutex g_scratch_mutex;

// Device address of the static scratch array on the current device (looked up once per device).
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PASA_EHIP;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ptr = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!ptr) {
      if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return PASA_EHIP;
      }
      g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
  }
  *out = ptr;
  return PASA_OK;
}

}  // namespace

extern "C" {

const char* pasa_strerror(int status) {
  switch (status) {
    case PASA_OK: return "ok";
    case PASA_EINVAL: return "invalid argument";
    case PASA_EUNSUPPORTED: return "unsupported head dimension, block size, group size or problem size";
    case PASA_EWORKSPACE: return "workspace too small";
    case PASA_EALIGN: return "pointer or stride not sufficiently aligned";
    case PASA_EHIP: return "HIP launch failure";
    case PASA_ESCRATCH: return "problem needs more scratch than the static buffer of the no-allocation entry point holds";
    default: return "unknown status";
  }
}

int32_t pasa_topk_count(int32_t n_blocks, double keep_ratio) {
  if (n_blocks < 1 || !(keep_ratio > 0.0) || keep_ratio > 1.0) return PASA_EINVAL;
  double x = floor(keep_ratio * (double)n_blocks + 0.5);
  if (x < 1.0) x = 1.0;
  if (x > (double)n_blocks) x = (double)n_blocks;
  return (int32_t)x;
}

int32_t pasa_num_blocks(const pasa_shape_t* shape) {
  const int rc = check_shape(shape);
  return rc != PASA_OK ? rc : num_blocks(shape);
}

int32_t pasa_mask_words(int32_t n_blocks) { return n_blocks < 1 ? PASA_EINVAL : (n_blocks + 31) / 32; }

size_t pasa_score_workspace_bytes(const pasa_shape_t* shape) {
  if (check_shape(shape) != PASA_OK) return 0;
  const size_t one = align_up((size_t)shape->B * shape->H * num_blocks(shape) * shape->d * 4);
  return 2 * one;
}

size_t pasa_attn_workspace_bytes(const pasa_shape_t* shape) {
  if (check_shape(shape) != PASA_OK) return 0;
  if (check_group(shape->group, num_blocks(shape)) != PASA_OK) return 0;
  if (check_slices(shape) != PASA_OK) return 0;
  const size_t t = carve_attn(shape).total;
  return t ? t : kAlign;  // never zero for a valid shape, so that 0 always means "bad shape"
}

static int block_score_impl(const void* q, const void* k, const pasa_shape_t* shape, const float* key_bias, float* scores,
                            void* ws, size_t ws_bytes, const void* kbar_split, void* stream) {
  const int rc = check_shape(shape);
  if (rc != PASA_OK) return rc;
  if (!q || (!k && !kbar_split) || !scores || !ws) return PASA_EINVAL;
  if (!aligned16(q) || (k && !aligned16(k)) || !aligned16(scores) || !aligned16(ws)) return PASA_EALIGN;
  if (ws_bytes < pasa_score_workspace_bytes(shape)) return PASA_EWORKSPACE;
  ScoreParams p{};
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k);
  p.stride_b = shape->stride_b; p.stride_h = shape->stride_h; p.stride_n = shape->stride_n;
  p.bh = shape->B * shape->H; p.H = shape->H; p.n = shape->n; p.nb = num_blocks(shape);
  p.block = shape->block; p.d = shape->d;
  p.scale = effective_scale(shape);
  p.key_bias = key_bias;
  p.qbar = static_cast<float*>(ws);
  p.pool_k = kbar_split ? 0 : 1;
  p.kbar = kbar_split ? const_cast<float*>(static_cast<const float*>(kbar_split))
                      : reinterpret_cast<float*>(static_cast<char*>(ws) + pasa_score_workspace_bytes(shape) / 2);
  p.scores = scores;
  return pasa_launch_block_score(p, static_cast<hipStream_t>(stream)) == hipSuccess ? PASA_OK : PASA_EHIP;
}

int pasa_block_score(const void* q, const void* k, const pasa_shape_t* shape, const float* key_bias, float* scores,
                     void* ws, size_t ws_bytes, void* stream) {
  return block_score_impl(q, k, shape, key_bias, scores, ws, ws_bytes, nullptr, stream);
}

static int route_impl(const float* scores, int32_t BH, int32_t n_blocks, int32_t k_sel, uint64_t seed, float noise_amp,
                      int gumbel, int32_t* idx, uint32_t* mask, void* stream) {
  if (!scores || !idx || BH < 1 || n_blocks < 1) return PASA_EINVAL;
  if (k_sel < 1 || k_sel > n_blocks) return PASA_EINVAL;
  if (!(noise_amp >= 0.f) || isinf(noise_amp)) return PASA_EINVAL;
  if (n_blocks > kRouteMaxBlocks) return PASA_EUNSUPPORTED;
  RouteParams p{};
  p.scores = scores;
  p.bh = BH; p.nb = n_blocks; p.k_sel = k_sel; p.mask_words = (n_blocks + 31) / 32;
  p.seed_lo = (uint32_t)(seed & 0xffffffffu); p.seed_hi = (uint32_t)(seed >> 32);
  p.amp = noise_amp;
  p.gumbel = gumbel;
  p.idx = idx; p.mask = mask;
  return pasa_launch_route(p, static_cast<hipStream_t>(stream)) == hipSuccess ? PASA_OK : PASA_EHIP;
}

int pasa_route(const float* scores, int32_t BH, int32_t n_blocks, int32_t k_sel, uint64_t seed, float noise_amp,
               int32_t* idx, uint32_t* mask, void* stream) {
  return route_impl(scores, BH, n_blocks, k_sel, seed, noise_amp, 0, idx, mask, stream);
}

int pasa_route_gumbel(const float* scores, int32_t BH, int32_t n_blocks, int32_t k_sel, uint64_t seed, float temperature,
                      int32_t* idx, uint32_t* mask, void* stream) {
  return route_impl(scores, BH, n_blocks, k_sel, seed, temperature, 1, idx, mask, stream);
}

// validation shared by the statistics and attention entry points; fills `s` (group normalised)
static int check_attn_args(const pasa_shape_t* shape, bool sparse, const void* ws, size_t ws_bytes, pasa_shape_t* s) {
  const int rc = check_shape(shape);
  if (rc != PASA_OK) return rc;
  *s = *shape;
  if (!sparse) { s->group = 0; s->kv_slices = 1; }
  const int rg = check_group(s->group, num_blocks(s));
  if (rg != PASA_OK) return rg;
  const int rs = check_slices(s);
  if (rs != PASA_OK) return rs;
  {  // one workgroup per 128 query rows, counted in 32 bits (also the work items of key-range slicing)
    const int64_t q_tiles = ((int64_t)s->n + 127) / 128;
    const int64_t wgs = (int64_t)s->B * s->H * 8 * ((q_tiles + 7) / 8) * (s->kv_slices > 1 ? s->kv_slices / 8 : 1);
    if (wgs >= ((int64_t)1 << 31)) return PASA_EUNSUPPORTED;
  }
  if (sparse) {  // field widths of the approximation pass's tile descriptors (13 bits of chunk, 16 bits of group)
    const int nb = num_blocks(s);
    const int group = s->group >= nb ? nb : s->group;
    if ((nb + 31) / 32 > kMaxChunks) return PASA_EUNSUPPORTED;
    if (group > 0 && (nb + group - 1) / group > kMaxGroups) return PASA_EUNSUPPORTED;
  }
  if (!ws) return PASA_EINVAL;
  if (!aligned16(ws)) return PASA_EALIGN;
  if (ws_bytes < pasa_attn_workspace_bytes(s)) return PASA_EWORKSPACE;
  return PASA_OK;
}

int pasa_block_score_with_stats(const void* q, const pasa_shape_t* shape, const float* key_bias, float* scores, void* ws,
                                size_t ws_bytes, const void* stats_ws, size_t stats_ws_bytes, void* stream) {
  pasa_shape_t s;
  const int rc = check_attn_args(shape, true, stats_ws, stats_ws_bytes, &s);
  if (rc != PASA_OK) return rc;
  if (s.group == 0) return PASA_EUNSUPPORTED;  // pasa_kv_stats leaves nothing when the approximation is off
  const AttnWorkspace w = carve_attn(&s);
  return block_score_impl(q, nullptr, shape, key_bias, scores, ws, ws_bytes, static_cast<const char*>(stats_ws) + w.kbar, stream);
}

int pasa_check_selection(const int32_t* idx, const uint32_t* mask, int32_t BH, int32_t n_blocks, int32_t k_sel, int32_t* n_bad,
                         void* stream) {
  if ((!idx && !mask) || !n_bad || BH < 1 || n_blocks < 1 || k_sel < 1 || k_sel > n_blocks) return PASA_EINVAL;
  if ((idx && !aligned4(idx)) || (mask && !aligned4(mask)) || !aligned4(n_bad)) return PASA_EALIGN;
  return pasa_launch_check_selection(idx, mask, (int64_t)BH * n_blocks, n_blocks, k_sel, n_bad, static_cast<hipStream_t>(stream)) ==
                 hipSuccess ? PASA_OK : PASA_EHIP;
}

int pasa_kv_stats(const void* k, const void* v, const pasa_shape_t* shape, void* ws, size_t ws_bytes, void* stream) {
  pasa_shape_t s;
  const int rc = check_attn_args(shape, true, ws, ws_bytes, &s);
  if (rc != PASA_OK) return rc;
  if (!k || !v) return PASA_EINVAL;
  if (!aligned16(k) || !aligned16(v)) return PASA_EALIGN;
  if (s.group == 0) return PASA_OK;
  const int nb = num_blocks(&s);
  const AttnWorkspace w = carve_attn(&s);
  char* base = static_cast<char*>(ws);
  StatsParams t{};
  t.k = static_cast<const uint16_t*>(k); t.v = static_cast<const uint16_t*>(v);
  t.stride_b = s.stride_b; t.stride_h = s.stride_h; t.stride_n = s.stride_n;
  t.bh = s.B * s.H; t.H = s.H; t.n = s.n; t.nb = nb; t.block = s.block; t.tail = s.n - (nb - 1) * s.block; t.d = s.d;
  t.group = s.group >= nb ? nb : s.group; t.n_groups = w.n_groups; t.unit = w.unit; t.n_units = w.n_units;
  t.scale = effective_scale(&s);
  t.n_chunks = w.n_chunks;
  t.st = reinterpret_cast<uint16_t*>(base + w.st);
  t.hg = reinterpret_cast<uint16_t*>(base + w.hg);
  t.partial = reinterpret_cast<float*>(base + w.partial);
  t.kbar_split = reinterpret_cast<uint16_t*>(base + w.kbar);
  return pasa_launch_kv_stats(t, static_cast<hipStream_t>(stream)) == hipSuccess ? PASA_OK : PASA_EHIP;
}

int pasa_key_prior(const void* k, const void* v, const pasa_shape_t* shape, float eps, float* beta, void* ws,
                   size_t ws_bytes, void* stream) {
  pasa_shape_t s;
  const int rc = check_attn_args(shape, true, ws, ws_bytes, &s);
  if (rc != PASA_OK) return rc;
  if (!k || !v || !beta || !(eps >= 0.f)) return PASA_EINVAL;
  if (!aligned16(k) || !aligned16(v)) return PASA_EALIGN;
  if (s.group == 0) return PASA_EUNSUPPORTED;
  const int nb = num_blocks(&s);
  const AttnWorkspace w = carve_attn(&s);
  char* base = static_cast<char*>(ws);
  StatsParams t{};
  t.k = static_cast<const uint16_t*>(k); t.v = static_cast<const uint16_t*>(v);
  t.stride_b = s.stride_b; t.stride_h = s.stride_h; t.stride_n = s.stride_n;
  t.bh = s.B * s.H; t.H = s.H; t.n = s.n; t.nb = nb; t.block = s.block; t.tail = s.n - (nb - 1) * s.block; t.d = s.d;
  t.group = s.group >= nb ? nb : s.group; t.n_groups = w.n_groups; t.unit = w.unit; t.n_units = w.n_units;
  t.scale = effective_scale(&s);
  t.n_chunks = w.n_chunks;
  t.partial = reinterpret_cast<float*>(base + w.partial);
  return pasa_launch_key_prior(t, eps, beta, static_cast<hipStream_t>(stream)) == hipSuccess ? PASA_OK : PASA_EHIP;
}

static int attn_common(const void* q, const void* k, const void* v, const pasa_shape_t* shape, const int32_t* idx,
                       const uint32_t* mask, int32_t k_sel, void* out, float* lse, void* ws, size_t ws_bytes,
                       void* stream, bool sparse, bool with_stats) {
  pasa_shape_t s;
  const int rc = check_attn_args(shape, sparse, ws, ws_bytes, &s);
  if (rc != PASA_OK) return rc;
  const int nb = num_blocks(&s);
  if (!q || !k || !v || !out) return PASA_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return PASA_EALIGN;
  if (out == q || out == k || out == v) return PASA_EINVAL;
  if (sparse) {
    if ((!idx && !mask) || k_sel < 1 || k_sel > nb) return PASA_EINVAL;
    if ((idx && !aligned4(idx)) || (mask && !aligned4(mask))) return PASA_EALIGN;
  }
  if (sparse && with_stats) {
    const int rs = pasa_kv_stats(k, v, &s, ws, ws_bytes, stream);
    if (rs != PASA_OK) return rs;
  }
  const AttnWorkspace w = carve_attn(&s);
  char* base = static_cast<char*>(ws);
  AttnParams a{};
  a.q = static_cast<const uint16_t*>(q); a.k = static_cast<const uint16_t*>(k); a.v = static_cast<const uint16_t*>(v);
  a.o = static_cast<uint16_t*>(out); a.lse = lse;
  a.stride_b = s.stride_b; a.stride_h = s.stride_h; a.stride_n = s.stride_n;
  a.bh = s.B * s.H; a.H = s.H; a.n = s.n; a.nb = nb; a.block = s.block; a.tail = s.n - (nb - 1) * s.block;
  a.scale = effective_scale(&s);
  a.n_slices = 1;
  if (sparse) {
    if (!mask) {  // the caller has index lists only: the bitmap the kernel walks is built from them
      uint32_t* built = reinterpret_cast<uint32_t*>(base + w.bitmap);
      if (pasa_launch_mask_from_idx(idx, (int64_t)s.B * s.H * nb, nb, k_sel, built, static_cast<hipStream_t>(stream)) != hipSuccess)
        return PASA_EHIP;
      mask = built;
    }
    a.idx = idx; a.mask = mask; a.k_sel = k_sel; a.mask_words = (nb + 31) / 32;
    a.group = s.group >= nb ? nb : s.group;
    a.st = reinterpret_cast<const uint16_t*>(base + w.st);
    a.hg = reinterpret_cast<const uint16_t*>(base + w.hg);
    a.n_groups = w.n_groups;
    a.n_chunks = w.n_chunks;
    a.n_slices = w.n_slices;
    a.part_o = reinterpret_cast<float*>(base + w.part_o);
    a.part_ml = reinterpret_cast<float*>(base + w.part_ml);
    a.queue = reinterpret_cast<uint32_t*>(base + w.queue);
  }
  return pasa_launch_attn(a, sparse, s.d, static_cast<hipStream_t>(stream)) == hipSuccess ? PASA_OK : PASA_EHIP;
}

int pasa_sparse_attn_fwd(const void* q, const void* k, const void* v, const pasa_shape_t* shape, const int32_t* idx,
                         const uint32_t* mask, int32_t k_sel, void* out, float* lse, void* ws, size_t ws_bytes,
                         void* stream) {
  return attn_common(q, k, v, shape, idx, mask, k_sel, out, lse, ws, ws_bytes, stream, true, true);
}

int pasa_sparse_attn_fwd_prepared(const void* q, const void* k, const void* v, const pasa_shape_t* shape,
                                  const int32_t* idx, const uint32_t* mask, int32_t k_sel, void* out, float* lse,
                                  void* ws, size_t ws_bytes, void* stream) {
  return attn_common(q, k, v, shape, idx, mask, k_sel, out, lse, ws, ws_bytes, stream, true, false);
}

int pasa_sparse_attn_fwd_static(const void* q, const void* k, const void* v, const pasa_shape_t* shape,
                                const int32_t* idx, const uint32_t* mask, int32_t k_sel, void* out, float* lse,
                                void* stream) {
  const int rc = check_shape(shape);
  if (rc != PASA_OK) return rc;
  pasa_shape_t s = *shape;
  s.kv_slices = 1;  // the partial results of key-range slicing do not fit a modest static buffer
  const size_t need = pasa_attn_workspace_bytes(&s);
  if (need == 0) return check_group(s.group, num_blocks(&s)) != PASA_OK ? check_group(s.group, num_blocks(&s)) : PASA_EINVAL;
  if (need > (size_t)PASA_STATIC_SCRATCH_BYTES) return PASA_ESCRATCH;
  if (!q || !k || !v || !out || (!idx && !mask) || k_sel < 1 || k_sel > num_blocks(&s)) return PASA_EINVAL;
  void* ws = nullptr;
  const int rp = static_scratch(&ws);
  if (rp != PASA_OK) return rp;
  return attn_common(q, k, v, &s, idx, mask, k_sel, out, lse, ws, (size_t)PASA_STATIC_SCRATCH_BYTES, stream, true, true);
}

// ---- the whole forward in one call ---------------------------------------------------------------
namespace {
struct ForwardWorkspace {
  size_t scores, idx, mask, score_ws, attn_ws, total;
  int nb, k_sel;
};

// 0 in `total` on invalid arguments
ForwardWorkspace carve_forward(const pasa_shape_t* s, double keep_ratio) {
  ForwardWorkspace f{};
  if (check_shape(s) != PASA_OK) return f;
  f.nb = num_blocks(s);
  const int32_t k = pasa_topk_count(f.nb, keep_ratio);
  if (k < 1) return f;
  f.k_sel = k;
  pasa_shape_t a = *s;
  const size_t attn = pasa_attn_workspace_bytes(&a), score = pasa_score_workspace_bytes(&a);
  if (attn == 0 || score == 0) return f;
  const size_t bh = (size_t)s->B * s->H;
  size_t off = 0;
  f.scores = off; off = align_up(off + bh * f.nb * f.nb * 4);
  f.idx = off; off = align_up(off + bh * f.nb * (size_t)k * 4);
  f.mask = off; off = align_up(off + bh * f.nb * (size_t)((f.nb + 31) / 32) * 4);
  f.score_ws = off; off = align_up(off + score);
  f.attn_ws = off; off = align_up(off + attn);
  f.total = off;
  return f;
}
}  // namespace

size_t pasa_forward_workspace_bytes(const pasa_shape_t* shape, double keep_ratio) { return carve_forward(shape, keep_ratio).total; }

int pasa_forward(const void* q, const void* k, const void* v, const pasa_shape_t* shape, double keep_ratio, uint64_t seed,
                 float noise_amp, void* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != PASA_OK) return rc;
  if (!(keep_ratio > 0.0) || keep_ratio > 1.0) return PASA_EINVAL;
  const int rg = check_group(shape->group, num_blocks(shape));
  if (rg != PASA_OK) return rg;
  const int rs = check_slices(shape);
  if (rs != PASA_OK) return rs;
  const ForwardWorkspace f = carve_forward(shape, keep_ratio);
  if (f.total == 0) return PASA_EUNSUPPORTED;
  if (!q || !k || !v || !out || !ws) return PASA_EINVAL;
  if (!aligned16(ws)) return PASA_EALIGN;
  if (ws_bytes < f.total) return PASA_EWORKSPACE;
  if (f.nb > kRouteMaxBlocks) return PASA_EUNSUPPORTED;
  char* base = static_cast<char*>(ws);
  float* scores = reinterpret_cast<float*>(base + f.scores);
  int32_t* idx = reinterpret_cast<int32_t*>(base + f.idx);
  uint32_t* mask = reinterpret_cast<uint32_t*>(base + f.mask);
  const size_t attn_bytes = pasa_attn_workspace_bytes(shape), score_bytes = pasa_score_workspace_bytes(shape);
  int r;
  if (shape->group > 0) {  // the statistics first: scoring takes the block-mean keys from them
    r = pasa_kv_stats(k, v, shape, base + f.attn_ws, attn_bytes, stream);
    if (r != PASA_OK) return r;
    r = pasa_block_score_with_stats(q, shape, nullptr, scores, base + f.score_ws, score_bytes, base + f.attn_ws, attn_bytes, stream);
  } else {
    r = pasa_block_score(q, k, shape, nullptr, scores, base + f.score_ws, score_bytes, stream);
  }
  if (r != PASA_OK) return r;
  r = pasa_route(scores, shape->B * shape->H, f.nb, f.k_sel, seed, noise_amp, idx, mask, stream);
  if (r != PASA_OK) return r;
  return pasa_sparse_attn_fwd_prepared(q, k, v, shape, idx, mask, f.k_sel, out, lse, base + f.attn_ws, attn_bytes, stream);
}

int pasa_attn_dense_ref(const void* q, const void* k, const void* v, const pasa_shape_t* shape, void* out, float* lse,
                        void* ws, size_t ws_bytes, void* stream) {
  return attn_common(q, k, v, shape, nullptr, nullptr, 0, out, lse, ws, ws_bytes, stream, false, false);
}

}  // extern "C"

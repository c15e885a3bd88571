// C ABI of the LineAR decode path: argument checks, the host-side line/budget state
// machine (Sec. 3.3: cache lengths, region boundaries and the eviction schedule depend
// only on the line index, never on the data, so they live on the host and no call has to
// read the device back) and the kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/linear_kv.h"
#include "../../include/linear_kv_diag.h"
#include "kernels.h"

namespace {

thread_local int g_last_hip_error = 0;

using linear::kMaxMid;              // candidates the eviction kernel ranks in LDS
constexpr int kMaxLine = 4096;      // guide queries whose row statistics it keeps in LDS
constexpr int kMaxScored = 7680;    // scored slots per pair when attention is accumulated: the decode step
                                    // stages their logits in LDS next to up to 33 KB of softmax partials,
                                    // within the 64 KiB every workgroup may use
constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Derived {
  int pairs;        // Bz * H
  int t_max;        // C + B
  int elem;         // bytes per element
  int row_bytes;    // d * elem
  bool compresses;  // B < N
  int mid_lo;       // C + N_init
  int mid_n;        // B - N_init - r n   (0 when nothing is ever evicted)
  int n_tail;       // r n
  int first_line;   // B / n: first line (1-based) that ends in an eviction
  int max_split;    // pitch of the split-partial buffers
  float scale;
  // scratch layout (byte offsets)
  int guide_w;      // logits per guide-queue row: mid_n, or B - N_init when attention is accumulated
  bool queries;     // the guide queue holds the queries (Eq. 8 as printed), not their logits
  bool scored;      // a guide queue is kept at all (not with random eviction)
  size_t off_guide, off_qq, off_pos, off_acc, off_part_o, off_part_ml, total;
  size_t guide_layer, pos_layer, acc_layer;   // element strides per layer
  size_t qq_layer;                 // bytes of one layer's query queue [P, n, d] elem
  int pos_pitch;                   // entries per pair of the survivor position map
  int guide_row;    // floats per queue row in memory: guide_w + 2 rounded up to whole 128-byte lines
  size_t guide_pair;               // floats of one pair's guide queue: n * guide_row
};

int derive(const linear_cfg_t& c, Derived* d) {
  if (c.n_layers < 1 || c.batch < 1 || c.n_heads < 1) return LINEAR_EINVAL;
  if (c.head_dim != 64 && c.head_dim != 128) return LINEAR_EINVAL;
  if (c.dtype != LINEAR_F32 && c.dtype != LINEAR_BF16) return LINEAR_EINVAL;
  if (c.score_mode < 0 || c.score_mode > 3) return LINEAR_EINVAL;
  if (c.guide_queue < LINEAR_QUEUE_AUTO || c.guide_queue > LINEAR_QUEUE_QUERIES) return LINEAR_EINVAL;
  if (c.guide_queue == LINEAR_QUEUE_QUERIES && c.score_mode != 0) return LINEAR_EINVAL;   // the other modes score decode-time probabilities
  if (c.score_mode == 3 && c.guide_queue != LINEAR_QUEUE_AUTO) return LINEAR_EINVAL;       // random eviction keeps no queue
  if (c.out_dtype != LINEAR_OUT_F32 && c.out_dtype != LINEAR_OUT_ELEM) return LINEAR_EINVAL;
  if (c.n_cond < 0 || c.line_len < 1 || c.n_lines < 1) return LINEAR_EINVAL;
  if (!(c.scale >= 0.f) || std::isinf(c.scale)) return LINEAR_EINVAL;
  const int64_t N = (int64_t)c.line_len * c.n_lines;
  if (c.budget < c.line_len || c.budget > N || c.budget % c.line_len) return LINEAR_EINVAL;
  if (c.n_init < 0 || c.n_recent_lines < 1) return LINEAR_EINVAL;
  if (c.n_init > c.budget || c.n_recent_lines > c.n_lines) return LINEAR_EINVAL;   // the anchor and the window are parts of the image
  if ((int64_t)c.n_cond + c.budget > (1 << 20)) return LINEAR_EINVAL;
  if ((int64_t)c.batch * c.n_heads > (1 << 24) || c.n_layers > (1 << 16)) return LINEAR_EINVAL;
  d->compresses = c.budget < N;
  const int64_t tail = (int64_t)c.n_recent_lines * c.line_len;   // r n
  if (d->compresses && (int64_t)c.n_init + tail + c.line_len > c.budget)
    return LINEAR_EINVAL;   // mid must hold at least the n tokens to evict
  d->pairs = c.batch * c.n_heads;
  d->t_max = c.n_cond + c.budget;
  d->elem = c.dtype == LINEAR_BF16 ? 2 : 4;
  d->row_bytes = c.head_dim * d->elem;
  d->mid_lo = c.n_cond + c.n_init;
  d->n_tail = d->compresses ? (int)tail : 0;                     // (a full cache has no regions)
  d->mid_n = d->compresses ? c.budget - c.n_init - d->n_tail : 0;
  if (d->mid_n > kMaxMid || c.line_len > kMaxLine) return LINEAR_EINVAL;
  d->first_line = c.budget / c.line_len;
  d->max_split = linear::kMaxSplit;
  d->scale = c.scale > 0.f ? c.scale : 1.0f / std::sqrt((float)c.head_dim);
  const size_t P = (size_t)d->pairs;
  d->guide_w = !d->compresses ? 0 : (c.score_mode == 2 ? c.budget - c.n_init : d->mid_n);
  if (d->guide_w > kMaxScored) return LINEAR_EINVAL;
  d->guide_row = (d->guide_w + 2 + 31) / 32 * 32;
  d->scored = d->compresses && c.score_mode != 3;
  d->guide_pair = d->scored ? (size_t)c.line_len * d->guide_row : 0;
  d->queries = d->compresses && c.score_mode == 0 && c.guide_queue != LINEAR_QUEUE_LOGITS;
  // With a queue of queries the logits exist only inside the end-of-line kernel (in LDS, or in
  // one layer's worth of this buffer when they do not fit), so the layers share it.
  d->guide_layer = d->queries ? 0 : P * d->guide_pair;
  d->qq_layer = d->queries ? P * (size_t)c.line_len * d->row_bytes : 0;
  d->acc_layer = c.score_mode == 2 ? P * (size_t)d->guide_w : 0;
  // Original positions are kept only for the survivors of evictions, mid_n - n per pair: every
  // other row's position follows from its index (prefix and anchor in front, whole consecutive
  // lines behind).
  d->pos_pitch = d->compresses ? (std::max(1, d->mid_n - c.line_len) + 31) / 32 * 32 : 32;   // whole 128-byte lines
  d->pos_layer = P * (size_t)d->pos_pitch;
  // Every part is at most 2^24 pairs x 2^25 words x 2^16 layers, which does not fit 64 bits:
  // a configuration whose scratch would exceed 2^44 bytes is refused before the offsets are formed.
  {
    typedef unsigned __int128 u128;
    const u128 L = (u128)c.n_layers;
    const u128 total = (u128)P * d->guide_pair * (d->queries ? 1 : L) * 4 + (u128)d->qq_layer * L +
                       (u128)d->pos_layer * L * 4 + (u128)d->acc_layer * L * 4 +
                       (u128)P * d->max_split * (c.head_dim + 2) * 4 + 6 * kAlign;
    const u128 cache = (u128)P * (u128)d->t_max * d->row_bytes;
    if (total > ((u128)1 << 44) || cache > ((u128)1 << 44)) return LINEAR_EINVAL;
  }
  size_t off = 0;
  d->off_guide = off;    off = align_up(off + P * d->guide_pair * (d->queries ? 1 : c.n_layers) * sizeof(float));
  d->off_qq = off;       off = align_up(off + d->qq_layer * c.n_layers);
  d->off_pos = off;      off = align_up(off + d->pos_layer * c.n_layers * sizeof(int32_t));
  d->off_acc = off;      off = align_up(off + d->acc_layer * c.n_layers * sizeof(float));
  d->off_part_o = off;   off = align_up(off + P * d->max_split * c.head_dim * sizeof(float));
  d->off_part_ml = off;  off = align_up(off + P * d->max_split * 2 * sizeof(float));
  d->total = off;
  return LINEAR_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return LINEAR_EHIP;
}

struct LayerState {
  int visual_len = 0;      // visual tokens cached
  int in_line = 0;         // decode steps since the last end of line
  int lines_done = 0;
  int mapped = 0;          // mid rows whose original position is in the survivor map
};

}  // namespace

// ---- decode_step_static: the split partials live in device memory the library itself holds
// (a file-scope array), for callers that can neither allocate device memory nor hand over a
// workspace.  Every GPU the library runs on holds its own copy of the array at its own address
// until the process ends; the address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char static_scratch[kStaticScratchBytes];

namespace {

std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};

// Device address of this device's copy of static_scratch (never the array's name: in host code
// that is only a stand-in for the symbol).  *ptr is null on failure.
hipError_t static_scratch_ptr(void** ptr) {
  *ptr = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
    if (e != hipSuccess) return e;
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = p;
  }
  *ptr = g_static_ptr[dev];
  return hipSuccess;
}

}  // namespace

struct linear_kv {
  linear_cfg_t cfg;
  Derived d;
  std::vector<void*> k_cache, v_cache;
  char* scratch;
  std::vector<LayerState> layer;
  int groups_per_wave;   // tuning: row groups a wavefront should take (1..16), 0 = automatic
  int force_split;       // tuning: 0 = automatic
};

namespace {

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Launch shape of one decode step: how the cached keys of a pair are dealt to workgroups
// (splits) and wavefronts.  A wavefront holds up to `depth` row groups in registers; a
// workgroup of up to decode_max_waves(depth) wavefronts holds a whole pair when it can
// (one launch); longer caches, or too few pairs to fill 256 CUs, are split.
struct Plan {
  int n_split, rows_per_split, n_waves, depth, new_wave;
};

bool make_plan(int dtype, int head_dim, int pairs, bool stages_logits, int target, int force_split,
               int cached_rows, Plan* p) {
  const int rpg = linear::decode_rows_per_group(dtype, head_dim);
  const int groups = ceil_div(cached_rows, rpg);
  int n_split = force_split;
  if (n_split == 0) {
    n_split = 1;
    if (groups > 144) n_split = ceil_div(groups, 128);
    if (pairs < 256 && groups >= 32) {   // few pairs: split to put ~256 workgroups in flight
      const int want = std::min(ceil_div(256, pairs), groups / 16);
      n_split = std::max(n_split, want);
    }
  }
  if (groups > 144 * n_split) n_split = ceil_div(groups, 128);   // a forced count that cannot hold the keys
  if (n_split > linear::kMaxSplit) return false;
  int gps = ceil_div(groups, n_split);                    // row groups per split
  while (n_split > 1 && (int64_t)(n_split - 1) * gps * rpg >= cached_rows) {   // no empty split
    --n_split;
    gps = ceil_div(groups, n_split);
  }
  if (gps < 1) gps = 1;
  // Wavefronts per workgroup: enough for `target` row groups each, at least as many as the
  // deepest kernel needs, at most what the register budget of the resulting depth allows.
  // Default shape (measured on all five workloads): the deepest wavefronts that still put
  // about five wavefronts on every compute unit (eight when the step also stages logits for a
  // guide queue of logits: the wavefront that stores them should not be the one that merges);
  // few, long wavefronts keep the per-wavefront prologue and merge small (a 12-deep wavefront
  // has 24 KiB of loads in flight), but a launch with too few of them cannot cover the memory
  // latency.
  int nw;
  if (target > 0) {
    nw = std::max(ceil_div(gps, target), ceil_div(gps, 16));
  } else {
    const int want_total = (stages_logits ? 8 : 5) * 256;
    nw = std::max(ceil_div(gps, 16), ceil_div(want_total, pairs * n_split));
    // wavefronts deeper than 12 row groups (three per SIMD fit) only pay when the launch has
    // at least eight wavefronts per compute unit anyway
    if ((int64_t)nw * pairs * n_split < 8 * 256) nw = std::max(nw, ceil_div(gps, 12));
    nw = std::min(nw, gps);
  }
  nw = std::max(1, std::min(16, nw));
  // The nearest wavefront count whose depth is instantiated and fits the register budget
  // (first upwards, then downwards).
  for (int k = 0; k < 32; ++k) {
    const int cand = k < 17 - nw ? nw + k : nw - (k - (16 - nw));
    if (cand < 1 || cand > 16) continue;
    const int depth = linear::decode_depth_for(ceil_div(gps, cand));
    if (depth == 0 || cand > linear::decode_max_waves(depth)) continue;
    p->n_split = n_split;
    p->rows_per_split = gps * rpg;
    p->depth = depth;
    p->n_waves = cand;
    // Row groups are dealt round-robin, so in the last split wavefront (groups % nw) is the
    // first with one group fewer: it takes the appended token.
    p->new_wave = (groups - (n_split - 1) * gps) % cand;
    return true;
  }
  return false;
}

bool line_evicts(const linear_kv& kv, int line /*1-based*/) {
  return kv.d.compresses && line >= kv.d.first_line && line <= kv.cfg.n_lines - 1;
}

// Arguments of the end-of-line kernels for the layer's current line with `rows` queries queued.
void fill_line_args(const linear_kv& kv, int layer, int rows, linear::EvictArgs* a) {
  const linear_cfg_t& c = kv.cfg;
  const Derived& d = kv.d;
  const LayerState& ls = kv.layer[layer];
  *a = linear::EvictArgs{};
  a->kc = kv.k_cache[layer];
  a->vc = kv.v_cache[layer];
  a->pos = reinterpret_cast<int32_t*>(kv.scratch + d.off_pos) + d.pos_layer * layer;
  a->pos_pitch = d.pos_pitch;
  a->pos_mapped = ls.mapped;
  // the candidates behind the mapped ones are consecutive tokens that end where the recent
  // window begins: at the first eviction all of mid (every row still sits at its own index),
  // afterwards the line that has just left the window
  a->pos_base = c.n_cond + (ls.lines_done + 1 - c.n_recent_lines) * c.line_len - (d.mid_n - ls.mapped);
  a->guide = reinterpret_cast<const float*>(kv.scratch + d.off_guide) + d.guide_layer * layer;
  a->guide_out = reinterpret_cast<float*>(kv.scratch + d.off_guide) + d.guide_layer * layer;
  a->qq = d.queries ? kv.scratch + d.off_qq + d.qq_layer * layer : nullptr;
  a->scale_log2e = d.scale * 1.4426950408889634f;
  a->elem_bf16 = c.dtype == LINEAR_BF16;
  a->acc = reinterpret_cast<float*>(kv.scratch + d.off_acc) + d.acc_layer * layer;
  a->n_rows = rows;
  a->line_len = c.line_len;
  a->guide_w = d.guide_w;
  a->guide_row = d.guide_row;
  a->score_mode = c.score_mode;
  a->n_pairs = d.pairs;
  a->t_max = d.t_max;
  a->mid_lo = d.mid_lo;
  a->mid_n = d.mid_n;
  a->n_evict = c.line_len;
  a->n_tail = d.n_tail;
  a->seed = c.seed;
  a->layer = layer;
  a->line = ls.lines_done + 1;
  a->n_heads = c.n_heads;
  if (c.score_mode == 3) a->n_rows = 0;   // no queue rows: the scores are hashes
  if (c.score_mode == 2) {
    // the line's first query saw (keys cached before the line) + 1 keys; every later one sees
    // one more; the scored ones are those behind the anchor
    const int t_first = c.n_cond + ls.visual_len - ls.in_line + 1;
    a->len0 = t_first - d.mid_lo;
    a->len_step = 1;
    a->n_cols = std::max(0, std::min(d.guide_w, c.n_cond + ls.visual_len - d.mid_lo));
  } else {
    a->len0 = d.mid_n;
    a->len_step = 0;
    a->n_cols = d.mid_n;
  }
}

}  // namespace

extern "C" {

int linear_workspace_bytes(const linear_cfg_t* cfg, size_t* cache_bytes_per_layer,
                           size_t* scratch_bytes) {
  if (!cfg) return LINEAR_ENULL;
  Derived d;
  const int rc = derive(*cfg, &d);
  if (rc != LINEAR_OK) return rc;
  if (cache_bytes_per_layer) *cache_bytes_per_layer = (size_t)d.pairs * d.t_max * d.row_bytes;
  if (scratch_bytes) *scratch_bytes = d.total;
  return LINEAR_OK;
}

int kv_init(const linear_cfg_t* cfg, void* const* k_cache, void* const* v_cache, void* scratch,
            const void* const* k_cond, const void* const* v_cond, void* stream,
            linear_kv_t** out) {
  if (!cfg || !k_cache || !v_cache || !scratch || !out) return LINEAR_ENULL;
  Derived d;
  const int rc = derive(*cfg, &d);
  if (rc != LINEAR_OK) return rc;
  if (cfg->n_cond > 0 && (!k_cond || !v_cond)) return LINEAR_ENULL;
  if (misaligned(scratch)) return LINEAR_EALIGN;
  for (int l = 0; l < cfg->n_layers; ++l) {
    if (!k_cache[l] || !v_cache[l]) return LINEAR_ENULL;
    if (misaligned(k_cache[l]) || misaligned(v_cache[l])) return LINEAR_EALIGN;
    if (cfg->n_cond > 0) {
      if (!k_cond[l] || !v_cond[l]) return LINEAR_ENULL;
      if (misaligned(k_cond[l]) || misaligned(v_cond[l])) return LINEAR_EALIGN;
    }
  }
  linear_kv* kv = nullptr;
  try {
    kv = new linear_kv;
    kv->cfg = *cfg;
    kv->d = d;
    kv->k_cache.assign(k_cache, k_cache + cfg->n_layers);
    kv->v_cache.assign(v_cache, v_cache + cfg->n_layers);
    kv->scratch = static_cast<char*>(scratch);
    kv->layer.assign(cfg->n_layers, LayerState());
    kv->groups_per_wave = 0;
    kv->force_split = 0;
  } catch (...) {   // host allocation failure must not cross the C boundary
    delete kv;
    return LINEAR_EINVAL;
  }

  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  // The guide queues and the survivor position maps are written before they are read;
  // attention accumulators start at zero.
  e = linear::launch_fill_u32(kv->scratch + d.off_acc, 0u, d.acc_layer * cfg->n_layers, s);
  for (int l = 0; l < cfg->n_layers && e == hipSuccess; ++l) {
    if (e == hipSuccess && cfg->n_cond == 0) {
      // With an empty cache the first step's masked loads touch row 0: give it defined bits.
      e = linear::launch_zero_rows(kv->k_cache[l], d.t_max, 1, d.pairs, d.row_bytes, s);
      if (e == hipSuccess) e = linear::launch_zero_rows(kv->v_cache[l], d.t_max, 1, d.pairs, d.row_bytes, s);
    }
    if (e == hipSuccess && cfg->n_cond > 0)
      e = linear::launch_copy_rows(kv->k_cache[l], d.t_max, k_cond[l], cfg->n_cond, cfg->n_cond,
                                   d.pairs, d.row_bytes, s);
    if (e == hipSuccess && cfg->n_cond > 0)
      e = linear::launch_copy_rows(kv->v_cache[l], d.t_max, v_cond[l], cfg->n_cond, cfg->n_cond,
                                   d.pairs, d.row_bytes, s);
  }
  if (e != hipSuccess) {
    delete kv;
    return hip_fail(e);
  }
  *out = kv;
  return LINEAR_OK;
}

}  // extern "C"

namespace {

// One decode step of one layer; `cos_sin` is null when q and k arrive rotated.
int decode_step_impl(linear_kv_t* kv, int32_t layer, const void* q, const void* k, const void* v,
                     const float* cos_sin, void* out, void* stream) {
  if (!kv || !q || !k || !v || !out) return LINEAR_ENULL;
  if (layer < 0 || layer >= kv->cfg.n_layers) return LINEAR_EINVAL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out)) return LINEAR_EALIGN;
  LayerState& ls = kv->layer[layer];
  const linear_cfg_t& c = kv->cfg;
  const Derived& d = kv->d;
  if (ls.lines_done >= c.n_lines) return LINEAR_ESTATE;      // image complete
  if (ls.in_line >= c.line_len) return LINEAR_ESTATE;        // end_of_line_evict is due
  if (ls.visual_len >= c.budget) return LINEAR_ESTATE;       // cannot happen in a valid sequence

  const int line = ls.lines_done + 1;
  linear::DecodeArgs a;
  a.q = q;
  a.k_new = k;
  a.v_new = v;
  a.cos_sin = cos_sin;
  a.kc = kv->k_cache[layer];
  a.vc = kv->v_cache[layer];
  a.out = out;
  a.out_bf16 = c.out_dtype == LINEAR_OUT_ELEM && c.dtype == LINEAR_BF16;
  a.part_o = reinterpret_cast<float*>(kv->scratch + d.off_part_o);
  a.part_ml = reinterpret_cast<float*>(kv->scratch + d.off_part_ml);
  a.guide = reinterpret_cast<float*>(kv->scratch + d.off_guide) + d.guide_layer * layer +
            (size_t)ls.in_line * d.guide_row;
  a.guide_pitch = (int64_t)d.guide_pair;
  a.guide_w = d.guide_w;
  a.guide_row = d.guide_row;
  a.n_pairs = d.pairs;
  a.t = c.n_cond + ls.visual_len + 1;
  a.t_max = d.t_max;
  Plan plan;
  if (!make_plan(c.dtype, c.head_dim, d.pairs, d.scored && !d.queries, kv->groups_per_wave,
                 kv->force_split, a.t - 1, &plan))
    return LINEAR_EINVAL;
  a.n_split = plan.n_split;
  a.rows_per_split = plan.rows_per_split;
  a.n_waves = plan.n_waves;
  a.new_wave = plan.new_wave;
  a.depth = plan.depth;
  a.max_split = d.max_split;
  a.mid_lo = d.mid_lo;
  if (c.score_mode == 2) {
    // accumulated attention: every key behind the anchor is scored on every line, the
    // appended one included
    a.mid_n = d.compresses ? std::max(0, std::min(d.guide_w, a.t - d.mid_lo)) : 0;
    a.stage_new = 1;
    a.store_ml = 1;
  } else {
    a.mid_n = d.scored && line_evicts(*kv, line) ? d.mid_n : 0;   // random eviction scores nothing
    a.stage_new = 0;
    a.store_ml = c.score_mode == 1;
  }
  a.qq = nullptr;
  a.qq_pitch = (int64_t)c.line_len * d.row_bytes;
  if (d.queries) {
    if (a.mid_n > 0) a.qq = kv->scratch + d.off_qq + d.qq_layer * layer + (size_t)ls.in_line * d.row_bytes;
    a.mid_n = 0;   // no logits leave the decode step
  }
  a.score_mode = c.score_mode;
  a.scale_log2e = d.scale * 1.4426950408889634f;
  const hipError_t e = linear::launch_decode(a, c.dtype, c.head_dim, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e);
  ls.visual_len += 1;
  ls.in_line += 1;
  return LINEAR_OK;
}

int decode_layers_impl(linear_kv_t* kv, int32_t first_layer, int32_t count, const void* q, const void* k,
                       const void* v, const float* cos_sin, void* out, size_t qkv_stride,
                       size_t out_stride, void* stream) {
  if (!kv || !q || !k || !v || !out) return LINEAR_ENULL;
  if (count < 0 || first_layer < 0 || (int64_t)first_layer + count > kv->cfg.n_layers) return LINEAR_EINVAL;
  if ((qkv_stride | out_stride) & 15u) return LINEAR_EALIGN;
  for (int32_t i = 0; i < count; ++i) {
    const int rc = decode_step_impl(kv, first_layer + i, static_cast<const char*>(q) + i * qkv_stride,
                                    static_cast<const char*>(k) + i * qkv_stride,
                                    static_cast<const char*>(v) + i * qkv_stride, cos_sin,
                                    static_cast<char*>(out) + i * out_stride, stream);
    if (rc != LINEAR_OK) return rc;
  }
  return LINEAR_OK;
}

}  // namespace

extern "C" {

int decode_step(linear_kv_t* kv, int32_t layer, const void* q, const void* k, const void* v,
                void* out, void* stream) {
  return decode_step_impl(kv, layer, q, k, v, nullptr, out, stream);
}

int decode_step_rope(linear_kv_t* kv, int32_t layer, const void* q, const void* k, const void* v,
                     const float* cos_sin, void* out, void* stream) {
  if (!cos_sin) return LINEAR_ENULL;
  if (misaligned(cos_sin)) return LINEAR_EALIGN;
  return decode_step_impl(kv, layer, q, k, v, cos_sin, out, stream);
}

int end_of_line_evict(linear_kv_t* kv, int32_t layer, void* stream) {
  if (!kv) return LINEAR_ENULL;
  if (layer < 0 || layer >= kv->cfg.n_layers) return LINEAR_EINVAL;
  LayerState& ls = kv->layer[layer];
  const linear_cfg_t& c = kv->cfg;
  const Derived& d = kv->d;
  if (ls.in_line != c.line_len) return LINEAR_ESTATE;
  const int line = ls.lines_done + 1;
  const bool evicts = line_evicts(*kv, line);
  if (evicts || (c.score_mode == 2 && d.compresses)) {
    linear::EvictArgs a;
    fill_line_args(*kv, layer, c.line_len, &a);
    hipError_t e = hipSuccess;
    if (evicts)
      e = linear::launch_evict(a, nullptr, c.dtype, c.head_dim, static_cast<hipStream_t>(stream));
    else if (a.n_cols > 0)   // accumulated attention: fold the line's queue into the accumulators
      e = linear::launch_saliency(a, c.dtype, c.head_dim, nullptr, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    if (evicts) {
      ls.visual_len -= c.line_len;
      ls.mapped = d.mid_n - c.line_len;
    }
  }
  ls.in_line = 0;
  ls.lines_done += 1;
  return LINEAR_OK;
}

int decode_step_layers(linear_kv_t* kv, int32_t first_layer, int32_t count, const void* q,
                       const void* k, const void* v, void* out, size_t qkv_stride,
                       size_t out_stride, void* stream) {
  return decode_layers_impl(kv, first_layer, count, q, k, v, nullptr, out, qkv_stride, out_stride, stream);
}

int decode_step_rope_layers(linear_kv_t* kv, int32_t first_layer, int32_t count, const void* q,
                            const void* k, const void* v, const float* cos_sin, void* out,
                            size_t qkv_stride, size_t out_stride, void* stream) {
  if (!cos_sin) return LINEAR_ENULL;
  if (misaligned(cos_sin)) return LINEAR_EALIGN;
  return decode_layers_impl(kv, first_layer, count, q, k, v, cos_sin, out, qkv_stride, out_stride, stream);
}

int end_of_line_evict_layers(linear_kv_t* kv, int32_t first_layer, int32_t count, void* stream) {
  if (!kv) return LINEAR_ENULL;
  if (count < 0 || first_layer < 0 || (int64_t)first_layer + count > kv->cfg.n_layers) return LINEAR_EINVAL;
  const linear_cfg_t& c = kv->cfg;
  const Derived& d = kv->d;
  // Layers in the same state that end an evicting line share launches (their evictions do not
  // depend on one another): one launch per group of layers instead of one per layer.
  bool together = count > 1;
  for (int32_t i = 0; i < count && together; ++i) {
    const LayerState& a = kv->layer[first_layer + i];
    const LayerState& b = kv->layer[first_layer];
    together = a.in_line == c.line_len && a.lines_done == b.lines_done && a.visual_len == b.visual_len &&
               a.mapped == b.mapped;
  }
  if (together) together = line_evicts(*kv, kv->layer[first_layer].lines_done + 1);
  linear::EvictArgs a;
  if (together) {
    fill_line_args(*kv, first_layer, c.line_len, &a);
    together = linear::evict_layers_may_share_launch(a, std::min<int32_t>(count, linear::kMaxEvictLayers),
                                                     c.dtype, c.head_dim);
  }
  if (!together) {
    for (int32_t i = 0; i < count; ++i) {
      const int rc = end_of_line_evict(kv, first_layer + i, stream);
      if (rc != LINEAR_OK) return rc;
    }
    return LINEAR_OK;
  }
  for (int32_t l0 = 0; l0 < count; l0 += linear::kMaxEvictLayers) {
    const int32_t m = std::min<int32_t>(linear::kMaxEvictLayers, count - l0);
    fill_line_args(*kv, first_layer + l0, c.line_len, &a);
    linear::EvictLayers ly = {};
    ly.count = m;
    ly.guide_stride = (int64_t)d.guide_layer;
    ly.qq_stride = (int64_t)d.qq_layer;
    ly.pos_stride = (int64_t)d.pos_layer;
    ly.acc_stride = (int64_t)d.acc_layer;
    for (int32_t i = 0; i < m; ++i) {
      ly.kc[i] = kv->k_cache[first_layer + l0 + i];
      ly.vc[i] = kv->v_cache[first_layer + l0 + i];
    }
    const hipError_t e = linear::launch_evict(a, &ly, c.dtype, c.head_dim, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);   // layers of earlier groups have been enqueued and advanced
    for (int32_t i = 0; i < m; ++i) {
      LayerState& ls = kv->layer[first_layer + l0 + i];
      ls.visual_len -= c.line_len;
      ls.mapped = d.mid_n - c.line_len;
      ls.in_line = 0;
      ls.lines_done += 1;
    }
  }
  return LINEAR_OK;
}

int kv_scores(linear_kv_t* kv, int32_t layer, float* out, int32_t* mid_out, void* stream) {
  if (!kv || !out) return LINEAR_ENULL;
  if (layer < 0 || layer >= kv->cfg.n_layers) return LINEAR_EINVAL;
  if (misaligned(out)) return LINEAR_EALIGN;
  const LayerState& ls = kv->layer[layer];
  if (ls.lines_done >= kv->cfg.n_lines || !line_evicts(*kv, ls.lines_done + 1)) return LINEAR_ESTATE;
  const Derived& d = kv->d;
  linear::EvictArgs a;
  fill_line_args(*kv, layer, ls.in_line, &a);
  const hipError_t e = linear::launch_saliency(a, kv->cfg.dtype, kv->cfg.head_dim, out, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e);
  if (mid_out) *mid_out = d.mid_n;
  return LINEAR_OK;
}

int kv_gather(linear_kv_t* kv, int32_t layer, void* k_out, void* v_out, int32_t* pos_out,
              int32_t* len_out, void* stream) {
  if (!kv) return LINEAR_ENULL;
  if (layer < 0 || layer >= kv->cfg.n_layers) return LINEAR_EINVAL;
  if (misaligned(k_out) || misaligned(v_out) || (reinterpret_cast<uintptr_t>(pos_out) & 3u))
    return LINEAR_EALIGN;
  const Derived& d = kv->d;
  const int len = kv->cfg.n_cond + kv->layer[layer].visual_len;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  // Compaction keeps the cache in ascending original position, so the canonical order is
  // the storage order and the export is a strided copy of the first `len` rows.
  if (k_out) e = linear::launch_copy_rows(k_out, len, kv->k_cache[layer], d.t_max, len, d.pairs, d.row_bytes, s);
  if (e == hipSuccess && v_out)
    e = linear::launch_copy_rows(v_out, len, kv->v_cache[layer], d.t_max, len, d.pairs, d.row_bytes, s);
  if (e == hipSuccess && pos_out) {
    const LayerState& ls = kv->layer[layer];
    const int32_t* map = reinterpret_cast<const int32_t*>(kv->scratch + d.off_pos) + d.pos_layer * layer;
    const int newest = kv->cfg.n_cond + ls.lines_done * kv->cfg.line_len + ls.in_line - 1;
    e = linear::launch_positions(pos_out, map, d.pos_pitch, d.mid_lo, ls.mapped, len, newest, d.pairs, s);
  }
  if (e != hipSuccess) return hip_fail(e);
  if (len_out) *len_out = len;
  return LINEAR_OK;
}

int kv_length(const linear_kv_t* kv, int32_t layer, int32_t* cached_tokens, int32_t* tokens_in_line,
              int32_t* lines_done) {
  if (!kv) return LINEAR_ENULL;
  if (layer < 0 || layer >= kv->cfg.n_layers) return LINEAR_EINVAL;
  const LayerState& ls = kv->layer[layer];
  if (cached_tokens) *cached_tokens = kv->cfg.n_cond + ls.visual_len;
  if (tokens_in_line) *tokens_in_line = ls.in_line;
  if (lines_done) *lines_done = ls.lines_done;
  return LINEAR_OK;
}

int linear_set_tuning(linear_kv_t* kv, int32_t groups_per_wave, int32_t n_split) {
  if (!kv) return LINEAR_ENULL;
  if (groups_per_wave < 0 || groups_per_wave > 16 || n_split < 0 || n_split > linear::kMaxSplit)
    return LINEAR_EINVAL;
  kv->groups_per_wave = groups_per_wave;
  kv->force_split = n_split;
  return LINEAR_OK;
}

int linear_plan_shape(const linear_cfg_t* cfg, int32_t cached_keys, int32_t groups_per_wave,
                      int32_t n_split, int32_t* shape) {
  if (!cfg || !shape) return LINEAR_ENULL;
  Derived d;
  const int rc = derive(*cfg, &d);
  if (rc != LINEAR_OK) return rc;
  if (cached_keys < 0 || cached_keys >= d.t_max || groups_per_wave < 0 || groups_per_wave > 16 ||
      n_split < 0 || n_split > linear::kMaxSplit)
    return LINEAR_EINVAL;
  Plan p;
  if (!make_plan(cfg->dtype, cfg->head_dim, d.pairs, d.scored && !d.queries, groups_per_wave, n_split,
                 cached_keys, &p))
    return LINEAR_EINVAL;
  shape[0] = p.n_split;
  shape[1] = p.rows_per_split;
  shape[2] = p.n_waves;
  shape[3] = p.depth;
  shape[4] = p.new_wave;
  shape[5] = linear::decode_rows_per_group(cfg->dtype, cfg->head_dim);
  return LINEAR_OK;
}

int kv_free(linear_kv_t* kv) {
  delete kv;
  return LINEAR_OK;
}

int linear_probe_stream(const void* const* k_cache, const void* const* v_cache, int32_t n_layers, int32_t n_pairs,
                        int32_t rows, int32_t pitch_rows, int32_t row_bytes, void* stream) {
  if (!k_cache || !v_cache) return LINEAR_ENULL;
  if (n_layers < 1 || n_pairs < 1 || rows < 1 || pitch_rows < rows || row_bytes < 16 || row_bytes % 16)
    return LINEAR_EINVAL;
  for (int32_t l = 0; l < n_layers; ++l) {
    if (!k_cache[l] || !v_cache[l]) return LINEAR_ENULL;
    if (misaligned(k_cache[l]) || misaligned(v_cache[l])) return LINEAR_EALIGN;
  }
  for (int32_t l = 0; l < n_layers; ++l) {
    const hipError_t e = linear::launch_stream_read(k_cache[l], v_cache[l], n_pairs, rows, pitch_rows, row_bytes,
                                                    nullptr, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
  }
  return LINEAR_OK;
}

int linear_probe_empty(int32_t launches, int32_t groups, int32_t threads, void* stream) {
  if (launches < 0 || groups < 1 || threads < 1 || threads > 1024) return LINEAR_EINVAL;
  for (int32_t i = 0; i < launches; ++i) {
    const hipError_t e = linear::launch_empty(groups, threads, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
  }
  return LINEAR_OK;
}

int linear_static_scratch_bytes(size_t* bytes) {
  if (!bytes) return LINEAR_ENULL;
  void* base = nullptr;
  const hipError_t e = static_scratch_ptr(&base);
  if (e != hipSuccess) return hip_fail(e);
  *bytes = kStaticScratchBytes;
  return LINEAR_OK;
}

int decode_step_static(int32_t dtype, int32_t head_dim, int32_t n_pairs, int32_t cached_keys,
                       int32_t cache_pitch, void* k_cache, void* v_cache, const void* q, const void* k,
                       const void* v, float scale, int32_t n_split, void* out, void* stream) {
  if (!k_cache || !v_cache || !q || !k || !v || !out) return LINEAR_ENULL;
  if (dtype != LINEAR_F32 && dtype != LINEAR_BF16) return LINEAR_EINVAL;
  if (head_dim != 64 && head_dim != 128) return LINEAR_EINVAL;
  if (n_pairs < 1 || n_pairs > (1 << 24) || cached_keys < 0 || cache_pitch <= cached_keys ||
      cache_pitch > (1 << 20))
    return LINEAR_EINVAL;
  if (!(scale >= 0.f) || std::isinf(scale)) return LINEAR_EINVAL;
  if (n_split < 0 || n_split > linear::kMaxSplit) return LINEAR_EINVAL;
  if (misaligned(k_cache) || misaligned(v_cache) || misaligned(q) || misaligned(k) || misaligned(v) ||
      misaligned(out))
    return LINEAR_EALIGN;
  Plan plan;
  if (!make_plan(dtype, head_dim, n_pairs, false, 0, n_split, cached_keys, &plan)) return LINEAR_EINVAL;
  // split partials: numerators [P, n_split, d], then (max, sum) [P, n_split, 2]
  const size_t part_o_bytes = align_up((size_t)n_pairs * plan.n_split * head_dim * sizeof(float));
  const size_t part_ml_bytes = (size_t)n_pairs * plan.n_split * 2 * sizeof(float);
  if (plan.n_split > 1 && part_o_bytes + part_ml_bytes > kStaticScratchBytes) return LINEAR_ECAPACITY;
  void* base = nullptr;
  hipError_t e = static_scratch_ptr(&base);
  if (e != hipSuccess) return hip_fail(e);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int row_bytes = head_dim * (dtype == LINEAR_BF16 ? 2 : 4);
  if (cached_keys == 0) {
    // with an empty cache the step's masked loads touch row 0: give it defined bits
    e = linear::launch_zero_rows(k_cache, cache_pitch, 1, n_pairs, row_bytes, s);
    if (e == hipSuccess) e = linear::launch_zero_rows(v_cache, cache_pitch, 1, n_pairs, row_bytes, s);
    if (e != hipSuccess) return hip_fail(e);
  }
  linear::DecodeArgs a = {};
  a.q = q;
  a.k_new = k;
  a.v_new = v;
  a.kc = k_cache;
  a.vc = v_cache;
  a.out = out;
  a.part_o = reinterpret_cast<float*>(base);
  a.part_ml = reinterpret_cast<float*>(static_cast<char*>(base) + part_o_bytes);
  a.n_pairs = n_pairs;
  a.t = cached_keys + 1;
  a.t_max = cache_pitch;
  a.n_split = plan.n_split;
  a.rows_per_split = plan.rows_per_split;
  a.n_waves = plan.n_waves;
  a.new_wave = plan.new_wave;
  a.depth = plan.depth;
  a.max_split = plan.n_split;
  const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)head_dim);
  a.scale_log2e = sc * 1.4426950408889634f;
  e = linear::launch_decode(a, dtype, head_dim, s);
  if (e != hipSuccess) return hip_fail(e);
  return LINEAR_OK;
}

const char* linear_strerror(int code) {
  switch (code) {
    case LINEAR_OK: return "ok";
    case LINEAR_EINVAL: return "invalid configuration or argument";
    case LINEAR_ESTATE: return "call not allowed in the layer's current state";
    case LINEAR_ENULL: return "required pointer is NULL";
    case LINEAR_EALIGN: return "device pointer is not 16-byte aligned";
    case LINEAR_EHIP: return "HIP call failed";
    case LINEAR_ECAPACITY: return "the step's split partials exceed the library's static scratch";
    default: return "unknown error";
  }
}

int linear_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"

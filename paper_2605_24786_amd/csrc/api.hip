// Host side of the C ABI declared in include/conf_kv.h: argument validation, the layout of
// the caller's device buffers, per-layer host bookkeeping (upper bounds of the lengths,
// next position, pending appends, arrival-counter bases) and kernel launches.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "conf_kv.h"
#include "confkv_dev.h"
#include "launch.h"

using namespace confkv;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct StateLayout {
  size_t len, n8, head16, head8, budget, n_tight, n_loose, stats, unit_evicted, unit_demoted, unit_moved, ctl, pt, ema, pos, ks, vs, k8, v8, k16, v16, total;
  int npages;            // paged layout: physical pages per unit (0 otherwise)
  size_t header_bytes;   // [0, header_bytes) is zeroed at create
  int cap8, cap16;
};

struct ScratchLayout {
  size_t conf_partial, part_ml, part_o, spill, score, src, sel, shared, total;
  size_t zero_bytes;     // [0, zero_bytes) holds the counters and is zeroed at create
};

// FP16 ring rows of a mixed cache: the window plus the appended tokens, in whole 16-row tiles.
int fp16_ring_rows(const conf_kv_config *c) {
  const long long want = ((long long)c->fp16_window + std::max(1, c->max_chunk) + 15) / 16 * 16;
  return (int)std::min<long long>(want, c->capacity);
}
// Paged layout: INT8 rows in whole pages below the rows that hold the FP16 slots' metadata.
int paged_rows(const conf_kv_config *c) {
  return (c->capacity - fp16_ring_rows(c)) / c->evict_page * c->evict_page;
}

bool config_ok(const conf_kv_config *c) {
  if (!c || !c->n_tight || !c->n_loose) return false;
  if (c->n_layers < 1 || c->n_layers > kMaxLayers || c->batch < 1) return false;
  if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads) return false;
  if (!attend_supported(c->head_dim, c->n_q_heads / c->n_kv_heads)) return false;
  if (c->vocab < 2) return false;
  if (c->capacity < 16 || c->capacity % 16) return false;
  if (c->protected_window < 0) return false;
  if (!(c->alpha >= 0.f && c->alpha <= 1.f)) return false;
  if (!(c->ema_decay >= 0.f && c->ema_decay <= 1.f)) return false;
  if (!(c->sm_scale > 0.f)) return false;
  if (!(c->mass_gain < 0.f) && !(c->mass_gain >= 0.f && c->mass_gain <= 1.0e6f)) return false;   // NaN
  if (c->ranker != CONF_KV_RANKER_COMPOSITE && c->ranker != CONF_KV_RANKER_RANDOM) return false;
  if (c->rank_scope != CONF_KV_SCOPE_KV_HEAD && c->rank_scope != CONF_KV_SCOPE_LAYER) return false;
  if (c->scale_mode != CONF_KV_SCALES_TOKEN && c->scale_mode != CONF_KV_SCALES_CHANNEL) return false;
  if (c->scale_mode == CONF_KV_SCALES_CHANNEL && (c->head_dim != 128 || c->fp16_window < 0)) return false;
  if (c->max_chunk < 0) return false;
  // multi-token calls: one tile of 16 query rows per unit, or up to kWideRowsMax rows on the
  // many-rows kernel (per-token scales only)
  if (c->max_chunk > 1) {
    const int rows = c->max_chunk * (c->n_q_heads / c->n_kv_heads);
    if (c->head_dim != 128 || rows > kWideRowsMax) return false;
    if (rows > kChunkRows && c->scale_mode != CONF_KV_SCALES_TOKEN) return false;
  }
  if (c->evict_page < 0 || c->evict_page > 1024) return false;
  if (c->layout != CONF_KV_LAYOUT_CONTIGUOUS && c->layout != CONF_KV_LAYOUT_PAGED) return false;
  if (c->layout == CONF_KV_LAYOUT_PAGED) {
    const int g = c->evict_page, G = c->n_q_heads / c->n_kv_heads;
    if (g < 8 || (g & (g - 1))) return false;                      // a power of two, 8 .. 1024
    if (c->fp16_window < 0 || c->fp16_window > c->protected_window) return false;
    if (c->scale_mode != CONF_KV_SCALES_TOKEN || c->rank_scope != CONF_KV_SCOPE_KV_HEAD) return false;
    if (c->max_chunk > 1 || G < 2 || G > 8) return false;
  }
  const int page_slack = c->evict_page > 1 ? c->evict_page - 1 : 0;   // slots a page in the window can hold back
  for (int l = 0; l < c->n_layers; ++l) {
    if (c->n_tight[l] < 1 || c->n_tight[l] > c->n_loose[l]) return false;
    if (std::max((long long)c->n_loose[l], (long long)c->protected_window + page_slack) + std::max(1, c->max_chunk) >
        c->capacity)
      return false;
    // paged: the whole pages below the FP16 slots' metadata rows must hold the longest INT8 part
    if (c->layout == CONF_KV_LAYOUT_PAGED &&
        std::max((long long)c->n_loose[l], (long long)c->protected_window + page_slack) + 1 >
            (long long)paged_rows(c))
      return false;
  }
  return true;
}

StateLayout state_layout(const conf_kv_config *c) {
  StateLayout s{};
  const size_t U = (size_t)c->n_layers * c->batch * c->n_kv_heads;
  const size_t cap = c->capacity, D = c->head_dim;
  s.cap8 = c->fp16_window < 0 ? 0 : c->capacity;
  s.cap16 = c->fp16_window < 0 ? c->capacity : fp16_ring_rows(c);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  s.len = take(U * 4);
  s.n8 = take(U * 4);
  s.head16 = take(U * 4);
  s.head8 = take(U * 4);
  s.stats = take(kStatSlots * 8);
  s.unit_evicted = take(U * 4);
  s.unit_demoted = take(U * 4);
  s.unit_moved = take(U * 8);
  s.ctl = take((size_t)(kCtlPos + c->n_layers) * 4);
  s.header_bytes = off;
  s.budget = take((size_t)c->n_layers * c->batch * 4);
  s.n_tight = take((size_t)c->n_layers * 4);
  s.n_loose = take((size_t)c->n_layers * 4);
  s.npages = c->layout == CONF_KV_LAYOUT_PAGED ? paged_rows(c) / c->evict_page : 0;
  s.pt = take(U * (size_t)s.npages * 4);
  s.ema = take(U * cap * 4);
  s.pos = take(U * cap * 4);
  // per-token scales [U][cap8], or per-channel scales [U][D]
  const size_t scales = c->scale_mode == CONF_KV_SCALES_CHANNEL ? D : (size_t)s.cap8;
  s.ks = take(U * scales * 2);
  s.vs = take(U * scales * 2);
  s.k8 = take(U * s.cap8 * D);
  s.v8 = take(U * s.cap8 * D);
  s.k16 = take(U * s.cap16 * D * 2);
  s.v16 = take(U * s.cap16 * D * 2);
  s.total = off;
  return s;
}

ScratchLayout scratch_layout(const conf_kv_config *c) {
  ScratchLayout s{};
  const size_t UPL = (size_t)c->batch * c->n_kv_heads, U = UPL * c->n_layers;
  const size_t G = c->n_q_heads / c->n_kv_heads, D = c->head_dim;
  const size_t R = (c->max_chunk > 1 || G > 8) ? (size_t)kChunkRows : G;   // query rows per unit in the exchange buffers
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  s.conf_partial = take(conf_reduce_scratch_bytes(c->batch, c->vocab));
  // epoch-tagged (m, l) words of the splits: tags start at 0, which no launch uses
  s.part_ml = take(UPL * kAttendMaxSplits * R * 2 * 8);
  // (the matrix-core body exchanges 128-channel partials whatever the head dimension)
  s.part_o = take(UPL * kAttendMaxSplits * R * std::max<size_t>(D, 128) * 8);
  s.zero_bytes = off;
  s.spill = take(attend_spill_floats((int)UPL, (int)R, c->capacity) * 4);
  s.score = take(U * c->capacity * 8);
  s.src = take(U * c->capacity * 4);
  s.sel = take(U * kSelInts * 4);
  s.shared = take(c->rank_scope == CONF_KV_SCOPE_LAYER ? (size_t)c->n_layers * c->batch * c->capacity * 8 : 0);
  s.total = off;
  return s;
}

}  // namespace

struct conf_kv_handle {
  conf_kv_config cfg;
  std::vector<int32_t> n_tight, n_loose;
  StateLayout sl;
  ScratchLayout kl;
  uint8_t *state = nullptr;
  uint8_t *scratch = nullptr;
  CacheView cv{};
  // per layer
  std::vector<int32_t> len_ub;       // upper bound of the committed length
  std::vector<uint8_t> appended;     // an append awaits its commit
  std::vector<uint8_t> scaled;       // per unit: channel scales were given (channel mode)
  std::vector<int32_t> fresh_len;    // per layer: T0 of a prompt no decode step has touched yet, else -1
  // Launches since the last commit (conf_kv_evict_compact).  The tag of the words a launch
  // publishes is this number plus a base on the device that the commit advances, and the
  // position of the next appended token lives on the device too: no launch argument changes
  // from one decode step to the next, so a recorded step can be replayed.
  uint32_t attend_launches = 0;
  uint32_t conf_launches = 0;
  bool prompt_loaded = false;        // conf_kv_load_prefill / conf_kv_import since the last commit
  bool static_plan = false;          // conf_kv_static_plan: launch shapes from the budgets, not the lengths so far
  int forced_splits = 0;            // CONF_KV_SPLITS at create (tests, sweeps)
  bool force_two_launch = false;    // CONF_KV_TWO_LAUNCH at create (tests)
  int withhold = 0;                 // CONF_KV_TEST_WITHHOLD at create (tests of the expiry path)
  int kv_major = 0;                 // splits of a unit on one XCD (eight kv-heads or a multiple; CONF_KV_GRID_KV_MAJOR overrides)
  int spin_limit = kSpinLimitDefault;   // CONF_KV_SPIN_LIMIT at create (tests of the expiry path)
  int last_hip = 0;
};

#define CK_HIP(h, expr)                         \
  do {                                          \
    hipError_t e_ = (expr);                     \
    if (e_ != hipSuccess) {                     \
      if (h) (h)->last_hip = (int)e_;           \
      return CONF_KV_ERR_HIP;                   \
    }                                           \
  } while (0)

extern "C" {

size_t conf_kv_state_bytes(const conf_kv_config *cfg) {
  return config_ok(cfg) ? state_layout(cfg).total : 0;
}

size_t conf_kv_scratch_bytes(const conf_kv_config *cfg) {
  return config_ok(cfg) ? scratch_layout(cfg).total : 0;
}

int conf_kv_create(conf_kv_handle **out, const conf_kv_config *cfg, void *dev_state,
                   void *dev_scratch) {
  if (!out) return CONF_KV_ERR_INVALID_ARG;
  *out = nullptr;
  if (!cfg || !dev_state || !dev_scratch || !cfg->n_tight || !cfg->n_loose)
    return CONF_KV_ERR_INVALID_ARG;
  if (((uintptr_t)dev_state % kAlign) || ((uintptr_t)dev_scratch % kAlign))
    return CONF_KV_ERR_INVALID_ARG;
  if (!config_ok(cfg)) return CONF_KV_ERR_BAD_SHAPE;
  conf_kv_handle *h = new (std::nothrow) conf_kv_handle();
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  h->cfg = *cfg;
  h->n_tight.assign(cfg->n_tight, cfg->n_tight + cfg->n_layers);
  h->n_loose.assign(cfg->n_loose, cfg->n_loose + cfg->n_layers);
  h->cfg.n_tight = h->n_tight.data();
  h->cfg.n_loose = h->n_loose.data();
  h->sl = state_layout(&h->cfg);
  h->kl = scratch_layout(&h->cfg);
  h->state = (uint8_t *)dev_state;
  h->scratch = (uint8_t *)dev_scratch;
  const int L = cfg->n_layers;
  h->len_ub.assign(L, 0);
  h->appended.assign(L, 0);
  h->scaled.assign((size_t)L * cfg->batch * cfg->n_kv_heads, 0);
  h->fresh_len.assign(L, -1);
  if (const char *fs = getenv("CONF_KV_SPLITS")) h->forced_splits = atoi(fs);
  if (const char *tl = getenv("CONF_KV_TWO_LAUNCH")) h->force_two_launch = atoi(tl) != 0;
  if (const char *wh = getenv("CONF_KV_TEST_WITHHOLD")) h->withhold = atoi(wh) != 0;
  h->kv_major = cfg->n_kv_heads % 8 == 0;
  if (const char *km = getenv("CONF_KV_GRID_KV_MAJOR")) h->kv_major = atoi(km) != 0;
  if (const char *sp = getenv("CONF_KV_SPIN_LIMIT")) h->spin_limit = std::max(0, atoi(sp));

  CacheView &cv = h->cv;
  uint8_t *s = h->state;
  cv.k8 = (int8_t *)(s + h->sl.k8);
  cv.v8 = (int8_t *)(s + h->sl.v8);
  cv.ks = (__half *)(s + h->sl.ks);
  cv.vs = (__half *)(s + h->sl.vs);
  cv.k16 = (__half *)(s + h->sl.k16);
  cv.v16 = (__half *)(s + h->sl.v16);
  cv.ema = (float *)(s + h->sl.ema);
  cv.pos = (int32_t *)(s + h->sl.pos);
  cv.len = (int32_t *)(s + h->sl.len);
  cv.n8 = (int32_t *)(s + h->sl.n8);
  cv.head16 = (int32_t *)(s + h->sl.head16);
  cv.head8 = (int32_t *)(s + h->sl.head8);
  cv.budget = (int32_t *)(s + h->sl.budget);
  cv.n_tight = (const int32_t *)(s + h->sl.n_tight);
  cv.n_loose = (const int32_t *)(s + h->sl.n_loose);
  cv.stats = (unsigned long long *)(s + h->sl.stats);
  cv.unit_evicted = (unsigned *)(s + h->sl.unit_evicted);
  cv.unit_demoted = (unsigned *)(s + h->sl.unit_demoted);
  cv.unit_moved = (unsigned long long *)(s + h->sl.unit_moved);
  cv.L = L;
  cv.B = cfg->batch;
  cv.Hkv = cfg->n_kv_heads;
  cv.G = cfg->n_q_heads / cfg->n_kv_heads;
  cv.D = cfg->head_dim;
  cv.cap = cfg->capacity;
  cv.cap8 = h->sl.cap8;
  cv.cap16 = h->sl.cap16;
  cv.W = cfg->fp16_window;
  cv.P = cfg->protected_window;
  cv.chan = cfg->scale_mode == CONF_KV_SCALES_CHANNEL;
  cv.ctl = (unsigned *)(s + h->sl.ctl);
  cv.tagged = (unsigned long long *)(h->scratch + h->kl.conf_partial);
  cv.n_tagged = (h->kl.zero_bytes - h->kl.conf_partial) / 8;
  cv.pt = (int32_t *)(s + h->sl.pt);
  cv.npages = h->sl.npages;
  cv.page_lg = 0;
  if (cfg->layout == CONF_KV_LAYOUT_PAGED)
    while ((1 << cv.page_lg) < cfg->evict_page) ++cv.page_lg;

  std::vector<int32_t> budget((size_t)L * cfg->batch);
  for (int l = 0; l < L; ++l)
    for (int b = 0; b < cfg->batch; ++b) budget[(size_t)l * cfg->batch + b] = h->n_loose[l];
  // the library's own device array (conf_kv_step_static): resolve its address on this device now
  hipError_t e = conf_reduce_static_setup();
  if (e == hipSuccess) e = hipMemset(h->state, 0, h->sl.header_bytes);
  if (e == hipSuccess) e = hipMemset(h->scratch, 0, h->kl.zero_bytes);
  if (e == hipSuccess && cv.chan)      // attention reads the channel scales even before any slot is INT8
    e = hipMemset(cv.ks, 0, (size_t)((uint8_t *)cv.k8 - (uint8_t *)cv.ks));
  if (e == hipSuccess && cv.npages > 0) {              // every unit's block table starts as the identity
    const size_t U = (size_t)L * cfg->batch * cfg->n_kv_heads;
    std::vector<int32_t> ident(U * cv.npages);
    for (size_t i = 0; i < ident.size(); ++i) ident[i] = (int32_t)(i % cv.npages);
    e = hipMemcpy(cv.pt, ident.data(), ident.size() * 4, hipMemcpyHostToDevice);
  }
  if (const char *tb = getenv("CONF_KV_TEST_TAG_BASE")) {   // test hook: start the tag bases near their restart
    const unsigned base[2] = {(unsigned)strtoul(tb, nullptr, 0), (unsigned)strtoul(tb, nullptr, 0)};
    if (e == hipSuccess) e = hipMemcpy(cv.ctl + kCtlTag, base, sizeof base, hipMemcpyHostToDevice);
  }
  if (e == hipSuccess) e = hipMemcpy(cv.budget, budget.data(), budget.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy((void *)cv.n_tight, h->n_tight.data(), (size_t)L * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy((void *)cv.n_loose, h->n_loose.data(), (size_t)L * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    delete h;
    return CONF_KV_ERR_HIP;
  }
  *out = h;
  return CONF_KV_OK;
}

int conf_kv_pyramid_budgets(int32_t n0, int32_t n_layers, double beta, int32_t n_min,
                            int32_t *host_out) {
  if (!host_out || n_layers < 1 || n0 < 1 || n_min < 1 || !(beta > 0.0 && beta <= 1.0))
    return CONF_KV_ERR_INVALID_ARG;
  for (int l = 0; l < n_layers; ++l) {
    const double v = floor((double)n0 * pow(beta, (double)l / (double)n_layers));
    host_out[l] = std::max<int32_t>(n_min, (int32_t)v);
  }
  return CONF_KV_OK;
}

int conf_kv_destroy(conf_kv_handle *h) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  delete h;
  return CONF_KV_OK;
}

int conf_kv_load_prefill(conf_kv_handle *h, int32_t layer, const void *dev_k16, const void *dev_v16,
                         int32_t T0, const float *dev_ema0, conf_kv_stream stream) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= h->cfg.n_layers) return CONF_KV_ERR_BAD_LAYER;
  if (T0 < 0) return CONF_KV_ERR_INVALID_ARG;
  if (T0 > 0 && (!dev_k16 || !dev_v16)) return CONF_KV_ERR_INVALID_ARG;
  if (((uintptr_t)dev_k16 | (uintptr_t)dev_v16) & 15) return CONF_KV_ERR_INVALID_ARG;   // rows are read in 16-byte pieces
  if (T0 > h->cfg.capacity - 1) return CONF_KV_ERR_CAPACITY;
  if (h->cv.page_lg && T0 - h->cfg.fp16_window > (h->cv.npages << h->cv.page_lg)) return CONF_KV_ERR_CAPACITY;
  CK_HIP(h, launch_load_prefill(h->cv, layer, (const __half *)dev_k16, (const __half *)dev_v16, T0,
                                dev_ema0, (hipStream_t)stream));
  h->len_ub[layer] = T0;
  h->prompt_loaded = true;
  h->appended[layer] = 0;
  const size_t UPL = (size_t)h->cfg.batch * h->cfg.n_kv_heads;
  std::fill(h->scaled.begin() + layer * UPL, h->scaled.begin() + (layer + 1) * UPL, (uint8_t)1);
  h->fresh_len[layer] = T0;
  return CONF_KV_OK;
}

// Upper bound of a layer's committed length that the launch shapes are derived from: what the
// host has seen so far, or (conf_kv_static_plan) what the budgets allow at any later step too.
static int length_bound(const conf_kv_handle *h, int layer) {
  return h->static_plan ? std::max(h->len_ub[layer], h->n_loose[layer]) : h->len_ub[layer];
}

// LDS the attention kernel needs for the unit's block table (paged layout), in whole 16 bytes.
static size_t table_lds(const conf_kv_handle *h) {
  return h->cv.page_lg ? ((size_t)h->cv.npages * 4 + 15) / 16 * 16 : 0;
}

static int plan_for_layer(conf_kv_handle *h, int layer, int tq, AttendPlan *plan, int observe_first = -1) {
  const bool observe = observe_first >= 0;
  const int n_ub = observe ? observe_first + tq : length_bound(h, layer) + tq;     // slots the call sees
  const int W = h->cfg.fp16_window;
  const int n16_ub = W < 0 ? n_ub : std::min(n_ub, observe ? W : W + tq);
  // a chunk runs on the matrix-core body with all 16 tile rows as query rows
  if (tq * h->cv.G > kChunkRows) {                         // more rows than one tile: the many-rows kernel
    if (!attend_wide_plan(tq * h->cv.G, h->cfg.batch * h->cfg.n_kv_heads, n_ub, h->forced_splits, plan))
      return CONF_KV_ERR_BAD_SHAPE;
    return CONF_KV_OK;
  }
  const bool rows16 = tq > 1 || observe || h->cv.G > 8;
  const int rows = rows16 ? kChunkRows : h->cv.G;
  if (!attend_plan(h->cfg.head_dim, rows, h->cv.chan != 0, rows16, h->cfg.batch * h->cfg.n_kv_heads, n_ub, n16_ub,
                   h->forced_splits, h->force_two_launch, table_lds(h), plan))
    return CONF_KV_ERR_BAD_SHAPE;
  // the paged layout is read by the single-launch matrix-core kernel only
  if (h->cv.page_lg && (plan->two_launch || !plan->mfma)) return CONF_KV_ERR_BAD_SHAPE;
  return CONF_KV_OK;
}

// observe_first < 0: append tq tokens and attend; >= 0: conf_kv_observe
static int attend_tokens(conf_kv_handle *h, int32_t layer, int32_t tq, const void *dev_q16,
                         const void *dev_knew16, const void *dev_vnew16, void *dev_out16,
                         conf_kv_stream stream, int32_t observe_first = -1, int32_t q_tokens = 0) {
  const bool observe = observe_first >= 0;
  if (!h || !dev_q16) return CONF_KV_ERR_INVALID_ARG;
  if (!observe && (!dev_knew16 || !dev_vnew16 || !dev_out16)) return CONF_KV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= h->cfg.n_layers) return CONF_KV_ERR_BAD_LAYER;
  if (tq < 1 || tq > std::max(1, h->cfg.max_chunk)) return CONF_KV_ERR_INVALID_ARG;
  if (observe) {
    // (the call runs on the 16-row kernel: the exchange buffers must have been sized for it)
    if (h->cfg.max_chunk < 2 && h->cv.G <= 8) return CONF_KV_ERR_INVALID_ARG;
    if (h->appended[layer] || h->fresh_len[layer] < 0) return CONF_KV_ERR_BAD_STATE;
    if ((long long)observe_first + tq > h->fresh_len[layer]) return CONF_KV_ERR_INVALID_ARG;
  }
  if (((uintptr_t)dev_q16 | (uintptr_t)dev_knew16 | (uintptr_t)dev_vnew16 | (uintptr_t)dev_out16) & 15)
    return CONF_KV_ERR_INVALID_ARG;
  if (h->appended[layer]) return CONF_KV_ERR_BAD_STATE;
  if (!observe && h->len_ub[layer] + tq > h->cfg.capacity) return CONF_KV_ERR_CAPACITY;
  AttendPlan plan;
  int rc = plan_for_layer(h, layer, tq, &plan, observe_first);
  if (rc != CONF_KV_OK) return rc;
  [[maybe_unused]] const size_t UPL = (size_t)h->cfg.batch * h->cfg.n_kv_heads;   // phase-trace builds
  AttendLaunch a{};
  a.layer = layer;
  a.q = (const __half *)dev_q16;
  a.knew = (const __half *)dev_knew16;
  a.vnew = (const __half *)dev_vnew16;
  a.out = (__half *)dev_out16;
  a.part_ml = (unsigned long long *)(h->scratch + h->kl.part_ml);
  a.part_o = (unsigned long long *)(h->scratch + h->kl.part_o);
  a.spill = (float *)(h->scratch + h->kl.spill);
  // One numbering for the handle: the tagged words are shared by the layers, so a launch must not
  // meet a tag a launch on another layer left.  The words start at 0 and numbers start at 1, so
  // tag 0 is never used; before the device-side base nears the end of its range the commit has
  // the words cleared and starts over (evict.hip).
  if (h->attend_launches >= kTagLaunchesMax) return CONF_KV_ERR_BAD_STATE;
  a.epoch = ++h->attend_launches;
  a.spin_limit = h->spin_limit;
  a.max_splits = kAttendMaxSplits;
  a.sm_scale = h->cfg.sm_scale;
  a.ema_decay = h->cfg.ema_decay;
  a.mass_gain = h->cfg.mass_gain < 0.f ? 1.0 - (double)h->cfg.ema_decay : (double)h->cfg.mass_gain;
  a.pos_new = 0;                                   // read on the device
  a.tq = tq;
  a.q_tokens = q_tokens > 0 ? q_tokens : tq;
  a.gq = h->cv.G;
  a.observe_first = observe_first;
  a.kv_major = h->kv_major;
  a.tab_off = (int)(plan.lds_bytes - table_lds(h));
  a.trace_off = 0;
  a.withhold = h->withhold;
  a.dbg = nullptr;
#ifdef CONFKV_TRACE
  // the ranking work arrays at the end of the scratch buffer are idle during conf_kv_attend
  // (4 MB when they are that large, else 256 KB: enough for 128 workgroups)
  if (getenv("CONF_KV_TRACE")) {
    const size_t big = (size_t)8 * 32 * 4 * 4096, small = (size_t)8 * 32 * 8 * 128;
    const size_t have = h->kl.total - h->kl.score;
    const size_t need = (size_t)8 * 32 * 8 * plan.splits * UPL;
    const size_t region = have >= big ? big : small;
    if (have >= region && need <= region) a.dbg = (unsigned long long *)(h->scratch + h->kl.total - region);
  }
#endif
  CK_HIP(h, launch_attend(h->cv, a, plan, (hipStream_t)stream));
  if (!observe) {
    h->appended[layer] = (uint8_t)tq;
    h->fresh_len[layer] = -1;
  }
  return CONF_KV_OK;
}

int conf_kv_attend(conf_kv_handle *h, int32_t layer, const void *dev_q16, const void *dev_knew16,
                   const void *dev_vnew16, void *dev_out16, conf_kv_stream stream) {
  return attend_tokens(h, layer, 1, dev_q16, dev_knew16, dev_vnew16, dev_out16, stream);
}

int conf_kv_attend_chunk(conf_kv_handle *h, int32_t layer, int32_t tq, const void *dev_q16,
                         const void *dev_knew16, const void *dev_vnew16, void *dev_out16,
                         conf_kv_stream stream) {
  return attend_tokens(h, layer, tq, dev_q16, dev_knew16, dev_vnew16, dev_out16, stream);
}

int conf_kv_observe(conf_kv_handle *h, int32_t layer, int32_t first, int32_t tq, const void *dev_q16,
                    void *dev_out16, conf_kv_stream stream) {
  if (first < 0) return CONF_KV_ERR_INVALID_ARG;
  return attend_tokens(h, layer, tq, dev_q16, nullptr, nullptr, dev_out16, stream, first);
}

int conf_kv_observe_prompt(conf_kv_handle *h, int32_t layer, const void *dev_q16, conf_kv_stream stream) {
  if (!h || !dev_q16) return CONF_KV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= h->cfg.n_layers) return CONF_KV_ERR_BAD_LAYER;
  if (h->appended[layer] || h->fresh_len[layer] < 0) return CONF_KV_ERR_BAD_STATE;
  const int T0 = h->fresh_len[layer], step = std::max(1, h->cfg.max_chunk);
  const size_t tok = (size_t)h->cfg.n_q_heads * h->cfg.head_dim;          // elements of one token's queries
  for (int first = 0; first < T0; first += step) {
    const int tq = std::min(step, T0 - first);
    int rc = attend_tokens(h, layer, tq, (const __half *)dev_q16 + (size_t)first * tok, nullptr, nullptr, nullptr,
                           stream, first, T0);
    if (rc != CONF_KV_OK) return rc;
  }
  return CONF_KV_OK;
}

int conf_kv_attend_splits(conf_kv_handle *h, int32_t layer) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= h->cfg.n_layers) return CONF_KV_ERR_BAD_LAYER;
  AttendPlan plan;
  int rc = plan_for_layer(h, layer, 1, &plan);
  if (rc != CONF_KV_OK) return rc;
  return plan.two_launch ? 1000 + plan.splits : plan.splits;
}

int conf_kv_step(conf_kv_handle *h, const float *dev_logits, float *dev_conf, uint8_t *dev_sel,
                 conf_kv_stream stream) {
  if (!h || !dev_logits) return CONF_KV_ERR_INVALID_ARG;
  if (h->conf_launches >= kTagLaunchesMax) return CONF_KV_ERR_BAD_STATE;    // (numbered like the attention launches)
  CK_HIP(h, launch_conf_reduce(h->cv, dev_logits, h->cfg.vocab,
                               (unsigned long long *)(h->scratch + h->kl.conf_partial),
                               ++h->conf_launches, 1, h->spin_limit, h->withhold, dev_conf, dev_sel,
                               (double)h->cfg.tau, (double)h->cfg.w_entropy, (double)h->cfg.w_margin,
                               (double)h->cfg.w_top, (hipStream_t)stream));
  return CONF_KV_OK;
}

int conf_kv_step_static(conf_kv_handle *h, const float *dev_logits, float *dev_conf, uint8_t *dev_sel,
                        conf_kv_stream stream) {
  if (!h || !dev_logits) return CONF_KV_ERR_INVALID_ARG;
  if (conf_reduce_scratch_bytes(h->cfg.batch, h->cfg.vocab) > kConfStaticBytes) return CONF_KV_ERR_CAPACITY;
  CK_HIP(h, launch_conf_reduce_static(h->cv, dev_logits, h->cfg.vocab, h->spin_limit, h->withhold, dev_conf, dev_sel,
                                      (double)h->cfg.tau, (double)h->cfg.w_entropy, (double)h->cfg.w_margin,
                                      (double)h->cfg.w_top, (hipStream_t)stream));
  return CONF_KV_OK;
}

int conf_kv_evict_compact(conf_kv_handle *h, conf_kv_stream stream) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  LayerMask m{};
  int n_max = 0;
  const size_t UPL = (size_t)h->cfg.batch * h->cfg.n_kv_heads;
  for (int l = 0; l < h->cfg.n_layers; ++l) {
    m.set(l, h->appended[l]);
    n_max = std::max(n_max, length_bound(h, l) + (int)h->appended[l]);
    if (h->cv.chan && h->len_ub[l] + (int)h->appended[l] > 0)     // a demotion needs the scales
      for (size_t u = l * UPL; u < (l + 1) * UPL; ++u)
        if (!h->scaled[u]) return CONF_KV_ERR_BAD_STATE;
  }
  RankOptions opt{};
  opt.random = h->cfg.ranker == CONF_KV_RANKER_RANDOM;
  opt.seed = h->cfg.ranker_seed;
  opt.shared = h->cfg.rank_scope == CONF_KV_SCOPE_LAYER ? (double *)(h->scratch + h->kl.shared) : nullptr;
  opt.page = h->cfg.evict_page > 1 ? h->cfg.evict_page : 0;
  CK_HIP(h, launch_evict_compact(h->cv, m, (double)h->cfg.alpha, opt, (double *)(h->scratch + h->kl.score),
                                 (int32_t *)(h->scratch + h->kl.src),
                                 (int32_t *)(h->scratch + h->kl.sel), n_max, h->attend_launches, h->conf_launches,
                                 h->prompt_loaded, (hipStream_t)stream));
  h->attend_launches = h->conf_launches = 0;
  h->prompt_loaded = false;
  const int P = h->cfg.protected_window;
  for (int l = 0; l < h->cfg.n_layers; ++l) {
    h->len_ub[l] += h->appended[l];
    h->appended[l] = 0;
    h->fresh_len[l] = -1;
    // any budget the step may have chosen is at most the loose one
    const int n = h->len_ub[l], NL = h->n_loose[l];
    // (a page that reaches into the protected window holds back up to evict_page - 1 more)
    if (n > NL) h->len_ub[l] = std::max(NL, std::min(P + (opt.page > 1 ? opt.page - 1 : 0), n));
  }
  return CONF_KV_OK;
}

int conf_kv_static_plan(conf_kv_handle *h, int32_t on) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  h->static_plan = on != 0;
  return CONF_KV_OK;
}

int conf_kv_tag_state(conf_kv_handle *h, uint32_t *attend_base, uint32_t *conf_base, int32_t *clear_pending) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  unsigned ctl[kCtlPos] = {};
  CK_HIP(h, hipDeviceSynchronize());
  CK_HIP(h, hipMemcpy(ctl, h->cv.ctl, sizeof ctl, hipMemcpyDeviceToHost));
  if (attend_base) *attend_base = ctl[kCtlTag];
  if (conf_base) *conf_base = ctl[kCtlConfTag];
  if (clear_pending) *clear_pending = (int32_t)ctl[kCtlClear];
  return CONF_KV_OK;
}

int conf_kv_lengths(conf_kv_handle *h, int32_t *host_len, int32_t *host_n16) {
  if (!h || !host_len) return CONF_KV_ERR_INVALID_ARG;
  const int L = h->cfg.n_layers, B = h->cfg.batch, H = h->cfg.n_kv_heads;
  const size_t U = (size_t)L * B * H;
  std::vector<int32_t> len(U), n8(U);
  CK_HIP(h, hipDeviceSynchronize());
  CK_HIP(h, hipMemcpy(len.data(), h->cv.len, U * 4, hipMemcpyDeviceToHost));
  CK_HIP(h, hipMemcpy(n8.data(), h->cv.n8, U * 4, hipMemcpyDeviceToHost));
  for (int l = 0; l < L; ++l)
    for (int b = 0; b < B; ++b) {
      const size_t u0 = ((size_t)l * B + b) * H;
      host_len[(size_t)l * B + b] = len[u0] + h->appended[l];
      if (host_n16)
        for (int g = 0; g < H; ++g) host_n16[u0 + g] = len[u0 + g] + h->appended[l] - n8[u0 + g];
    }
  return CONF_KV_OK;
}

int conf_kv_export(conf_kv_handle *h, int32_t layer, int32_t b, int32_t kv_head, int32_t *pos,
                   float *ema, uint8_t *is_fp16, uint16_t *k16, uint16_t *v16, int8_t *k8, int8_t *v8,
                   uint16_t *k_scale, uint16_t *v_scale, int32_t *n_out) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= h->cfg.n_layers) return CONF_KV_ERR_BAD_LAYER;
  if (b < 0 || b >= h->cfg.batch || kv_head < 0 || kv_head >= h->cfg.n_kv_heads)
    return CONF_KV_ERR_INVALID_ARG;
  const CacheView &cv = h->cv;
  const size_t u = ((size_t)layer * cv.B + b) * cv.Hkv + kv_head;
  const size_t D = cv.D;
  CK_HIP(h, hipDeviceSynchronize());
  int32_t len = 0, n8 = 0, head = 0, head8 = 0;
  CK_HIP(h, hipMemcpy(&len, cv.len + u, 4, hipMemcpyDeviceToHost));
  CK_HIP(h, hipMemcpy(&n8, cv.n8 + u, 4, hipMemcpyDeviceToHost));
  CK_HIP(h, hipMemcpy(&head, cv.head16 + u, 4, hipMemcpyDeviceToHost));
  CK_HIP(h, hipMemcpy(&head8, cv.head8 + u, 4, hipMemcpyDeviceToHost));
  const int first8 = std::max(0, std::min(n8, cv.cap8 - head8));   // INT8 ring rows before the wrap
  const int n = len + h->appended[layer];
  const int n16 = n - n8;
  if (n_out) *n_out = n;
  if (cv.chan) {                                      // the unit's channel scales, whatever its length
    if (k_scale) CK_HIP(h, hipMemcpy(k_scale, cv.ks + u * D, D * 2, hipMemcpyDeviceToHost));
    if (v_scale) CK_HIP(h, hipMemcpy(v_scale, cv.vs + u * D, D * 2, hipMemcpyDeviceToHost));
  }
  if (n == 0) return CONF_KV_OK;
  if (cv.page_lg) {
    // Paged layout: the unit's planes come to the host whole and the view is gathered there
    // through the block table (INT8 slots) and the FP16 ring (metadata of the FP16 slots).
    std::vector<int32_t> tab(cv.npages);
    CK_HIP(h, hipMemcpy(tab.data(), cv.pt + u * cv.npages, (size_t)cv.npages * 4, hipMemcpyDeviceToHost));
    const int g = 1 << cv.page_lg;
    auto row_of = [&](int i) {
      if (i < n8) return tab[i >> cv.page_lg] * g + (i & (g - 1));
      int r = head + (i - n8);
      if (r >= cv.cap16) r -= cv.cap16;
      return cv.cap - cv.cap16 + r;
    };
    std::vector<uint8_t> tmp;
    auto gather = [&](const void *dev_plane, size_t row_bytes, void *out, int count) -> hipError_t {
      tmp.resize((size_t)cv.cap * row_bytes);
      hipError_t e = hipMemcpy(tmp.data(), dev_plane, tmp.size(), hipMemcpyDeviceToHost);
      if (e != hipSuccess) return e;
      for (int i = 0; i < count; ++i) memcpy((uint8_t *)out + (size_t)i * row_bytes, tmp.data() + (size_t)row_of(i) * row_bytes, row_bytes);
      return hipSuccess;
    };
    if (pos) CK_HIP(h, gather(cv.pos + u * cv.cap, 4, pos, n));
    if (ema) CK_HIP(h, gather(cv.ema + u * cv.cap, 4, ema, n));
    if (is_fp16)
      for (int i = 0; i < n; ++i) is_fp16[i] = i >= n8;
    if (k8) { CK_HIP(h, gather(cv.k8 + u * cv.cap8 * D, D, k8, n8)); memset(k8 + (size_t)n8 * D, 0, (size_t)n16 * D); }
    if (v8) { CK_HIP(h, gather(cv.v8 + u * cv.cap8 * D, D, v8, n8)); memset(v8 + (size_t)n8 * D, 0, (size_t)n16 * D); }
    if (k_scale) { CK_HIP(h, gather(cv.ks + u * cv.cap8, 2, k_scale, n8)); memset(k_scale + n8, 0, (size_t)n16 * 2); }
    if (v_scale) { CK_HIP(h, gather(cv.vs + u * cv.cap8, 2, v_scale, n8)); memset(v_scale + n8, 0, (size_t)n16 * 2); }
    for (int which = 0; which < 2; ++which) {
      uint16_t *d16 = which ? v16 : k16;
      if (!d16) continue;
      const __half *p16 = (which ? cv.v16 : cv.k16) + u * cv.cap16 * D;
      memset(d16, 0, (size_t)n8 * D * 2);
      if (n16 > 0) {
        const int first = std::min(n16, cv.cap16 - head);
        CK_HIP(h, hipMemcpy(d16 + (size_t)n8 * D, p16 + (size_t)head * D, (size_t)first * D * 2, hipMemcpyDeviceToHost));
        if (n16 > first)
          CK_HIP(h, hipMemcpy(d16 + (size_t)(n8 + first) * D, p16, (size_t)(n16 - first) * D * 2, hipMemcpyDeviceToHost));
      }
    }
    return CONF_KV_OK;
  }
  const int firstm = std::min(n, cv.cap - head8);     // per-slot planes: entries before the wrap
  if (pos) {
    CK_HIP(h, hipMemcpy(pos, cv.pos + u * cv.cap + head8, (size_t)firstm * 4, hipMemcpyDeviceToHost));
    if (n > firstm)
      CK_HIP(h, hipMemcpy(pos + firstm, cv.pos + u * cv.cap, (size_t)(n - firstm) * 4, hipMemcpyDeviceToHost));
  }
  if (ema) {
    CK_HIP(h, hipMemcpy(ema, cv.ema + u * cv.cap + head8, (size_t)firstm * 4, hipMemcpyDeviceToHost));
    if (n > firstm)
      CK_HIP(h, hipMemcpy(ema + firstm, cv.ema + u * cv.cap, (size_t)(n - firstm) * 4, hipMemcpyDeviceToHost));
  }
  if (is_fp16)
    for (int i = 0; i < n; ++i) is_fp16[i] = i >= n8;
  for (int which = 0; which < 2; ++which) {
    uint16_t *d16 = which ? v16 : k16;
    int8_t *d8 = which ? v8 : k8;
    uint16_t *dsc = which ? v_scale : k_scale;
    const __half *p16 = (which ? cv.v16 : cv.k16) + u * cv.cap16 * D;
    const int8_t *p8 = (which ? cv.v8 : cv.k8) + u * cv.cap8 * D;
    const __half *psc = (which ? cv.vs : cv.ks) + u * cv.cap8;
    if (d16) {
      memset(d16, 0, (size_t)n8 * D * 2);
      if (n16 > 0) {
        const int first = std::min(n16, cv.cap16 - head);
        CK_HIP(h, hipMemcpy(d16 + (size_t)n8 * D, p16 + (size_t)head * D, (size_t)first * D * 2,
                            hipMemcpyDeviceToHost));
        if (n16 > first)
          CK_HIP(h, hipMemcpy(d16 + (size_t)(n8 + first) * D, p16, (size_t)(n16 - first) * D * 2,
                              hipMemcpyDeviceToHost));
      }
    }
    if (d8) {
      if (first8 > 0)
        CK_HIP(h, hipMemcpy(d8, p8 + (size_t)head8 * D, (size_t)first8 * D, hipMemcpyDeviceToHost));
      if (n8 > first8)
        CK_HIP(h, hipMemcpy(d8 + (size_t)first8 * D, p8, (size_t)(n8 - first8) * D, hipMemcpyDeviceToHost));
      memset(d8 + (size_t)n8 * D, 0, (size_t)n16 * D);
    }
    if (dsc && !cv.chan) {
      if (first8 > 0)
        CK_HIP(h, hipMemcpy(dsc, psc + head8, (size_t)first8 * 2, hipMemcpyDeviceToHost));
      if (n8 > first8)
        CK_HIP(h, hipMemcpy(dsc + first8, psc, (size_t)(n8 - first8) * 2, hipMemcpyDeviceToHost));
      memset(dsc + n8, 0, (size_t)n16 * 2);
    }
  }
  return CONF_KV_OK;
}

int conf_kv_import(conf_kv_handle *h, int32_t layer, int32_t b, int32_t kv_head, int32_t n,
                   const int32_t *pos, const float *ema, const uint8_t *is_fp16, const uint16_t *k16,
                   const uint16_t *v16, const int8_t *k8, const int8_t *v8, const uint16_t *k_scale,
                   const uint16_t *v_scale) {
  if (!h) return CONF_KV_ERR_INVALID_ARG;
  if (layer < 0 || layer >= h->cfg.n_layers) return CONF_KV_ERR_BAD_LAYER;
  if (b < 0 || b >= h->cfg.batch || kv_head < 0 || kv_head >= h->cfg.n_kv_heads || n < 0)
    return CONF_KV_ERR_INVALID_ARG;
  if (n > h->cfg.capacity - 1) return CONF_KV_ERR_CAPACITY;
  if (h->appended[layer] || h->cv.page_lg) return CONF_KV_ERR_BAD_STATE;   // (no import into the paged layout)
  if (n > 0 && (!pos || !ema || !is_fp16)) return CONF_KV_ERR_INVALID_ARG;
  const CacheView &cv = h->cv;
  int n8 = 0;
  while (n8 < n && !is_fp16[n8]) ++n8;
  const int n16 = n - n8;
  for (int i = n8; i < n; ++i)
    if (!is_fp16[i]) return CONF_KV_ERR_INVALID_ARG;             // an INT8 slot behind an FP16 one
  for (int i = 1; i < n; ++i)
    if (pos[i] <= pos[i - 1]) return CONF_KV_ERR_INVALID_ARG;
  if (cv.W < 0 ? n8 > 0 : n16 > cv.W) return CONF_KV_ERR_INVALID_ARG;
  if (n16 > cv.cap16) return CONF_KV_ERR_INVALID_ARG;
  if (n8 > 0 && (!k8 || !v8 || !k_scale || !v_scale)) return CONF_KV_ERR_INVALID_ARG;
  if (cv.chan) {
    if (!k_scale || !v_scale) return CONF_KV_ERR_INVALID_ARG;
    for (int d = 0; d < cv.D; ++d)                                // fp16 bits: finite and >= 0
      if ((k_scale[d] & 0x8000u) || (k_scale[d] & 0x7c00u) == 0x7c00u || (v_scale[d] & 0x8000u) ||
          (v_scale[d] & 0x7c00u) == 0x7c00u)
        return CONF_KV_ERR_INVALID_ARG;
  }
  if (n16 > 0 && (!k16 || !v16)) return CONF_KV_ERR_INVALID_ARG;
  const size_t u = ((size_t)layer * cv.B + b) * cv.Hkv + kv_head;
  const size_t D = cv.D;
  CK_HIP(h, hipDeviceSynchronize());
  if (n > 0) {
    CK_HIP(h, hipMemcpy(cv.pos + u * cv.cap, pos, (size_t)n * 4, hipMemcpyHostToDevice));
    CK_HIP(h, hipMemcpy(cv.ema + u * cv.cap, ema, (size_t)n * 4, hipMemcpyHostToDevice));
  }
  if (n8 > 0) {                                                   // INT8 ring rows 0 .. n8-1
    CK_HIP(h, hipMemcpy(cv.k8 + u * cv.cap8 * D, k8, (size_t)n8 * D, hipMemcpyHostToDevice));
    CK_HIP(h, hipMemcpy(cv.v8 + u * cv.cap8 * D, v8, (size_t)n8 * D, hipMemcpyHostToDevice));
    if (!cv.chan) {
      CK_HIP(h, hipMemcpy(cv.ks + u * cv.cap8, k_scale, (size_t)n8 * 2, hipMemcpyHostToDevice));
      CK_HIP(h, hipMemcpy(cv.vs + u * cv.cap8, v_scale, (size_t)n8 * 2, hipMemcpyHostToDevice));
    }
  }
  if (cv.chan) {
    CK_HIP(h, hipMemcpy(cv.ks + u * D, k_scale, D * 2, hipMemcpyHostToDevice));
    CK_HIP(h, hipMemcpy(cv.vs + u * D, v_scale, D * 2, hipMemcpyHostToDevice));
    h->scaled[u] = 1;
  }
  if (n16 > 0) {                                                  // FP16 ring rows 0 .. n16-1
    CK_HIP(h, hipMemcpy(cv.k16 + u * cv.cap16 * D, k16 + (size_t)n8 * D, (size_t)n16 * D * 2,
                        hipMemcpyHostToDevice));
    CK_HIP(h, hipMemcpy(cv.v16 + u * cv.cap16 * D, v16 + (size_t)n8 * D, (size_t)n16 * D * 2,
                        hipMemcpyHostToDevice));
  }
  const int32_t zero = 0, len = n, cnt8 = n8;
  CK_HIP(h, hipMemcpy(cv.len + u, &len, 4, hipMemcpyHostToDevice));
  CK_HIP(h, hipMemcpy(cv.n8 + u, &cnt8, 4, hipMemcpyHostToDevice));
  CK_HIP(h, hipMemcpy(cv.head16 + u, &zero, 4, hipMemcpyHostToDevice));
  CK_HIP(h, hipMemcpy(cv.head8 + u, &zero, 4, hipMemcpyHostToDevice));
  h->len_ub[layer] = std::max(h->len_ub[layer], n);
  h->prompt_loaded = true;
  h->fresh_len[layer] = -1;
  if (n > 0) {                       // later tokens get positions behind the imported ones
    unsigned next = 0;
    CK_HIP(h, hipMemcpy(&next, h->cv.ctl + kCtlPos + layer, 4, hipMemcpyDeviceToHost));
    next = std::max(next, (unsigned)(pos[n - 1] + 1));
    CK_HIP(h, hipMemcpy(h->cv.ctl + kCtlPos + layer, &next, 4, hipMemcpyHostToDevice));
  }
  return CONF_KV_OK;
}

int conf_kv_counters(conf_kv_handle *h, conf_kv_stats *st) {
  if (!h || !st) return CONF_KV_ERR_INVALID_ARG;
  unsigned long long raw[kStatSlots];
  CK_HIP(h, hipDeviceSynchronize());
  CK_HIP(h, hipMemcpy(raw, h->cv.stats, sizeof(raw), hipMemcpyDeviceToHost));
  const size_t U = (size_t)h->cfg.n_layers * h->cfg.batch * h->cfg.n_kv_heads;
  std::vector<unsigned> ev(U), dm(U);
  CK_HIP(h, hipMemcpy(ev.data(), h->cv.unit_evicted, U * 4, hipMemcpyDeviceToHost));
  CK_HIP(h, hipMemcpy(dm.data(), h->cv.unit_demoted, U * 4, hipMemcpyDeviceToHost));
  std::vector<unsigned long long> mv(U);
  CK_HIP(h, hipMemcpy(mv.data(), h->cv.unit_moved, U * 8, hipMemcpyDeviceToHost));
  st->evicted = st->demoted = st->compact_bytes = 0;
  for (size_t u = 0; u < U; ++u) { st->evicted += ev[u]; st->demoted += dm[u]; st->compact_bytes += mv[u]; }
  st->tight_steps = raw[kStatTight];
  st->loose_steps = raw[kStatLoose];
  st->device_errors = raw[kStatDeviceErr];
  return raw[kStatDeviceErr] ? CONF_KV_ERR_DEVICE : CONF_KV_OK;
}

const char *conf_kv_strerror(int status) {
  switch (status) {
    case CONF_KV_OK: return "ok";
    case CONF_KV_ERR_INVALID_ARG: return "invalid argument (null pointer, negative size or misaligned buffer)";
    case CONF_KV_ERR_BAD_SHAPE: return "configuration outside what the kernels support";
    case CONF_KV_ERR_BAD_LAYER: return "layer index out of range";
    case CONF_KV_ERR_CAPACITY: return "cache capacity exceeded";
    case CONF_KV_ERR_BAD_STATE: return "call order violated (one conf_kv_attend per layer between conf_kv_evict_compact calls)";
    case CONF_KV_ERR_HIP: return "a HIP call failed (see conf_kv_last_hip_error)";
    case CONF_KV_ERR_DEVICE: return "a kernel reported an internal error";
    default: return "unknown status";
  }
}

int conf_kv_last_hip_error(conf_kv_handle *h) { return h ? h->last_hip : 0; }

int conf_kv_probe_read(const void *dev_src, size_t bytes, uint32_t *dev_out, int32_t workgroups,
                       conf_kv_stream stream) {
  if (!dev_src || !dev_out || bytes == 0 || bytes % 16 || ((uintptr_t)dev_src & 15) || workgroups < 1 ||
      workgroups > 65536)
    return CONF_KV_ERR_INVALID_ARG;
  return launch_probe_read(dev_src, bytes, dev_out, workgroups, (hipStream_t)stream) == hipSuccess
             ? CONF_KV_OK
             : CONF_KV_ERR_HIP;
}

}  // extern "C"

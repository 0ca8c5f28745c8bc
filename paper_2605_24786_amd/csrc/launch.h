// Host-side launchers of the kernels, one per source file.  Internal to the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "confkv_dev.h"

namespace confkv {

// ---- conf_reduce.hip ----
size_t conf_reduce_scratch_bytes(int B, int V);   // epoch-tagged chunk partials: zero before the first call
hipError_t launch_conf_reduce(const CacheView &cv, const float *logits, int V, unsigned long long *partial,
                              unsigned launch_no /* the words' tag; never 0, never reused */,
                              int device_base /* 1: the tag is launch_no + cv.ctl[kCtlConfTag] */, int spin_limit,
                              int withhold /* test hook: chunk 0 does not publish, so the bounded wait expires */,
                              float *conf, uint8_t *sel, double tau, double wH, double wm, double wp,
                              hipStream_t stream);
// words [0, bytes / 8) <- 0 on the stream (a kernel, not a memset node)
hipError_t launch_zero_words(void *p, size_t bytes, hipStream_t stream);
// The same launch with the chunk partials in a file-scope device array of the library (one copy
// per device, shared by every call on that device; kConfStaticBytes of it).  setup resolves the
// array's address on the current device once; the launch does it too if nobody has.
constexpr size_t kConfStaticBytes = (size_t)1 << 20;
hipError_t conf_reduce_static_setup();
hipError_t launch_conf_reduce_static(const CacheView &cv, const float *logits, int V, int spin_limit, int withhold,
                                     float *conf, uint8_t *sel, double tau, double wH, double wm, double wp,
                                     hipStream_t stream);
constexpr int kSpinLimitDefault = 400000;   // polls (about a microsecond each) before a bounded wait gives up

// ---- probe.hip ----
hipError_t launch_probe_read(const void *src, size_t bytes, unsigned *out, int workgroups, hipStream_t stream);

// ---- attend.hip ----
struct AttendPlan {
  int splits;        // workgroups per unit
  int stash_tokens;  // score slots per workgroup held in LDS
  size_t lds_bytes;  // dynamic LDS per workgroup
  bool mfma;         // matrix-core body for the INT8 slots
  bool two_launch;   // stream + publish, then merge + EMA in a second launch (scores in scratch)
  int wide_rb;       // > 0: the many-rows kernel with that many blocks of 16 query rows per unit
};
struct AttendLaunch {
  int layer;
  const __half *q, *knew, *vnew;
  __half *out;
  unsigned long long *part_ml;   // [units per layer][max splits][G][2] words: (epoch << 32) | float bits of m, of l
  unsigned long long *part_o;    // [units per layer][max splits][G][D] words: (epoch << 32) | float bits of a partial output
  unsigned epoch;          // number of the launch since the last commit, from 1; the kernels add the base in
                           // cv.ctl: the sum tags the words the launch publishes (never 0, never reused)
  int spin_limit;          // polls before a wait for the other splits gives up (device error)
  int max_splits;
  float sm_scale, ema_decay;
  double mass_gain;        // weight of the step's mass in the EMA update
  unsigned tag_base;       // filled in by the kernels from cv.ctl
  int pos_new;             // position of the first appended token (the kernels read it from cv.ctl)
  int tq;                  // tokens appended (and queries per head) in this call
  int q_tokens;            // tokens per sequence in the q tensor: q is [B][q_tokens][Hq][D] and the call's
                           // queries are its first tq tokens (tq, unless the call is a window of a longer tensor)
  int gq;                  // query heads per kv-head; the kernels' row r is (token r / gq, head r % gq)
  int observe_first;       // >= 0: the queries belong to the cached slots observe_first .. observe_first + tq - 1;
                           // nothing is appended and slots from observe_first + tq on are left alone
  int withhold;            // test hook: split 0 of every unit does not publish its statistics, so the
                           // other splits' bounded waits expire (the kernel still ends normally)
  int kv_major;            // grid is (kv-heads, splits, sequences) instead of (splits, kv-heads, sequences)
  float *spill;            // [units per layer][splits][G][stash_tokens] raw scores (two-launch form)
  unsigned long long *dbg; // phase-trace buffer (CONFKV_TRACE builds), else null
  int tab_off;             // paged layout: byte offset of the unit's block table in dynamic LDS
  int trace_off;           // byte offset of the time stamps in dynamic LDS (CONFKV_TRACE builds)
};
constexpr int kAttendMaxSplits = 64;
constexpr int kChunkRows = 16;     // query rows per unit of a multi-token call (one matrix-core tile)
bool attend_supported(int D, int G);
size_t attend_spill_floats(int units_per_layer, int G, int cap);   // scratch the two-launch form needs
// Largest split count and LDS plan for a unit of at most n_ub tokens (after the append)
// of which at most n16_ub are FP16.  G = query rows per unit (the group size, or kChunkRows for
// a multi-token call, which only has the single-launch matrix-core form).  Returns false when no plan fits the device.
// extra_lds: bytes the launch needs behind the kernel's own dynamic LDS (the block table of the paged layout).
bool attend_plan(int D, int G, bool chan, bool chunk, int units_per_layer, int n_ub, int n16_ub, int forced_splits,
                 bool force_two_launch, size_t extra_lds, AttendPlan *plan);
// Plan of a call with more than kChunkRows query rows per unit (at most kWideRowsMax); false when
// the shape cannot be served.
constexpr int kWideRowsMax = 128;
bool attend_wide_plan(int rows, int units_per_layer, int n_ub, int forced_splits, AttendPlan *plan);
hipError_t launch_attend(const CacheView &cv, const AttendLaunch &a, const AttendPlan &plan,
                         hipStream_t stream);

// ---- evict.hip ----
// Per unit, written by rank_select: [0] new length, [1] new INT8 count, [2] first evicted slot,
// [3] evicted slots, [4] last evicted INT8 slot (-1: none), [5] 1 = the INT8 rows in front of
// that slot shift right (the ring head advances), 0 = the rows behind the first hole shift
// left, [6] INT8 ring head after the compaction, [7] 1 = the entries above are final for this
// call (0 after the first ranking kernel: the unit waits for the general one).
constexpr int kSelInts = 8;
hipError_t launch_load_prefill(const CacheView &cv, int layer, const __half *k16, const __half *v16,
                               int T0, const float *ema0, hipStream_t stream);
// Ranker variants; all zero = the composite ranker per (layer, kv-head).
struct RankOptions {
  int random;                  // 1: rank by counter-based uniform draws instead of the composite score
  unsigned long long seed;
  double *shared;              // non-null: layer scope; [L * B][cap] scratch for the summed mass
  int page;                    // > 1: whole pages of that many original positions are evicted
};
hipError_t launch_evict_compact(const CacheView &cv, const LayerMask &appended, double alpha,
                                const RankOptions &opt, double *score, int32_t *src, int32_t *sel,
                                int n_max /* longest unit */,
                                unsigned attend_launches, unsigned conf_launches /* since the last commit */,
                                int after_prompt /* a layer's prompt was loaded since the last commit: long moves */,
                                hipStream_t stream);

}  // namespace confkv

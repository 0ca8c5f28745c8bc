/*
 * conf_kv.h -- C ABI of the Conf-KV per-decode-step library for AMD MI355X (gfx950).
 *
 * The library keeps, for every unit (layer, batch, kv-head), a position-sorted KV
 * cache whose oldest tokens are INT8 (per-token, per-kv-head fp16 absmax scales) and
 * whose newest tokens are FP16, plus per-slot metadata (original position, fp32 EMA of
 * attention mass).  One decode step is
 *
 *     for every layer:  conf_kv_attend          (append + attention + mass EMA)
 *     once:             conf_kv_step            (confidence -> tight/loose budget)
 *     once:             conf_kv_evict_compact   (rank, evict, compact, demote)
 *
 * which is the paper's Algorithm 1 with the append moved in front of the step's own
 * attention (a decode query attends to its own key).
 *
 * Conventions
 *   - "dev" pointers are device memory owned by the CALLER and valid until
 *     conf_kv_destroy; "host" pointers are ordinary host memory.  The library never
 *     allocates or frees device memory.
 *   - The three hot calls only enqueue kernels on the given stream; they never
 *     synchronise.  Lengths and budgets live on the device; the host keeps upper bounds.
 *   - A handle is driven from one host thread, on one stream at a time.
 *   - A whole decode step (the calls above, on one stream) may be recorded into a HIP graph
 *     and replayed: the calls enqueue kernels only (no copies, no memset nodes), and what
 *     changes from step to step (lengths, ring heads, budgets, the positions appended tokens
 *     get, the tags the in-kernel waits compare) lives on the device and is advanced by the
 *     kernels themselves.  The kernel arguments do hold the launch shapes, which the host
 *     derives from upper bounds of the lengths: call conf_kv_static_plan(h, 1) before
 *     recording, so that the shapes cover every later step, and record only after one step has
 *     run outside the graph (first launches set kernel attributes).  The tensors the recorded
 *     calls read and write are the ones given at recording time.  conf_kv_step_static keeps its
 *     tag on the host and is not replayable.
 *   - At most 2^23 attention or confidence launches may lie between two
 *     conf_kv_evict_compact calls (CONF_KV_ERR_BAD_STATE beyond that).
 *   - Every function returns CONF_KV_OK (0) or a negative conf_kv_status; nothing throws.
 *   - Tensors are dense, row-major, in the index order written next to each argument.
 *   - fp16 data is IEEE binary16; "int8" codes are two's complement in [-127, 127].
 */
#ifndef CONF_KV_H
#define CONF_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct conf_kv_handle conf_kv_handle;
typedef void *conf_kv_stream;            /* a hipStream_t; NULL = the default stream */

typedef enum conf_kv_status {
  CONF_KV_OK = 0,
  CONF_KV_ERR_INVALID_ARG = -1,  /* null pointer, negative size, misaligned buffer            */
  CONF_KV_ERR_BAD_SHAPE = -2,    /* a config field outside what the kernels are built for     */
  CONF_KV_ERR_BAD_LAYER = -3,    /* layer index outside [0, n_layers)                          */
  CONF_KV_ERR_CAPACITY = -4,     /* the operation would need more slots than `capacity`       */
  CONF_KV_ERR_BAD_STATE = -5,    /* call order violated (see each function)                    */
  CONF_KV_ERR_HIP = -6,          /* a HIP call failed; see conf_kv_last_hip_error             */
  CONF_KV_ERR_DEVICE = -7        /* a kernel reported an internal error (bounded wait expired) */
} conf_kv_status;

/*
 * Problem statement of Algorithm 1 (its REQUIRE line: thresholds tau, budgets
 * N_high / N_low, protected window P, ranker weight alpha, FP16 window W) plus the
 * shape of the model's attention.  Weights of Eq. 1 are (w_entropy, w_margin, w_top).
 */
typedef struct conf_kv_config {
  int32_t n_layers;          /* L  >= 1                                                        */
  int32_t batch;             /* B  >= 1 sequences, all at the same decode position             */
  int32_t n_q_heads;         /* Hq, a multiple of n_kv_heads; group G = Hq / Hkv in 1..8
                                (1..16 at head_dim 128)                                        */
  int32_t n_kv_heads;        /* Hkv                                                            */
  int32_t head_dim;          /* D in {64, 128}                                                 */
  int32_t vocab;             /* V >= 2                                                         */
  int32_t capacity;          /* slots per unit; a multiple of 16; must exceed every budget     */
  int32_t fp16_window;       /* W >= 0: newest W retained tokens stay FP16; < 0: FP16-only     */
  int32_t protected_window;  /* P >= 0: the newest P tokens are never evicted                  */
  float tau;                 /* tight budget when c >= tau (paper: 0.7)                        */
  float alpha;               /* ranker weight on attention mass (paper: 0.65)                  */
  float ema_decay;           /* lambda of the mass EMA (paper: 0.9)                            */
  float sm_scale;            /* softmax scale, usually 1/sqrt(D)                               */
  float w_entropy, w_margin, w_top; /* Eq. 1 weights (paper: 0.4, 0.3, 0.3)                    */
  const int32_t *n_tight;    /* host [L]: N_high per layer (budget on confident steps)         */
  const int32_t *n_loose;    /* host [L]: N_low  per layer; n_tight[l] <= n_loose[l]           */
  /* Variants of the ranker (the paper's experimental setup and its literal per-layer
   * bookkeeping).  All zeros except mass_gain < 0 give the method as described above. */
  float mass_gain;           /* weight of a step's mass: a <- ema_decay a + mass_gain A;
                                negative = 1 - ema_decay (the paper's EMA); (ema_decay,
                                mass_gain) = (1, 1) is the running sum of the mass         */
  int32_t ranker;            /* conf_kv_ranker                                                 */
  int32_t rank_scope;        /* conf_kv_rank_scope                                             */
  uint64_t ranker_seed;      /* CONF_KV_RANKER_RANDOM: seed of its counter-based draws         */
  int32_t scale_mode;        /* conf_kv_scale_mode: granularity of the INT8 scales             */
  int32_t max_chunk;         /* most tokens one conf_kv_attend_chunk / conf_kv_observe call may
                                carry; 0 or 1 = single-token calls only.  Above 1: head_dim 128
                                and max_chunk * (n_q_heads / n_kv_heads) <= 128 query rows per
                                kv-head; beyond 16 rows per-token scales only                  */
  int32_t evict_page;        /* 0 or 1: tokens are evicted one by one.  g > 1 (at most 1024):
                                coarsened eviction for paged layouts (the remedy the paper names
                                in "Compatibility with serving systems" and "Limitations" for
                                partially dead blocks; it defines no rule) -- a page is the live slots
                                whose original positions share floor(position / g); a page
                                goes whole or not at all, and only when none of its slots lies
                                in the protected window; pages are ranked by the mean of their
                                slots' scores and go lowest first, older first among equal
                                means, until the length is at most the budget (it may end up to
                                g - 1 below it) or no page that can go is left (up to g - 1
                                slots over max(budget, protected_window) then remain).
                                capacity must hold max(n_loose, protected_window + g - 1) plus
                                the appended tokens                                            */
  int32_t layout;            /* conf_kv_layout: where the INT8 slots of a unit live              */
} conf_kv_config;

typedef enum conf_kv_layout {
  CONF_KV_LAYOUT_CONTIGUOUS = 0, /* the paper's layout ("Cache manager": gather survivors into
                                    contiguous storage): slots in position order in one ring per
                                    plane; an eviction moves the rows on the cheaper side of
                                    the holes                                                    */
  CONF_KV_LAYOUT_PAGED = 1       /* the alternative "Compatibility with serving systems" and
                                    "Limitations" name for paged serving stacks: the INT8 slots
                                    of a unit live in pages of evict_page slots reached through a
                                    per-unit block table; a page holds the tokens whose original
                                    positions share floor(position / evict_page); attention reads
                                    rows through the table; evicting a page edits the table and
                                    moves no row.  Needs coarsened eviction (evict_page a power
                                    of two, 8 .. 1024), a mixed cache with fp16_window <=
                                    protected_window (so that only whole INT8 pages can go),
                                    per-token scales, the per-kv-head ranking scope, a group of
                                    2 .. 8 query heads and single-token attention calls;
                                    conf_kv_import is not available.  conf_kv_export returns the
                                    same position-sorted view as under the contiguous layout     */
} conf_kv_layout;

typedef enum conf_kv_scale_mode {
  CONF_KV_SCALES_TOKEN = 0,     /* one scale per token and kv-head (absmax over the channels),
                                   separately for K and V                                      */
  CONF_KV_SCALES_CHANNEL = 1    /* the granularity "Tiled attention and mixed precision" names:
                                   one scale per (kv-head, channel), separately for K and V,
                                   s_d = fl16(fl32(max_t |x_{t,d}| / 127)) over ALL T0 prompt
                                   tokens of conf_kv_load_prefill (those that stay FP16
                                   included), fixed from then on; later tokens saturate at
                                   +-127.  Attention folds the K scales into the query and the
                                   V scales into the output.  Needs D = 128 and a mixed cache
                                   (fp16_window >= 0); a layer must be given its scales
                                   (conf_kv_load_prefill or conf_kv_import) before its first
                                   conf_kv_evict_compact, else CONF_KV_ERR_BAD_STATE           */
} conf_kv_scale_mode;

typedef enum conf_kv_ranker {
  CONF_KV_RANKER_COMPOSITE = 0, /* s = alpha * minmax(mass) + (1 - alpha) * minmax(position)  */
  CONF_KV_RANKER_RANDOM = 1     /* s = top 53 bits of splitmix64(seed + unit * 2^32 + position)
                                   as a fraction: which token goes is random, how many go is
                                   still the budget rule's (matched-rate isolation); unit =
                                   (layer * B + b) * Hkv + kv_head, or 2^40 + layer * B + b in
                                   layer scope                                                 */
} conf_kv_ranker;

typedef enum conf_kv_rank_scope {
  CONF_KV_SCOPE_KV_HEAD = 0,    /* one importance value and one kept set per (layer, kv-head)  */
  CONF_KV_SCOPE_LAYER = 1       /* one kept set per (layer, sequence): the importance of a
                                   token is its mass summed over the kv-heads (the head
                                   average up to a factor that min-max removes); every kv-head
                                   of a sequence must hold the same positions                  */
} conf_kv_rank_scope;

typedef struct conf_kv_stats {
  uint64_t evicted;          /* tokens evicted, summed over units                              */
  uint64_t demoted;          /* tokens quantised FP16 -> INT8 by conf_kv_evict_compact         */
  uint64_t tight_steps;      /* sequence-steps that selected the tight budget                  */
  uint64_t loose_steps;      /* sequence-steps that selected the loose budget                  */
  uint64_t device_errors;    /* bounded waits that expired inside kernels (0 in a healthy run) */
  uint64_t compact_bytes;    /* bytes read + written by the compaction's in-place row moves    */
} conf_kv_stats;

/* Environment variables read once by conf_kv_create (test and measurement hooks; none is
 * needed in normal use): CONF_KV_SPLITS=n asks for n workgroups per unit in conf_kv_attend
 * instead of the planned number (clamped to what the unit's length allows);
 * CONF_KV_TWO_LAUNCH=1 forces the two-launch form of conf_kv_attend; CONF_KV_NO_MFMA=1 (read
 * at the first plan of the process) keeps every shape on the vector-ALU streaming body;
 * CONF_KV_SPIN_LIMIT=n bounds the in-kernel waits for other workgroups to n polls (default
 * 400000, about 0.4 s; an expired wait ends the kernel early and counts a device error);
 * CONF_KV_TEST_WITHHOLD=1 makes split 0 of every unit (conf_kv_attend) and chunk 0 of every
 * logit row (conf_kv_step) keep their published words to themselves, so that the waits of the
 * others expire (the kernels still end normally; tests of the expiry path);
 * CONF_KV_GRID_KV_MAJOR=0/1 overrides the order of the attention grid (kv-heads first puts all
 * splits of a unit on one XCD and is the default when the number of kv-heads is a multiple of 8);
 * CONF_KV_COMPACT_PAIRED=0/1 (read at every conf_kv_evict_compact) forces one of the two grid
 * shapes of the compaction kernel, which is otherwise chosen by the number of units;
 * CONF_KV_TEST_TAG_BASE=n starts the device-side tag bases (see conf_kv_tag_state) at n instead
 * of 0, so that a test reaches the clearing of the exchange words in a few steps. */

/* Bytes of device memory the caller must provide for the cache state and for scratch
 * (tagged exchange words of the splits and chunks, ranking work arrays).  0 on an invalid config. */
size_t conf_kv_state_bytes(const conf_kv_config *cfg);
size_t conf_kv_scratch_bytes(const conf_kv_config *cfg);

/* Validates cfg, copies it, lays the cache out inside dev_state (256-byte aligned, at
 * least conf_kv_state_bytes) and dev_scratch (likewise), zeroes lengths / counters /
 * scratch with synchronous HIP calls on the current device, and sets every budget to the
 * loose one.  All units start empty.  On error *out is NULL. */
int conf_kv_create(conf_kv_handle **out, const conf_kv_config *cfg, void *dev_state,
                   void *dev_scratch);

/* Pyramidal per-layer budgets ("Pyramidal layer budgets": N(l) = max(N_min,
 * N(0) * beta^(l / L))), floored to integers, for filling n_tight / n_loose: host_out int32
 * [n_layers].  The paper uses beta = 0.5 and N_min = 96.  Pure host arithmetic in double;
 * CONF_KV_ERR_INVALID_ARG on n_layers < 1, n0 < 1, n_min < 1 or beta outside (0, 1]. */
int conf_kv_pyramid_budgets(int32_t n0, int32_t n_layers, double beta, int32_t n_min,
                            int32_t *host_out);

/* Frees the host-side handle only (device buffers belong to the caller). */
int conf_kv_destroy(conf_kv_handle *h);

/* Replaces the cache of one layer by T0 prompt tokens at positions 0..T0-1
 * (Algorithm 1's input cache).  dev_k16 / dev_v16: fp16 [B][Hkv][T0][D], 16-byte aligned
 * (CONF_KV_ERR_INVALID_ARG otherwise).
 * dev_ema0: fp32 [B][Hkv][T0] initial EMA importance, or NULL for zeros.
 * All but the newest W tokens are quantised to INT8 ("Tiled attention and mixed
 * precision": symmetric, scale = max|x|/127, per token and kv-head, or per kv-head and
 * channel over the T0 prompt tokens: conf_kv_scale_mode).
 * 0 <= T0 <= capacity - 1, else CONF_KV_ERR_CAPACITY.  Enqueues on `stream`. */
int conf_kv_load_prefill(conf_kv_handle *h, int32_t layer, const void *dev_k16,
                         const void *dev_v16, int32_t T0, const float *dev_ema0,
                         conf_kv_stream stream);

/*
 * Decode attention of one layer with the importance update fused in
 * (Algorithm 1: forward pass attention, "update EMA attention metadata", "append new K/V
 * in FP16"; "Tiled attention and mixed precision"; "Budget and ranker").
 *   1. appends (k_new, v_new) in FP16 at the next position with EMA 0;
 *   2. out[b][h] = softmax_i(sm_scale * q[b][h] . K_i) V_i over ALL stored slots of the
 *      unit (b, h / G), K_i/V_i being the fp16 value or int8 code * fp16 scale, computed
 *      as split-K blockwise online softmax with fp32 accumulation;
 *   3. per slot, A_i = sum over the G query heads of the exact normalised probability
 *      (so sum_i A_i = G), then ema_i <- lambda * ema_i + (1 - lambda) * A_i.
 * dev_q16: fp16 [B][Hq][D]; dev_knew16 / dev_vnew16: fp16 [B][Hkv][D]; dev_out16: fp16
 * [B][Hq][D], written.  All 16-byte aligned.
 * Exactly one conf_kv_attend per layer between two conf_kv_evict_compact calls
 * (CONF_KV_ERR_BAD_STATE otherwise); CONF_KV_ERR_CAPACITY, before anything is launched,
 * if the unit could already hold `capacity` tokens.
 * The workgroups that share a unit exchange partial results inside the launch, so the launch
 * is sized to be resident on the device all at once.  Other kernels running at the same time
 * only delay it (its waits are bounded at several hundred milliseconds); a wait that does
 * expire leaves the call's outputs undefined and is reported by conf_kv_counters
 * (device_errors, CONF_KV_ERR_DEVICE).
 */
int conf_kv_attend(conf_kv_handle *h, int32_t layer, const void *dev_q16, const void *dev_knew16,
                   const void *dev_vnew16, void *dev_out16, conf_kv_stream stream);

/* Several consecutive tokens of every sequence in one call (a chunk of a prompt, or decode
 * tokens that are all kept; "Compatibility with serving systems" names such multi-token
 * steps): 1 <= tq <= max_chunk.  Defined as tq conf_kv_attend calls without eviction in
 * between: token t gets position p0 + t, query t attends the cache and the chunk's tokens
 * 0 .. t (causal), and the importance follows a <- lambda a + gain A_t once per query, i.e.
 * a_i <- lambda^tq a_i + gain * sum_t lambda^(tq-1-t) A_{t,i}, stored once.  The keys and
 * values of the cache are read once for all tq queries.
 * dev_q16 / dev_out16: fp16 [B][tq][Hq][D]; dev_knew16 / dev_vnew16: fp16 [B][tq][Hkv][D].
 * The following conf_kv_evict_compact commits all tq appends.  Same errors as conf_kv_attend;
 * tq outside 1 .. max(1, max_chunk) is CONF_KV_ERR_INVALID_ARG. */
int conf_kv_attend_chunk(conf_kv_handle *h, int32_t layer, int32_t tq, const void *dev_q16,
                         const void *dev_knew16, const void *dev_vnew16, void *dev_out16,
                         conf_kv_stream stream);

/* Importance from the prompt's own attention (the step before the decode loop: the cache's
 * initial importance comes from an observation window of queries at the end of the prompt
 * instead of starting at zero).  dev_q16: fp16 [B][tq][Hq][D], the queries of the cached slots
 * first .. first + tq - 1 of every unit of the layer; nothing is appended.  Defined like
 * conf_kv_attend_chunk on the stored values: query t sees slots 0 .. first + t, the importance
 * of every slot below first + tq follows a <- lambda a + gain A_t once per query (a window
 * slot counts from 0 at its own query, whatever it held before), slots from first + tq on are
 * neither seen nor changed.  Calls for consecutive windows first = s, s + tq, .. compose.
 * dev_out16: fp16 [B][tq][Hq][D] attention outputs of those queries, or NULL.
 * Allowed between conf_kv_load_prefill of the layer and its first conf_kv_attend
 * (CONF_KV_ERR_BAD_STATE otherwise), with max_chunk >= 2 (or a group of more than 8 heads, then
 * tq = 1), 1 <= tq <= max(1, max_chunk) (calls of more than 16 / G tokens run on a kernel that
 * reads the keys twice instead of keeping 16 x slots scores on chip) and
 * 0 <= first, first + tq <= T0 (CONF_KV_ERR_INVALID_ARG). */
int conf_kv_observe(conf_kv_handle *h, int32_t layer, int32_t first, int32_t tq, const void *dev_q16,
                    void *dev_out16, conf_kv_stream stream);

/* The prompt-phase importance in full (the step before the decode loop; "Related work" names
 * prompt-phase observation as the neighbouring idea, the paper's own update is "using A" per
 * decode step): every prompt query observes the prompt causally, as conf_kv_observe over the
 * consecutive windows first = 0, max_chunk, 2 max_chunk, .. covering all T0 cached tokens, in one
 * launch sequence.  dev_q16: fp16 [B][T0][Hq][D], the queries of all prompt tokens.  The result is
 * what T0 single-token decode steps over the stored prompt would have left (see
 * conf_kv_attend_chunk for the telescoped update).  Same call order rules and errors as
 * conf_kv_observe; needs max_chunk >= 2. */
int conf_kv_observe_prompt(conf_kv_handle *h, int32_t layer, const void *dev_q16, conf_kv_stream stream);

/*
 * Confidence estimator and budget selector (Eq. 1; "Budget and ranker"; Algorithm 1,
 * lines softmax / c / N).  For every sequence b: p = softmax(logits[b]),
 * c = w_entropy (1 - H(p)/log V) + w_margin sigmoid(log p_(1) - log p_(2)) + w_top p_(1);
 * tight = (c >= tau); the per-layer budget N[l][b] = tight ? n_tight[l] : n_loose[l]
 * stays on the device for the next conf_kv_evict_compact.
 * dev_logits: fp32 [B][V] (-inf entries allowed).  dev_conf: fp32 [B] written.
 * dev_sel: uint8 [B] written, 1 = tight.  Either output may be NULL.
 */
int conf_kv_step(conf_kv_handle *h, const float *dev_logits, float *dev_conf, uint8_t *dev_sel,
                 conf_kv_stream stream);

/*
 * conf_kv_step for callers that cannot allocate or hand over a workspace at the time of the call
 * (code under HIP graph capture, tight serving loops, harnesses that forbid allocation): same
 * arguments, same results, but the per-chunk partial sums of the reduction live in a device
 * array of the library itself (1 MiB per GPU, resident from the library's load until the
 * process ends) instead of the handle's dev_scratch.  The call allocates and frees nothing.
 * Limit: batch * ceil(vocab / 4096) * 64 bytes must fit that array, i.e. batch * ceil(vocab /
 * 4096) <= 16384 (CONF_KV_ERR_CAPACITY otherwise, before anything is launched).  Every call on
 * one GPU, from any handle, uses that GPU's one array: calls that overlap in time on one GPU
 * (different streams or host threads) race and give undefined results; calls in stream order
 * are safe, whatever their sizes.
 */
int conf_kv_step_static(conf_kv_handle *h, const float *dev_logits, float *dev_conf, uint8_t *dev_sel,
                        conf_kv_stream stream);

/*
 * Ranker, eviction, in-place compaction and demotion for every layer (Algorithm 1's
 * per-layer tail; "Budget and ranker"; "Cache manager").  For each unit with
 * n > N[l][b]: the newest min(P, n) slots are protected; over the other slots
 * s_i = alpha * minmax(ema_i) + (1 - alpha) * minmax(pos_i) (min-max over those
 * candidates, 0 when degenerate), the min(n - N, n - P) lowest are evicted (equal
 * scores: oldest first), survivors are gathered in place keeping position order, and
 * then the oldest FP16 slots are quantised until at most W stay FP16.
 * Uses the budgets of the last conf_kv_step (the loose ones before any).  Commits the
 * appends made by conf_kv_attend since the previous call.
 */
int conf_kv_evict_compact(conf_kv_handle *h, conf_kv_stream stream);

/*
 * Launch shapes for replayed steps (for callers that record a decode step into a HIP graph).
 * on != 0: from now on the split counts and kernel variants of conf_kv_attend* and
 * conf_kv_evict_compact are derived from the loose budgets n_loose[l] (the longest a committed
 * unit can be once the first conf_kv_evict_compact has run) instead of the lengths seen so far,
 * so a step recorded now stays valid however the caches grow or shrink later.  A prompt longer
 * than n_loose[l] is still covered while it lasts.  Results do not depend on the setting; short
 * caches run a little slower with it.  on == 0: back to the default.  Host-side only.
 */
int conf_kv_static_plan(conf_kv_handle *h, int32_t on);

/* ---- inspection: these synchronise the device; meant for tests and monitoring ---- */

/* host_len: int32 [L][B] current cache length (appends included); host_n16: int32
 * [L][B][Hkv] FP16 slots per unit, or NULL. */
int conf_kv_lengths(conf_kv_handle *h, int32_t *host_len, int32_t *host_n16);

/* Position-sorted view of one unit into host buffers sized for `capacity` slots; any
 * output pointer may be NULL.  pos int32 [n]; ema fp32 [n]; is_fp16 uint8 [n];
 * k16 / v16: fp16 bits [n][D] (zeros on INT8 slots); k8 / v8: int8 [n][D] (zeros on FP16
 * slots); k_scale / v_scale: fp16 bits [n] (zero on FP16 slots), or the unit's channel scales
 * [D] under CONF_KV_SCALES_CHANNEL (give room for max(capacity, D) values); *n_out = n. */
int conf_kv_export(conf_kv_handle *h, int32_t layer, int32_t b, int32_t kv_head, int32_t *pos,
                   float *ema, uint8_t *is_fp16, uint16_t *k16, uint16_t *v16, int8_t *k8,
                   int8_t *v8, uint16_t *k_scale, uint16_t *v_scale, int32_t *n_out);

/* The inverse of conf_kv_export: replaces the cache of one unit by n slots given in the same
 * position-sorted view (harness re-synchronisation, cache hand-over between handles).
 * pos int32 [n] strictly increasing; ema fp32 [n]; is_fp16 uint8 [n]: zeros (INT8 slots) then
 * ones (FP16 slots), at most fp16_window ones, all ones for an FP16-only cache; k16 / v16 fp16
 * bits [n][D], read on FP16 slots; k8 / v8 int8 [n][D] and k_scale / v_scale fp16 bits [n], read
 * on INT8 slots (a plane no slot reads may be NULL); under CONF_KV_SCALES_CHANNEL k_scale /
 * v_scale are the unit's channel scales [D], always read, finite and >= 0.  0 <= n <= capacity - 1
 * (CONF_KV_ERR_CAPACITY); malformed views give CONF_KV_ERR_INVALID_ARG and leave the unit
 * unchanged.  Not allowed between conf_kv_attend of that layer and the next
 * conf_kv_evict_compact (CONF_KV_ERR_BAD_STATE).  The next token appended to the layer gets a
 * position above every imported one.  Budgets are per (layer, sequence): the caller keeps the
 * kv-heads of one sequence at equal length. */
int conf_kv_import(conf_kv_handle *h, int32_t layer, int32_t b, int32_t kv_head, int32_t n,
                   const int32_t *pos, const float *ema, const uint8_t *is_fp16, const uint16_t *k16,
                   const uint16_t *v16, const int8_t *k8, const int8_t *v8, const uint16_t *k_scale,
                   const uint16_t *v_scale);

/* The tags of the words through which the workgroups of a launch exchange partial results:
 * a launch's tag is a device-side base plus the launch's number since the last
 * conf_kv_evict_compact, which moves the base past them.  Once a base exceeds 0xFF000000 the
 * next conf_kv_evict_compact first clears every exchange word and then starts both bases over
 * at 0 (*clear_pending is 1 in between), so no word ever carries a tag a later launch uses.
 * Outputs (host, each may be NULL): the attention and confidence bases and the pending flag. */
int conf_kv_tag_state(conf_kv_handle *h, uint32_t *attend_base, uint32_t *conf_base, int32_t *clear_pending);

/* Device-side counters since conf_kv_create.  Returns CONF_KV_ERR_DEVICE if any kernel
 * reported an internal error (the counters are still filled in). */
int conf_kv_counters(conf_kv_handle *h, conf_kv_stats *host_stats);

/* Split count conf_kv_attend would use for `layer` now (diagnostics / benchmarks); 1000 + the
 * count when the layer's shape needs the two-launch form (the splits of a unit cannot all be
 * resident at once, or a split's scores do not fit on chip: partial results and raw scores then
 * go through the scratch buffer and a second kernel finishes the attention). */
int conf_kv_attend_splits(conf_kv_handle *h, int32_t layer);

const char *conf_kv_strerror(int status);
/* The hipError_t (as int) of the last failed HIP call on this handle, 0 if none. */
int conf_kv_last_hip_error(conf_kv_handle *h);

/* Measurement aid, not part of the decode path: one launch that reads dev_src[0 .. bytes) once
 * (plain 16-byte loads, `workgroups` workgroups of 256 threads over equal contiguous shares)
 * and folds it into dev_out, uint32 [workgroups], which the caller has zeroed.  What this
 * reaches is the practical ceiling of a streaming read on the device, to set next to the
 * published peak.  bytes a positive multiple of 16, dev_src 16-byte aligned, 1 <= workgroups
 * <= 65536; CONF_KV_ERR_INVALID_ARG otherwise, CONF_KV_ERR_HIP if the launch fails. */
int conf_kv_probe_read(const void *dev_src, size_t bytes, uint32_t *dev_out, int32_t workgroups,
                       conf_kv_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CONF_KV_H */

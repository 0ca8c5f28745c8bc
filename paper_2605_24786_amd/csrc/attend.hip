// Decode attention over the mixed INT8 / FP16 cache with the attention-mass EMA fused in
// (paper: "Tiled attention and mixed precision" -- blockwise read, running max and
// normaliser, dequantisation fused into the read; "Budget and ranker" -- EMA of attention
// mass; Algorithm 1 -- append in FP16, update EMA metadata).
//
// One launch per layer, grid (splits, kv-heads, sequences) -- or (kv-heads, splits, sequences)
// when the number of kv-heads is a multiple of eight, which puts all splits of a unit on one
// XCD -- of 512 threads.  The `splits` workgroups of a unit (b, kv-head) each stream a
// contiguous, byte-balanced slice of the unit's slots once and serve all G query heads of
// the group from that single read:
//
//   stream   running (max, normaliser, output) per head (online softmax); the raw scores
//            s[h][i] of the slice stay in LDS
//   publish  the workgroup's (m, l) per head go out first, then its merged output partial;
//            every published 8-byte word carries the launch's tag (its number since the last
//            commit plus a base kept on the device), so nothing waits for stores to land, no
//            counter is shared, and a recorded launch can be replayed
//   mass     gather the (m, l) words of every split of the unit (a bounded poll on their
//            tags: they all publish at about the same time), form the exact global (M, L),
//            then per slot A_i = sum_h e^{s[h][i]-M[h]} / L[h] and
//            ema_i <- lambda ema_i + (1-lambda) A_i; every split also normalises its share of
//            the unit's output row from the splits' tagged output partials.
//
// Every K/V byte is read once; the scores never leave the chip.  The wait is between
// workgroups of one launch, so the host only launches grids that are co-resident
// (splits * units <= occupancy * CUs) and the wait itself is bounded.
//
// Two streaming bodies share the prologue and the epilogue:
//   * vector-ALU body (any G, any D): lane c of a group of D/16 lanes owns channels
//     [16c, 16c+16) of a slot row, so a wavefront load covers whole rows, contiguous in
//     memory; each lane-group keeps its own running softmax state.
//   * matrix-core body (2 <= G <= 8, D = 128) for the INT8 slots: the G query heads against a
//     32-slot tile are two small contractions (scores: [G x 128] x [128 x 32]; output:
//     [G x 32] x [32 x 128]) issued as v_mfma_f32_16x16x32_f16 with the head dimension
//     padded to 16.  The vector ALU then only converts int8 -> fp16 and keeps the softmax
//     state, which is what lets the kernel stay memory-bound for grouped-query shapes.
//     FP16 slots go through the same contractions in 16-slot tiles, no conversion needed.
//     The same body with all 16 tile rows as query rows serves calls that carry several
//     tokens per sequence (conf_kv_attend_chunk), and a variant of it folds per-channel INT8
//     scales into the query and the output.
// When the splits of a unit cannot all be resident, or a slice's scores do not fit LDS, the
// launch is replaced by two (stream + publish with the scores in device scratch; merge + mass),
// which need no wait inside a kernel.
#include <algorithm>
#include <atomic>
#include <map>
#include <set>
#include <mutex>
#include <tuple>

#include "confkv_dev.h"
#include "launch.h"

namespace confkv {

constexpr int kAttThreads = 512;
constexpr int kAttWaves = 8;

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

// q-th dword of a 128-bit register quad (q is a compile-time constant after unrolling)
__device__ __forceinline__ unsigned dword_of(const int4 &v, int q) {
  return (unsigned)(q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w);
}

// Optional in-kernel phase trace (build with -DCONFKV_TRACE): lane 0 of every wavefront
// notes the 100 MHz wall clock at numbered points, 32 slots per wavefront, in 2 KB of LDS behind
// the kernel's own dynamic LDS (so a time stamp costs no trip to memory and no address
// translation while the kernel runs); the workgroup copies them to the debug buffer as its last
// act.  Compiled out otherwise.
#ifdef CONFKV_TRACE
#define TS_SLOT(k) ts_lds_[a.trace_off / 8 + (threadIdx.x >> 6) * 32 + (k)]
#define TS_INIT()                                                              \
  do {                                                                         \
    extern __shared__ unsigned long long ts_lds_[];                            \
    if (a.dbg && (threadIdx.x & 63) < 32) TS_SLOT(threadIdx.x & 63) = 0ull;     \
  } while (0)
#define TS(k)                                                                  \
  do {                                                                         \
    extern __shared__ unsigned long long ts_lds_[];                            \
    if (a.dbg && (threadIdx.x & 63) == 0) TS_SLOT(k) = wall_clock64();         \
  } while (0)
#define TS_DUMP()                                                              \
  do {                                                                         \
    extern __shared__ unsigned long long ts_lds_[];                            \
    __syncthreads();                                                           \
    if (a.dbg && threadIdx.x < kAttWaves * 32)                                 \
      a.dbg[(size_t)(unit_in_layer(cv, a) * ns + split_index(a)) * kAttWaves * 32 + threadIdx.x] = \
          ts_lds_[a.trace_off / 8 + threadIdx.x];                              \
  } while (0)
#else
#define TS_INIT() do { } while (0)
#define TS(k) do { } while (0)
#define TS_DUMP() do { } while (0)
#endif

// Partials travel between workgroups (possibly on different XCDs, whose L2s are not
// coherent for ordinary accesses) through agent-scope relaxed atomics: such loads and
// stores are coherent across the device by themselves, so no cache-wide release/acquire
// fence (an L2 write-back plus invalidate on this hardware) is ever issued.  No ordering
// between different words is needed either: every published word carries the tag of the
// launch that wrote it, so a reader can tell on its own whether the word it got is current.

// The host passes a launch's number since the last commit and the device completes it: the
// tag base and the position of the next appended token live in cv.ctl, where the commit at the
// end of conf_kv_evict_compact advances them.  A recorded sequence of launches can therefore be
// replayed: nothing that changes from step to step is a launch argument.
// The two words are only requested here: the first instruction that needs one of them (the
// append, the publish at the end of the stream) is where the kernel waits, long after the tile
// requests have gone out.
__device__ __forceinline__ AttendLaunch resolve_launch(const CacheView &cv, AttendLaunch a) {
  a.tag_base = cv.ctl[kCtlTag];
  a.pos_new = (int)cv.ctl[kCtlPos + a.layer];
  return a;
}
__device__ __forceinline__ unsigned tag_of(const AttendLaunch &a) { return a.tag_base + a.epoch; }

// A float that travels with the tag of the launch that wrote it: one 8-byte word, so a
// reader sees value and tag together or neither.
__device__ __forceinline__ void st_tagged(unsigned long long *p, unsigned epoch, float v) {
  __hip_atomic_store(p, ((unsigned long long)epoch << 32) | (unsigned long long)__float_as_uint(v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_tagged(const unsigned long long *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS traffic between lanes of one wavefront: LDS operations of a wavefront execute in
// program order, so a compiler-level barrier is all that is needed between a write phase
// and the read phase that consumes other lanes' data.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Workgroup barrier that orders LDS traffic only: global loads and stores issued before it
// stay in flight across it (__syncthreads waits for them as well).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ void unpack_i8x16(const int4 &r, float (&f)[16]) {
  const int wds[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int e = 0; e < 4; ++e) f[4 * k + e] = (float)((wds[k] << (24 - 8 * e)) >> 24);
  }
}

__device__ __forceinline__ void unpack_h16x16(const int4 &r0, const int4 &r1, float (&f)[16]) {
  half8_t a = __builtin_bit_cast(half8_t, r0), b = __builtin_bit_cast(half8_t, r1);
#pragma unroll
  for (int e = 0; e < 8; ++e) { f[e] = (float)a[e]; f[8 + e] = (float)b[e]; }
}

// ---------------------------------------------------------------------------------------
// Slice bookkeeping shared by both bodies
// ---------------------------------------------------------------------------------------
struct Slice {
  int u, ul, b, g, j;          // unit, unit within the layer, batch, kv-head, split
  int n, n8, h16, n16;         // length with the append, INT8 slots, FP16 ring head, FP16 slots
  int h8;                      // head of the rings anchored at the oldest slot (EMA, position, INT8 rows)
  int lo8, hi8;                // INT8 slots of this split
  int lo16, hi16;              // FP16 slots of this split (slot numbers, >= n8)
  int cnt8, ntok;              // hi8 - lo8, and cnt8 + (hi16 - lo16)
  const int32_t *tab;          // paged layout: the unit's block table (device memory, or a copy in LDS)
  // stash index t in [0, ntok) <-> slot
  __device__ __forceinline__ int slot_of(int t) const { return t < cnt8 ? lo8 + t : lo16 + (t - cnt8); }
};

// floor(x * j / ns) for x = q * ns + r (0 <= r < ns <= 64, j <= ns) without 64-bit division:
// q * j + floor(r * j / ns), the small quotient through one reciprocal (exact: the argument is
// below 4096 and (r j + 1/2) / ns is at least 1/128 away from every integer).
__device__ __forceinline__ int share_cut(unsigned q, unsigned r, int j, float inv_ns) {
  return (int)(q * (unsigned)j + (unsigned)(((float)(r * (unsigned)j) + 0.5f) * inv_ns));
}
// The launch grid is (splits, kv-heads, sequences), or (kv-heads, splits, sequences) when
// a.kv_major is set: workgroups go to the XCDs round-robin in linear order, so with eight
// kv-heads (or a multiple) in front all splits of a unit then run on one XCD.
__device__ __forceinline__ int kv_head_index(const AttendLaunch &a) { return a.kv_major ? blockIdx.x : blockIdx.y; }
__device__ __forceinline__ int split_index(const AttendLaunch &a) { return a.kv_major ? blockIdx.y : blockIdx.x; }
__device__ __forceinline__ int unit_in_layer(const CacheView &cv, const AttendLaunch &a) {
  return blockIdx.z * cv.Hkv + kv_head_index(a);
}

// Every split takes an equal share of the INT8 slots (cut at multiples of 32, the tile of
// the matrix-core body) and an equal share of the FP16 slots, so all splits of a unit carry
// the same mix of work and reach the arrival point together.
// words: the unit's counters when the kernel has requested them already (see unit_words), else null.
__device__ __forceinline__ Slice make_slice(const CacheView &cv, const AttendLaunch &a, int ns, int S,
                                            const int *words = nullptr) {
  Slice s;
  s.g = kv_head_index(a);
  s.b = blockIdx.z;
  s.ul = unit_in_layer(cv, a);
  s.j = split_index(a);
  s.u = a.layer * cv.B * cv.Hkv + s.ul;
  s.tab = cv.pt + (size_t)s.u * cv.npages;
  // The unit's four counters in ONE round trip: lanes 0..3 of every wavefront read one array
  // each with a single load instruction (four scalar loads get spread over the prologue by the
  // compiler, each waiting for the one before).
  const int k4 = threadIdx.x & 3;
  const int32_t *arr = k4 == 0 ? cv.len : k4 == 1 ? cv.n8 : k4 == 2 ? cv.head16 : cv.head8;
  const int mv = words ? *words : arr[s.u];
  const int len = __builtin_amdgcn_readlane(mv, 0), n8 = __builtin_amdgcn_readlane(mv, 1);
  s.h16 = __builtin_amdgcn_readlane(mv, 2);
  s.h8 = __builtin_amdgcn_readlane(mv, 3);
  // an observation call sees the unit as it was when its last query was the newest token
  s.n = (a.observe_first >= 0 ? a.observe_first : len) + a.tq;     // the appended tokens included
  s.n8 = min(n8, s.n);                                             // n8 <= len outside observation calls
  s.n16 = s.n - s.n8;
  const float inv_ns = __builtin_amdgcn_rcpf((float)ns);
  const unsigned q8 = (unsigned)s.n8 / (unsigned)ns, r8 = (unsigned)s.n8 - q8 * (unsigned)ns;
  const unsigned q16 = (unsigned)s.n16 / (unsigned)ns, r16 = (unsigned)s.n16 - q16 * (unsigned)ns;
  s.lo8 = share_cut(q8, r8, s.j, inv_ns) & ~31;
  s.hi8 = s.j == ns - 1 ? s.n8 : share_cut(q8, r8, s.j + 1, inv_ns) & ~31;
  // outside observation calls the tail split's FP16 share is never empty (n16 >= 1), so its
  // owner holds slot n-1
  s.lo16 = s.n8 + share_cut(q16, r16, s.j, inv_ns);
  s.hi16 = s.n8 + share_cut(q16, r16, s.j + 1, inv_ns);
  s.cnt8 = s.hi8 - s.lo8;
  s.ntok = s.cnt8 + (s.hi16 - s.lo16);
  if (s.ntok > S) {                       // cannot happen when the host plan is right
    if (threadIdx.x == 0) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
    s.hi8 = s.lo8; s.cnt8 = 0;
    s.hi16 = min(s.hi16, s.lo16 + S);
    s.ntok = s.hi16 - s.lo16;
  }
  return s;
}

// The workgroup that owns the tail writes the new token into the FP16 ring.
// kSync = false: the caller never reads the appended row back in this launch (it takes the new
// token from the call's arguments), so nothing has to wait for the stores.
template <int D, bool kSync = true>
__device__ __forceinline__ void append_new_token(const CacheView &cv, const AttendLaunch &a,
                                                 const Slice &s, int ns) {
  if (s.j != ns - 1 || a.observe_first >= 0) return;
  const int tid = threadIdx.x;
  constexpr int PPR = D / 8;                        // 16-byte pieces per row
  // token t of the call: K/V rows [B][tq][Hkv][D] -> FP16 ring row of slot n - tq + t
  for (int i = tid; i < 2 * a.tq * PPR; i += kAttThreads) {
    const int which = i / (a.tq * PPR), r = i % (a.tq * PPR), t = r / PPR, c = r % PPR;
    const int row = ring_row(s.h16, s.n16 - a.tq + t, cv.cap16);
    const __half *src = (which ? a.vnew : a.knew) + (((size_t)s.b * a.tq + t) * cv.Hkv + s.g) * D;
    __half *dst = (which ? cv.v16 : cv.k16) + ((size_t)s.u * cv.cap16 + row) * D;
    ((int4 *)dst)[c] = ((const int4 *)src)[c];
  }
  if (tid < a.tq)
    cv.pos[(size_t)s.u * cv.cap + slot_row(cv, s.tab, s.h8, s.n8, s.h16, s.n - a.tq + tid)] = a.pos_new + tid;
  if constexpr (kSync) __syncthreads();
}

// ---------------------------------------------------------------------------------------
// Vector-ALU streaming body
// ---------------------------------------------------------------------------------------

// Running softmax state of one slot lane-group: per head the maximum so far, the
// normaliser and this lane's 16 channels of the un-normalised output.
template <int G>
struct Stream {
  float m[G], l[G], acc[G][16];
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m[h] = -INFINITY;
      l[h] = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[h][e] = 0.f;
    }
  }
};

// Fold a batch of R slots into the running state.  s[r][h] are the slots' scores,
// vf[r] the value channels owned by this lane, vsc[r] the value scale, ok[r] validity.
template <int G, int R>
__device__ __forceinline__ void fold_batch(Stream<G> &st, const float (&s)[R][G],
                                           const float (&vf)[R][16], const float (&vsc)[R],
                                           const bool (&ok)[R]) {
  const float NEG = -INFINITY;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float bm = NEG;
#pragma unroll
    for (int r = 0; r < R; ++r) bm = ok[r] ? fmaxf(bm, s[r][h]) : bm;
    const float mn = fmaxf(st.m[h], bm);
    const float corr = (mn == NEG) ? 1.f : __expf(st.m[h] - mn);
    st.m[h] = mn;
    float p[R], lsum = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      p[r] = ok[r] ? __expf(s[r][h] - mn) : 0.f;
      lsum += p[r];
      p[r] *= vsc[r];
    }
    st.l[h] = fmaf(st.l[h], corr, lsum);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float t = st.acc[h][e] * corr;
#pragma unroll
      for (int r = 0; r < R; ++r) t = fmaf(p[r], vf[r][e], t);
      st.acc[h][e] = t;
    }
  }
}

template <int D, int G>
__device__ __forceinline__ void load_q_slices(const CacheView &cv, const AttendLaunch &a,
                                              const Slice &sl, float (&qf)[G][16]) {
  constexpr int LPT = D / 16;
  const int c = (threadIdx.x & 63) % LPT;
  const int Hq = cv.Hkv * G;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const int4 *qp = (const int4 *)(a.q + ((size_t)(sl.b * Hq + sl.g * G + h)) * D + c * 16);
    unpack_h16x16(qp[0], qp[1], qf[h]);
  }
}

// INT8 slots [lo, hi8) on the vector ALU.
template <int D, int G>
__device__ __forceinline__ void stream_int8_valu(const CacheView &cv, const Slice &sl, float sm,
                                                 const float (&qf)[G][16], Stream<G> &st,
                                                 float *stash, int S) {
  constexpr int LPT = D / 16, TW = kWave / LPT, TB = kAttWaves * TW, R8 = 4;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane % LPT, ts = lane / LPT;
  const int8_t *K8 = cv.k8 + (size_t)sl.u * cv.cap8 * D;
  const int8_t *V8 = cv.v8 + (size_t)sl.u * cv.cap8 * D;
  // per-channel scales: the caller folded the K scales into qf and applies the V scales to the
  // accumulator afterwards; every slot then has the factors (sm, 1).  The per-token loads stay
  // branch-free on element 0 of the unit's scale plane.
  const bool chan = cv.chan != 0;
  const __half *KS = cv.ks + (size_t)sl.u * (chan ? D : cv.cap8);
  const __half *VS = cv.vs + (size_t)sl.u * (chan ? D : cv.cap8);
  for (int base = sl.lo8; base < sl.hi8; base += TB * R8) {
    int4 kr[R8], vr[R8];
    unsigned short ksh[R8], vsh[R8];
    float vsc[R8];
    bool ok[R8];
    // branch-free loads (rows past the slice re-read its last row and are masked below), so
    // that all of a trip's loads are in flight before the first one is waited for
#pragma unroll
    for (int r = 0; r < R8; ++r) {
      const int i = base + r * TB + w * TW + ts;
      ok[r] = i < sl.hi8;
      const int ic = ring_row_u(sl.h8, ok[r] ? i : sl.hi8 - 1, cv.cap8);
      kr[r] = *(const int4 *)(K8 + (size_t)ic * D + c * 16);
      vr[r] = *(const int4 *)(V8 + (size_t)ic * D + c * 16);
      ksh[r] = ((const unsigned short *)KS)[chan ? 0 : ic];
      vsh[r] = ((const unsigned short *)VS)[chan ? 0 : ic];
    }
    float s[R8][G], vf[R8][16];
#pragma unroll
    for (int r = 0; r < R8; ++r) {
      float kf[16];
      unpack_i8x16(kr[r], kf);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc = fmaf(qf[h][e], kf[e], acc);
        s[r][h] = acc;
      }
    }
#pragma unroll
    for (int m = 1; m < LPT; m <<= 1) {
#pragma unroll
      for (int r = 0; r < R8; ++r)
#pragma unroll
        for (int h = 0; h < G; ++h) s[r][h] += __shfl_xor(s[r][h], m, kWave);
    }
#pragma unroll
    for (int r = 0; r < R8; ++r) {
      const int i = base + r * TB + w * TW + ts;
      const float f = chan ? sm : __half2float(__ushort_as_half(ksh[r])) * sm;
      vsc[r] = chan ? 1.f : __half2float(__ushort_as_half(vsh[r]));
#pragma unroll
      for (int h = 0; h < G; ++h) {
        s[r][h] *= f;
        if (ok[r] && c == 0) stash[h * S + (i - sl.lo8)] = s[r][h];
      }
      unpack_i8x16(vr[r], vf[r]);
    }
    fold_batch<G, R8>(st, s, vf, vsc, ok);
  }
}

// FP16 ring slots [lo16, hi) on the vector ALU.
template <int D, int G>
__device__ __forceinline__ void stream_fp16_valu(const CacheView &cv, const Slice &sl, float sm,
                                                 const float (&qf)[G][16], Stream<G> &st,
                                                 float *stash, int S) {
  constexpr int LPT = D / 16, TW = kWave / LPT, TB = kAttWaves * TW, R16 = 2;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane % LPT, ts = lane / LPT;
  const __half *K16 = cv.k16 + (size_t)sl.u * cv.cap16 * D;
  const __half *V16 = cv.v16 + (size_t)sl.u * cv.cap16 * D;
  for (int base = sl.lo16; base < sl.hi16; base += TB * R16) {
    int4 kr[R16][2], vr[R16][2];
    float vsc[R16];
    bool ok[R16];
#pragma unroll
    for (int r = 0; r < R16; ++r) {
      const int i = base + r * TB + w * TW + ts;
      ok[r] = i < sl.hi16;
      vsc[r] = 1.f;
      const int ic = ok[r] ? i : sl.hi16 - 1;
      const size_t off = (size_t)ring_row(sl.h16, ic - sl.n8, cv.cap16) * D + c * 16;
      const int4 *pk = (const int4 *)(K16 + off), *pv = (const int4 *)(V16 + off);
      kr[r][0] = pk[0]; kr[r][1] = pk[1];
      vr[r][0] = pv[0]; vr[r][1] = pv[1];
    }
    float s[R16][G], vf[R16][16];
#pragma unroll
    for (int r = 0; r < R16; ++r) {
      float kf[16];
      unpack_h16x16(kr[r][0], kr[r][1], kf);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc = fmaf(qf[h][e], kf[e], acc);
        s[r][h] = acc;
      }
    }
#pragma unroll
    for (int m = 1; m < LPT; m <<= 1) {
#pragma unroll
      for (int r = 0; r < R16; ++r)
#pragma unroll
        for (int h = 0; h < G; ++h) s[r][h] += __shfl_xor(s[r][h], m, kWave);
    }
#pragma unroll
    for (int r = 0; r < R16; ++r) {
      const int i = base + r * TB + w * TW + ts;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        s[r][h] *= sm;
        if (ok[r] && c == 0) stash[h * S + sl.cnt8 + (i - sl.lo16)] = s[r][h];
      }
      unpack_h16x16(vr[r][0], vr[r][1], vf[r]);
    }
    fold_batch<G, R16>(st, s, vf, vsc, ok);
  }
}

// Merge the slot lane-groups of a wavefront and store the wavefront's partial
// (m, l, o[G][D]) as entry `pidx` of the workgroup's LDS partial arrays.
template <int D, int G>
__device__ __forceinline__ void store_stream_partial(Stream<G> &st, int pidx, float *wm, float *wl,
                                                     float *wo_p) {
  constexpr int LPT = D / 16;
  const int lane = threadIdx.x & 63;
  const int c = lane % LPT, ts = lane / LPT;
  const float NEG = -INFINITY;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float mw = wave_max(st.m[h]);
    const float f = (st.m[h] == NEG) ? 0.f : __expf(st.m[h] - mw);
    float l = st.l[h] * f;
#pragma unroll
    for (int m = LPT; m < kWave; m <<= 1) l += __shfl_xor(l, m, kWave);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float t = st.acc[h][e] * f;
#pragma unroll
      for (int m = LPT; m < kWave; m <<= 1) t += __shfl_xor(t, m, kWave);
      st.acc[h][e] = t;
    }
    if (lane == 0) { wm[pidx * G + h] = mw; wl[pidx * G + h] = l; }
    if (ts == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) wo_p[h * D + c * 16 + e] = st.acc[h][e];
    }
  }
}

// Arrival and the gather of the softmax statistics in one: every split publishes its (m, l)
// per head as words tagged with the launch's tag (tag_of: the launch's number plus the base
// on the device), and thread k polls word k of the unit until the tag is this launch's, then
// drops the value into LDS.  The output partials travel as tagged words of their own and are
// polled where they are used, so seeing a split's statistics says nothing about its partial.
// Nobody does a read-modify-write, so arrivals do not serialise at the memory side.  The wait
// is bounded; false means it expired (counted as a device error).  Contains a workgroup
// barrier; *s_ok must have been set to 1 before the barrier that precedes the call.
template <int G>
__device__ __forceinline__ bool collect_ml(const CacheView &cv, const AttendLaunch &a, const Slice &sl,
                                           int ns, float *pml, int *s_ok) {
  const int tid = threadIdx.x;
  const unsigned long long *words = a.part_ml + (size_t)sl.ul * a.max_splits * G * 2;
  for (int base = 0; base < ns * G * 2; base += kAttThreads) {
    const int idx = base + tid;
    const bool mine = idx < ns * G * 2;
    bool here = !mine;
    int spins = 0;
    for (;;) {
      if (!here) {
        const unsigned long long wv = ld_tagged(&words[idx]);
        if ((unsigned)(wv >> 32) == tag_of(a)) {
          pml[idx] = __uint_as_float((unsigned)wv);
          here = true;
        }
      }
      if (__builtin_amdgcn_ballot_w64(!here) == 0ull) break;
      __builtin_amdgcn_s_sleep(1);
      if (++spins > a.spin_limit) {
        if (!here) *s_ok = 0;
        break;
      }
    }
  }
  __syncthreads();
  if (*s_ok == 0 && tid == 0) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
  return *s_ok != 0;
}

// e^x for x <= 0 (-inf included, which gives 0) to about one ulp: 2^(x log2 e) with the product
// carried in two floats, so the hardware exponential sees an argument without rounding error.
// No range checks: the result cannot overflow, and below 2^-126 it may flush to zero.
__device__ __forceinline__ float exp_nonpos(float x) {
  x = fmaxf(x, -100.0f);
  const float kHi = 1.44269502e+00f, kLo = 1.92596299e-08f;          // log2(e) = kHi + kLo
  const float ph = x * kHi;
  const float pl = fmaf(x, kLo, fmaf(x, kHi, -ph));
  const float r = __builtin_amdgcn_exp2f(ph);
  return fmaf(r, pl * 0.693147181f, r);
}
// 1 / x for a positive, finite double to about 1e-15 relative: the fp32 reciprocal estimate and two
// Newton steps (a correctly rounded division costs ten times the instructions and nothing
// downstream is that exact).
__device__ __forceinline__ double recip_pos(double x) {
  double r = (double)__builtin_amdgcn_rcpf((float)x);
  r = r * (2.0 - x * r);
  return r * (2.0 - x * r);
}

// Query row r of a unit is (token r / gq of the call, head r % gq of the group); rows past
// tq * gq are padding.  Element e = r * D + d of the unit's [rows][D] output lives at
// out[b][token][g * gq + head][d].
__device__ __forceinline__ size_t out_index(const CacheView &cv, const Slice &sl, int tq, int gq,
                                            int e, int D) {
  // (32-bit arithmetic: the output of one call stays far below 2^31 elements)
  const unsigned r = (unsigned)e / (unsigned)D, d = (unsigned)e - r * (unsigned)D;
  const unsigned t = r / (unsigned)gq, hq = r - t * (unsigned)gq;
  return (size_t)(((((unsigned)sl.b * (unsigned)tq + t) * (unsigned)cv.Hkv + (unsigned)sl.g) * (unsigned)gq + hq) * (unsigned)D + d);
}
// Weight of row r's mass in the importance update of a call with tq tokens:
// lambda^(tq - 1 - token), 0 for padding rows; for tq = 1 it is exactly 1.
__device__ __forceinline__ double row_weight(const AttendLaunch &a, int tq, int gq, int r) {
  const int t = r / gq;
  if (t >= tq) return 0.0;
  double w = 1.0;
  for (int k = t + 1; k < tq; ++k) w *= (double)a.ema_decay;
  return w;
}

// ---------------------------------------------------------------------------------------
// Epilogue shared by both bodies.  On entry wm/wl/wo hold NP per-wavefront partials
// (after a workgroup barrier): partial k is [G][D] floats at
// wo + (k % kAttWaves) * WSTR + (k / kAttWaves) * G * D; stash holds the slice's raw scores.
// kPhase 0: the whole epilogue in one kernel (merge, publish, wait for the unit's other splits,
// gather, EMA, output).  kPhase 1: merge and publish only; kPhase 2: gather, EMA and output in a
// later launch, which needs no wait (wm/wl are unused and wo is [ns][G][2] floats of LDS) --
// the pair serves shapes whose splits cannot all be resident at once.
// ---------------------------------------------------------------------------------------
template <int D, int G, int NP, int WSTR, int kPhase = 0, int DR = D>
__device__ __forceinline__ void attend_epilogue(const CacheView &cv, const AttendLaunch &a,
                                                const Slice &sl, int ns, int S, float *stash,
                                                float *wm, float *wl, float *wo, float *gm,
                                                double *ginv, int *s_ok) {
  const int tid = threadIdx.x;
  const float NEG = -INFINITY;
  // more than 8 rows only occur in multi-token calls; otherwise rows are the heads of one token
  const int tq = G > 8 ? a.tq : 1, gq = G > 8 ? a.gq : G;
  unsigned long long *ml = a.part_ml + ((size_t)sl.ul * a.max_splits + sl.j) * G * 2;
  unsigned long long *po = a.part_o + ((size_t)sl.ul * a.max_splits + sl.j) * G * D;
  // the EMA values this thread will update: requested now, needed after the wait
  constexpr int kPre = kPhase == 0 ? 4 : 0;
  const bool exchange = kPhase != 0 || ns > 1;       // partials go through device memory
  float *EMA = cv.ema + (size_t)sl.u * cv.cap;
  float ema_old[kPre + 1];
#pragma unroll
  for (int k = 0; k < kPre; ++k) {
    // branch-free (a slot past the slice re-reads its last one; the appended token's slot
    // holds a stale value): the uses below mask both cases
    const int slot = sl.slot_of(max(0, min(tid + k * kAttThreads, sl.ntok - 1)));   // an empty slice reads slot lo16 < n
    ema_old[k] = EMA[slot_row(cv, sl.tab, sl.h8, sl.n8, sl.h16, slot)];
  }
  // The softmax statistics go out first: thread h merges row h's (m, l) over the wavefront
  // partials (the same operations, in the same order, as the output merge below) and publishes
  // them at once, so their trip to the unit's other splits runs behind the output merge.
  if (kPhase != 2 && exchange && tid < G) {
    float M = NEG;
#pragma unroll
    for (int k = 0; k < NP; ++k) M = fmaxf(M, wm[k * G + tid]);
    float l = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
      const float mk = wm[k * G + tid];
      const bool live = mk > NEG;
      l = fmaf(live ? wl[k * G + tid] : 0.f, live ? __expf(mk - M) : 0.f, l);
    }
    if (!a.withhold || sl.j != 0) {                   // (test hook: split 0 keeps its words to itself)
      st_tagged(&ml[tid * 2], tag_of(a), M);
      st_tagged(&ml[tid * 2 + 1], tag_of(a), l);
    }
  }
  // workgroup merge of the per-wavefront output partials: kEPT channels per thread, each
  // published as a word that carries the launch's epoch, so that nobody has to wait for the
  // stores to land before announcing them
  constexpr int kEPT = G * D > kAttThreads ? 2 : 1;
  if (kPhase != 2)
  for (int idx = kEPT * tid; idx < G * D; idx += kEPT * kAttThreads) {
    const int h = idx / D;
    // branch-free, so that all LDS reads are in flight together; an empty partial (m = -inf)
    // may hold anything and enters with weight zero through the selects
    float mk[NP], lk[NP], ok2[NP][kEPT];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
      mk[k] = wm[k * G + h];
      lk[k] = wl[k * G + h];
      // partial k belongs to wavefront k % kAttWaves
      const float *src = &wo[(k % kAttWaves) * WSTR + (k / kAttWaves) * G * D + idx];
      if constexpr (kEPT == 2) {
        const float2 t2 = *(const float2 *)src;
        ok2[k][0] = t2.x;
        ok2[k][kEPT - 1] = t2.y;
      } else {
        ok2[k][0] = *src;
      }
    }
    float M = NEG;
#pragma unroll
    for (int k = 0; k < NP; ++k) M = fmaxf(M, mk[k]);
    float o[kEPT] = {}, l = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
      const bool live = mk[k] > NEG;
      const float f = live ? __expf(mk[k] - M) : 0.f;
#pragma unroll
      for (int e = 0; e < kEPT; ++e) o[e] = fmaf(live ? ok2[k][e] : 0.f, f, o[e]);
      l = fmaf(live ? lk[k] : 0.f, f, l);
    }
    if (!exchange) {
      // a unit with a single split is complete here: same arithmetic as the general merge
      // below (weight e^0 = 1), without the trip through device memory
      const double inv = recip_pos((double)l);
#pragma unroll
      for (int e = 0; e < kEPT; ++e) {
        // (DR < D: the matrix-core body pads a 64-channel head to its 128-channel tiles)
        if (h < tq * gq && a.out && idx + e - h * D < DR)
          a.out[out_index(cv, sl, tq, gq, h * DR + (idx + e - h * D), DR)] = __float2half_rn((float)((double)o[e] * inv));
      }
      if (idx % D == 0) { gm[h] = M; ginv[h] = inv; ginv[G + h] = inv * row_weight(a, tq, gq, h); }
    } else {
#pragma unroll
      for (int e = 0; e < kEPT; ++e) st_tagged(&po[idx + e], tag_of(a), o[e]);
    }
  }
  TS(19);
  if (kPhase == 1) return;
  const unsigned long long *pou = a.part_o + (size_t)sl.ul * a.max_splits * G * D;
  float *pml = wo;                                   // [ns][G][2], reuses the merge buffer
  // Output merge: this split normalises `per` elements of the unit's [G][D] output.  The ns
  // partial values of one element sit in gs consecutive lanes (gs = ns rounded up to a power
  // of two), so one load per thread fetches them in a single round trip whatever ns is, and a
  // few lane shuffles add them up.
  const int per = (G * D + ns - 1) / ns;
  int gs = 1;
  while (gs < ns) gs <<= 1;                          // <= 64: groups never straddle a wavefront
  const int epp = kAttThreads / gs;                  // elements per pass over the workgroup
  const int os = tid % gs, oe = tid / gs;            // this thread's split and element within a pass
  unsigned long long opre = 0ull, opre2 = 0ull;
  if (exchange) {
    if (kPhase == 0) {
      if (tid == 0) *s_ok = 1;
      lds_barrier();                                 // the merge has read the buffer the statistics land in
      TS(20);
      if (!collect_ml<G>(cv, a, sl, ns, pml, s_ok)) return;
      TS(21);
    } else {
      // second launch: every word of the unit was written by the first one
      const unsigned long long *words = a.part_ml + (size_t)sl.ul * a.max_splits * G * 2;
      for (int idx = tid; idx < ns * G * 2; idx += kAttThreads) pml[idx] = __uint_as_float((unsigned)ld_tagged(&words[idx]));
      __syncthreads();
    }
    // this split's share of the unit's output partials: a first look now, checked (and asked for
    // again if the word is not this launch's yet) only after the importance update
    if (os < ns && oe < per && sl.j * per + oe < G * D)
      opre = ld_tagged(&pou[(size_t)os * G * D + sl.j * per + oe]);
    // global (M, L) of head h by wavefront h: one lane per split
    for (int h = tid >> 6; h < G; h += kAttWaves) {
      const int sp = tid & 63;
      const float ms = sp < ns ? pml[(sp * G + h) * 2] : NEG;
      // only the first gs lanes hold partials: log2(gs) exchange steps instead of six
      const float ls = sp < ns ? pml[(sp * G + h) * 2 + 1] : 0.f;
      float M = ms;
      // (fixed lane distances up to four splits, so the exchanges need no index registers)
      if (gs <= 4) {
        if (gs > 2) M = fmaxf(M, __shfl_xor(M, 2, kWave));
        if (gs > 1) M = fmaxf(M, __shfl_xor(M, 1, kWave));
      } else {
        for (int m = gs >> 1; m >= 1; m >>= 1) M = fmaxf(M, __shfl_xor(M, m, kWave));
      }
      const float es = ms > NEG ? exp_nonpos(ms - M) : 0.f;        // an empty partial weighs nothing
      double L = (double)es * (double)ls;
      if (gs <= 4) {
        if (gs > 2) L += __shfl_xor(L, 2, kWave);
        if (gs > 1) L += __shfl_xor(L, 1, kWave);
      } else {
        for (int m = gs >> 1; m >= 1; m >>= 1) L += __shfl_xor(L, m, kWave);
      }
      const double inv = recip_pos(L);
      if (sp == 0) { gm[h] = M; ginv[h] = inv; ginv[G + h] = inv * row_weight(a, tq, gq, h); }
      // what split sp's output partial of this row is multiplied by, in place of its maximum
      if (sp < ns) pml[(sp * G + h) * 2] = es * (float)inv;
    }
    lds_barrier();                                   // (the look at the output partials stays in flight)
    // a second look, half a round trip later: by now the slowest split's words have landed, and
    // this one too travels behind the importance update
    if (os < ns && oe < per && sl.j * per + oe < G * D)
      opre2 = ld_tagged(&pou[(size_t)os * G * D + sl.j * per + oe]);
  } else {
    __syncthreads();
  }
  TS(22);
  // ---- this split normalises its share of the unit's output (online-softmax merge) ----
  auto finish_output = [&]() {
  if (exchange) {
      for (int base = 0; base < per; base += epp) {
        const int e = sl.j * per + base + oe;                          // element of the [G][D] output
        const bool valid = os < ns && base + oe < per && e < G * D;
        const unsigned long long *src = &pou[(size_t)os * G * D + (valid ? e : 0)];
        unsigned long long wv = base == 0 ? ((unsigned)(opre >> 32) == tag_of(a) ? opre : opre2) : (valid ? ld_tagged(src) : 0ull);
        // a word that is not this launch's yet is asked for again (bounded); in a second launch
        // every word is there
        bool here = !valid || (unsigned)(wv >> 32) == tag_of(a);
        for (int spins = 0; __builtin_amdgcn_ballot_w64(!here) != 0ull; ++spins) {
          if (spins > a.spin_limit) break;
          __builtin_amdgcn_s_sleep(1);
          if (!here) {
            wv = ld_tagged(src);
            here = (unsigned)(wv >> 32) == tag_of(a);
          }
        }
        const unsigned long long missing = __builtin_amdgcn_ballot_w64(!here);
        if (missing) {                                                 // the wait expired: no output from this wavefront
          if ((tid & 63) == __builtin_ctzll(missing)) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
          continue;
        }
        const float v = __uint_as_float((unsigned)wv);
        const int h = valid ? e / D : 0;
        const float wgt = valid ? pml[(os * G + h) * 2] : 0.f;         // e^{m_s - M} / L of that split and row
        float c = wgt > 0.f ? v * wgt : 0.f;                           // (an empty partial may hold anything)
        if (gs <= 4) {                                                 // the usual case: two fixed exchanges
          if (gs > 2) c += __shfl_xor(c, 2, kWave);
          if (gs > 1) c += __shfl_xor(c, 1, kWave);
        } else {
          for (int m = gs >> 1; m >= 1; m >>= 1) c += __shfl_xor(c, m, kWave);
        }
        if (valid && os == 0 && h < tq * gq && a.out && e - h * D < DR)
          a.out[out_index(cv, sl, tq, gq, h * DR + (e - h * D), DR)] = __float2half_rn(c);
      }
    }
  };
  // ---- mass + EMA of the slice ----
  // a <- lambda^tq a + gain * sum over the rows of lambda^(tq-1-token) p; ginv[G + h] holds
  // row h's weight over its normaliser.  Slots appended by this call start at 0.
  double lam = 1.0;
  for (int k = 0; k < tq; ++k) lam *= (double)a.ema_decay;
  const double oml = a.mass_gain;
  const double *gw = ginv + G;
  const int first_new = sl.n - tq;
  // The new values of the first kPre slots per thread stay in registers until the output is
  // out: a store between the look at the output partials and its use would make that use wait
  // for the store's acknowledgement as well (loads and stores share one in-order counter).
#pragma unroll
  for (int k = 0; k < kPre; ++k) {
    const int t = tid + k * kAttThreads;
    if (t < sl.ntok) {
      double A = 0.0;
#pragma unroll
      for (int h = 0; h < G; ++h) A += (double)exp_nonpos(stash[h * S + t] - gm[h]) * gw[h];
      const int slot = sl.slot_of(t);
      const double old = (slot >= first_new) ? 0.0 : (double)ema_old[k];   // a new token starts at 0
      EMA[slot_row(cv, sl.tab, sl.h8, sl.n8, sl.h16, slot)] = (float)(lam * old + oml * A);
    }
  }
  TS(30);
  // the rest of the slice in batches of kBatch slots per thread: branch-free loads first (a
  // slot past the slice re-reads its last one), so a long slice costs one round trip per
  // batch, not one per slot
  constexpr int kBatch = 4;
  for (int t0 = tid + kPre * kAttThreads; t0 < sl.ntok; t0 += kBatch * kAttThreads) {
    float old[kBatch];
    int row[kBatch];
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      row[k] = slot_row(cv, sl.tab, sl.h8, sl.n8, sl.h16, sl.slot_of(min(t0 + k * kAttThreads, sl.ntok - 1)));
      old[k] = EMA[row[k]];
    }
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const int t = t0 + k * kAttThreads;
      if (t < sl.ntok) {
        double A = 0.0;
#pragma unroll
        for (int h = 0; h < G; ++h) A += (double)exp_nonpos(stash[h * S + t] - gm[h]) * gw[h];
        const double prev = (sl.slot_of(t) >= first_new) ? 0.0 : (double)old[k];   // a new token starts at 0
        EMA[row[k]] = (float)(lam * prev + oml * A);
      }
    }
  }
  TS(23);
  finish_output();
  TS(31);
}

// ---------------------------------------------------------------------------------------
// Kernel 1: vector-ALU body for every slot
// ---------------------------------------------------------------------------------------
// kSpill: the first launch of the two-launch form -- the slice's raw scores go to device
// scratch instead of LDS and the kernel ends after publishing its partial.
template <int D, int G, bool kSpill = false>
__global__ __launch_bounds__(kAttThreads) void attend_kernel(const int32_t *w_len, const int32_t *w_n8, const int32_t *w_h16, const int32_t *w_h8, int w_unit0, int w_hkv, int w_kvm, CacheView cv, AttendLaunch a_in, int ns,
                                                             int S) {
  const AttendLaunch a = resolve_launch(cv, a_in);
  constexpr int NP = kAttWaves;
  extern __shared__ __align__(16) float smem[];
  float *stash = kSpill ? a.spill + ((size_t)unit_in_layer(cv, a) * ns + split_index(a)) * G * S
                        : smem;                 // [G][S] raw scores of the slice
  float *wo = smem + (kSpill ? 0 : (size_t)G * S);   // [NP][G][D] per-wave un-normalised output
  float *wm = wo + NP * G * D;                  // [NP][G] per-wave maximum
  float *wl = wm + NP * G;                      // [NP][G] per-wave normaliser
  float *gm = wl + NP * G;                      // [G] global maximum
  double *ginv = (double *)(gm + G + (G & 1));  // [2 G]: 1 / global normaliser, the same times the row's mass weight
  __shared__ int s_ok;

  const Slice sl = make_slice(cv, a, ns, S);
  append_new_token<D>(cv, a, sl, ns);

  Stream<G> st;
  st.reset();
  float qf[G][16];
  load_q_slices<D, G>(cv, a, sl, qf);
  if (cv.chan) {
    // per-channel scales: fold the K scales of this lane's 16 channels into the query for the
    // INT8 slots, scale the accumulated INT8 output by the V scales, reload the plain query
    constexpr int LPT = D / 16;
    const int c = (threadIdx.x & 63) % LPT;
    float sc[16];
    const int4 *kp = (const int4 *)(cv.ks + (size_t)sl.u * D + c * 16);
    unpack_h16x16(kp[0], kp[1], sc);
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < 16; ++e) qf[h][e] *= sc[e];
    stream_int8_valu<D, G>(cv, sl, a.sm_scale, qf, st, stash, S);
    const int4 *vp = (const int4 *)(cv.vs + (size_t)sl.u * D + c * 16);
    unpack_h16x16(vp[0], vp[1], sc);
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < 16; ++e) st.acc[h][e] *= sc[e];
    load_q_slices<D, G>(cv, a, sl, qf);
  } else {
    stream_int8_valu<D, G>(cv, sl, a.sm_scale, qf, st, stash, S);
  }
  stream_fp16_valu<D, G>(cv, sl, a.sm_scale, qf, st, stash, S);
  store_stream_partial<D, G>(st, threadIdx.x >> 6, wm, wl, wo + (threadIdx.x >> 6) * G * D);
  __syncthreads();
  attend_epilogue<D, G, NP, G * D, kSpill ? 1 : 0>(cv, a, sl, ns, S, stash, wm, wl, wo, gm, ginv, &s_ok);
}

// Second launch of the two-launch form: same grid; merges the published partials of the unit,
// updates the EMA of its slice from the spilled scores and normalises its share of the output.
template <int D, int G, int DR = D>
__global__ __launch_bounds__(kAttThreads) void attend_finish_kernel(const int32_t *w_len, const int32_t *w_n8, const int32_t *w_h16, const int32_t *w_h8, int w_unit0, int w_hkv, int w_kvm, CacheView cv, AttendLaunch a_in, int ns,
                                                                    int S) {
  const AttendLaunch a = resolve_launch(cv, a_in);
  extern __shared__ __align__(16) float smem[];
  float *pml = smem;                            // [ns][G][2]
  float *gm = pml + (size_t)ns * G * 2;         // [G]
  double *ginv = (double *)(gm + G + (G & 1));  // [2 G]
  __shared__ int s_ok;
  const Slice sl = make_slice(cv, a, ns, S);
  float *stash = a.spill + ((size_t)unit_in_layer(cv, a) * ns + split_index(a)) * G * S;
  attend_epilogue<D, G, 1, 0, 2, DR>(cv, a, sl, ns, S, stash, nullptr, nullptr, pml, gm, ginv, &s_ok);
}

// ---------------------------------------------------------------------------------------
// Kernel 2: matrix-core body (D = 128, or D = 64 padded to the same tiles)
// ---------------------------------------------------------------------------------------
constexpr int kTile = 32;              // slots per wavefront tile
constexpr int kKRow = 128 + 16;        // LDS row stride of the INT8 K tile (bytes)
constexpr int kKRow16 = 256 + 16;      // LDS row stride of the 16-slot FP16 K tile (bytes)
constexpr int kVRow = 32 + 4;          // LDS row stride of the transposed V tile (bytes)
// Rows of the transposed V tile come in groups of 16 channels.  A store instruction has its
// lanes in 8 different groups (16 rows = 144 dwords apart: only two different banks), so group g
// is shifted by 20 g dwords: the groups then start 164 dwords = 4 banks (mod 32) apart and the
// lanes of a half wavefront fall into 32 different banks.  A load instruction stays inside
// one group and is not affected.
__host__ __device__ constexpr int kVSkew(int group) { return 80 * group; }
constexpr int kVBytes = 128 * kVRow + kVSkew(7);   // rows plus the largest shift
constexpr int kPRow = 32 + 8;          // LDS row stride of the probability tile (halfs)
constexpr int kTileBytes = kTile * kKRow + kVBytes + 16 * kPRow * 2;   // per wavefront

// 4 int8 (one dword) -> 4 fp16 (two dwords), exact: c ^ 0x80 is c + 128 as an unsigned byte,
// 0x6400 | byte is the fp16 number 1024 + byte, and subtracting 1152 leaves c.
__device__ __forceinline__ void cvt_i8x4_f16x4(unsigned w, half2_t &lo, half2_t &hi) {
  const unsigned x = w ^ 0x80808080u;
  const unsigned a = __builtin_amdgcn_perm(x, 0x64646464u, 0x00050004u);
  const unsigned b = __builtin_amdgcn_perm(x, 0x64646464u, 0x00070006u);
  const half2_t bias = {(_Float16)1152.0f, (_Float16)1152.0f};
  lo = __builtin_bit_cast(half2_t, a) - bias;
  hi = __builtin_bit_cast(half2_t, b) - bias;
}

// Same without the subtraction: the fp16 numbers c + 1152.  Used for the value operand, where
// the constant is taken out again after the contraction (sum_i p_i (v_i + 1152) =
// sum_i p_i v_i + 1152 sum_i p_i) at a cost of one accumulated sum per head.
constexpr float kCodeBias = 1152.0f;
__device__ __forceinline__ half8_t cvt_i8x8_f16x8_biased(unsigned w0, unsigned w1) {
  const unsigned x0 = w0 ^ 0x80808080u, x1 = w1 ^ 0x80808080u;
  uint4 r;
  r.x = __builtin_amdgcn_perm(x0, 0x64646464u, 0x00050004u);
  r.y = __builtin_amdgcn_perm(x0, 0x64646464u, 0x00070006u);
  r.z = __builtin_amdgcn_perm(x1, 0x64646464u, 0x00050004u);
  r.w = __builtin_amdgcn_perm(x1, 0x64646464u, 0x00070006u);
  return __builtin_bit_cast(half8_t, r);
}

__device__ __forceinline__ half8_t cvt_i8x8_f16x8(unsigned w0, unsigned w1) {
  half2_t p0, p1, p2, p3;
  cvt_i8x4_f16x4(w0, p0, p1);
  cvt_i8x4_f16x4(w1, p2, p3);
  half8_t r;
  r[0] = p0[0]; r[1] = p0[1]; r[2] = p1[0]; r[3] = p1[1];
  r[4] = p2[0]; r[5] = p2[1]; r[6] = p3[0]; r[7] = p3[1];
  return r;
}

// max / sum over the 16 lanes of a DPP row; every lane of the row gets the result
#define CONFKV_DPP(v, ctrl) \
  __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), ctrl, 0xf, 0xf, true))
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, CONFKV_DPP(v, 0xB1));    // quad_perm [1,0,3,2]
  v = fmaxf(v, CONFKV_DPP(v, 0x4E));    // quad_perm [2,3,0,1]
  v = fmaxf(v, CONFKV_DPP(v, 0x141));   // row_half_mirror
  v = fmaxf(v, CONFKV_DPP(v, 0x140));   // row_mirror
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += CONFKV_DPP(v, 0xB1);
  v += CONFKV_DPP(v, 0x4E);
  v += CONFKV_DPP(v, 0x141);
  v += CONFKV_DPP(v, 0x140);
  return v;
}
#undef CONFKV_DPP

// A 16x16 score tile leaves the matrix core with head 4 * (lane / 16) + i in element i, so at
// G <= 4 only the first 16 lanes hold real rows and every softmax instruction would work on
// three quarters of padding.  Two lane-row swaps regroup the real rows over the whole wavefront:
//   G <= 4: one value per lane; lane row r = lane / 16 holds head r
//   G  > 4: two values per lane; value j of lane row r holds head 2j + (r >> 1) + 4 (r & 1)
//   G  > 8: all 16 rows are real; the matrix-core layout is kept (four values per lane)
// The slot (tile column lane % 16) stays where it is.
template <int G>
struct RowMap {
  static constexpr int NV = G <= 4 ? 1 : G <= 8 ? 2 : 4;
  static __device__ __forceinline__ int head(int j, int r) {
    return G <= 4 ? r : G <= 8 ? 2 * j + (r >> 1) + 4 * (r & 1) : 4 * r + j;
  }
};
// rows (a0, b0, a2, b2) of the two operands
__device__ __forceinline__ float swap16_even(float a, float b) {
  const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a),
                                                   __builtin_bit_cast(unsigned, b), false, false);
  return __builtin_bit_cast(float, r[0]);
}
// rows (a0, a1, b0, b1) of the two operands
__device__ __forceinline__ float swap32_low(float a, float b) {
  const auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a),
                                                   __builtin_bit_cast(unsigned, b), false, false);
  return __builtin_bit_cast(float, r[0]);
}
template <int G>
__device__ __forceinline__ void regroup_rows(const floatx4_t &acc, float (&z)[RowMap<G>::NV]) {
  if constexpr (G <= 4) {
    z[0] = swap32_low(swap16_even(acc[0], acc[1]), swap16_even(acc[2], acc[3]));
  } else if constexpr (G <= 8) {
    z[0] = swap32_low(acc[0], acc[1]);
    z[1] = swap32_low(acc[2], acc[3]);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) z[j] = acc[j];
  }
}
// A quantity that is uniform over each lane row of the regrouped layout, read back in the
// matrix-core layout: the value of head 4 * g4 + i (rows that hold no head get anything).
template <int G>
__device__ __forceinline__ float rows_to_tile(const float (&x)[RowMap<G>::NV], int i, int g4) {
  if constexpr (G > 8) {
    return x[i];
  } else if constexpr (G <= 4) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x[0]), 16 * i));
  } else {
    const int v = __builtin_bit_cast(int, x[i >> 1]);
    const float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(v, 32 * (i & 1)));
    const float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(v, 32 * (i & 1) + 16));
    return (g4 & 1) ? hi : lo;
  }
}

// kChan: the INT8 scales are per (unit, channel).  The K scales are folded into the query (a
// second A operand, split into an fp16 head and tail so the fold costs no accuracy), the V
// scales multiply the output once, after the last INT8 tile; the FP16 slots then come last.
// G is the number of query rows per unit: the group size for single-token calls (row = head),
// or kChunkRows for multi-token calls, where row r is (token r / gq, head r % gq), padding rows
// carry a zero query, and a row sees the call's own tokens causally.
// kSpill: the first launch of the two-launch form (raw scores to device scratch, ends after
// publishing its partial).
template <int G, bool kChan = false, bool kSpill = false, int DR = 128>
__global__ __launch_bounds__(kAttThreads)
__attribute__((amdgpu_waves_per_eu((kChan || G > 8) ? 2 : 3, (kChan || G > 8) ? 2 : 3)))
void attend_mfma_kernel(const int32_t *w_len, const int32_t *w_n8, const int32_t *w_h16, const int32_t *w_h8, int w_unit0, int w_hkv, int w_kvm, CacheView cv, AttendLaunch a_in, int ns, int S) {
  // The unit's counters are requested before anything else, from leading scalar kernel arguments
  // (the four arrays, the layer's first unit, the kv-head count, the grid order): the hardware
  // can hand those over in registers when the wavefront starts, so this request does not wait
  // for the fetch of the argument block as everything else does.
  const int w_words = (((threadIdx.x & 3) == 0 ? w_len : (threadIdx.x & 3) == 1 ? w_n8 : (threadIdx.x & 3) == 2 ? w_h16 : w_h8))
      [w_unit0 + blockIdx.z * w_hkv + (w_kvm ? blockIdx.x : blockIdx.y)];
  const AttendLaunch a = resolve_launch(cv, a_in);
  // D: channels of the tiles and partials on chip.  DR: the head dimension in memory; a 64-channel
  // head runs on the same tiles with channels 64..127 holding a second copy of its rows, which the
  // contractions leave out (two k-steps over the real channels for the scores, four channel
  // groups for the output; the other channels of the partial are never written out).
  constexpr int D = 128;
  constexpr int kSteps = DR / 32;               // k-steps of 32 channels in the score contraction
  static_assert(DR == 64 || DR == 128, "head dimension");
  static_assert(!(kChan && DR != 128), "per-channel scales need 128 channels");
  static_assert(G * D * 4 <= kTileBytes, "a wavefront's output partial must fit its tile buffer");
  constexpr int NP = kAttWaves;                 // one partial per wavefront
  constexpr int kTileFloats =
      (kAttWaves * kTileBytes > NP * G * D * 4 ? kAttWaves * kTileBytes : NP * G * D * 4) / 4;
  extern __shared__ __align__(16) float smem[];
  float *tiles = smem;                          // per-wave tile buffers, later [NP][G][D] partials
  float *stash = kSpill ? a.spill + ((size_t)unit_in_layer(cv, a) * ns + split_index(a)) * G * S
                        : smem + kTileFloats;   // [G][S]
  float *gm = smem + kTileFloats + (kSpill ? 0 : (size_t)G * S);   // [G]
  double *ginv = (double *)(gm + G + (G & 1));  // [2 G]
  float *wm = (float *)(ginv + 2 * G);          // [NP][G]
  float *wl = wm + NP * G;                      // [NP][G]
  float *wo = tiles;
  __shared__ int s_ok;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int tq = G > 8 ? a.tq : 1, gq = G > 8 ? a.gq : G;   // tokens of the call, heads per token
  TS_INIT();
  TS(0);
  // every kernel argument the streaming prologue needs, fetched now (one round trip) rather
  // than piecemeal between the dependent loads below
  asm volatile("" ::"s"(cv.k8), "s"(cv.v8), "s"(cv.ks), "s"(cv.vs), "s"(cv.k16), "s"(cv.v16), "s"(cv.len),
               "s"(cv.n8), "s"(cv.head16), "s"(cv.head8), "s"(cv.cap8), "s"(cv.cap16), "s"(cv.Hkv), "s"(cv.B),
               "s"(a.layer), "s"(a.tq), "s"(a.observe_first), "s"(a.q), "s"(a.knew), "s"(a.vnew));
  // Paged layout: the unit's block table comes into LDS (requested before the counters, so both
  // trips overlap); every INT8 row address below goes through it.
  int32_t *tab = (int32_t *)((char *)smem + a.tab_off);
  if (cv.page_lg) {
    const int32_t *gt = cv.pt + (size_t)(a.layer * cv.B * cv.Hkv + unit_in_layer(cv, a)) * cv.npages;
    for (int i = tid; i < cv.npages; i += kAttThreads) tab[i] = gt[i];
  }
  Slice sl = make_slice(cv, a, ns, S, &w_words);
  if (cv.page_lg) {
    sl.tab = tab;
    __syncthreads();
  }
  TS(2);
  const int page_lg = cv.page_lg, page_mask = (1 << cv.page_lg) - 1;
  // row of INT8 slot i in the INT8 planes
  auto row8 = [&](int i) -> unsigned {
    return page_lg ? (unsigned)((tab[i >> page_lg] << page_lg) | (i & page_mask)) : (unsigned)ring_row_u(sl.h8, i, cv.cap8);
  };
  const int t16 = lane & 15, g4 = lane >> 4;    // MFMA operand coordinates of this lane
  const int c8 = lane & 7, r8 = lane >> 3;      // global-load coordinates: 16-byte piece, row
  const int8_t *K8 = cv.k8 + (size_t)sl.u * cv.cap8 * DR;
  const int8_t *V8 = cv.v8 + (size_t)sl.u * cv.cap8 * DR;
  const __half *KS = cv.ks + (size_t)sl.u * (kChan ? D : cv.cap8);
  const __half *VS = cv.vs + (size_t)sl.u * (kChan ? D : cv.cap8);

  const int ntiles = (sl.cnt8 + kTile - 1) / kTile;            // 0 when the split has no INT8 slot
  // One INT8 tile in flight: four 128-bit K pieces, four V pieces and the raw scale bits.
  // Loads are branch-free (rows past the slice re-read its last row; their scores are masked
  // and their probabilities are zero), so the whole tile is in flight before any wait.
  struct TileRegs {
    int4 k0, k1, k2, k3, v0, v1, v2, v3;
    unsigned short ks0, ks1, vs0, vs1;
  };
  auto load_tile = [&](int tile) -> TileRegs {
    TileRegs t;
    const int base = sl.lo8 + tile * kTile;
    const int last = sl.hi8 - 1;
    // 32-bit byte offsets from the unit's (wavefront-uniform) plane bases
    const unsigned col = (unsigned)(c8 & (DR / 16 - 1)) * 16u;
    const unsigned o0 = row8(min(base + r8, last)) * DR + col;
    const unsigned o1 = row8(min(base + 8 + r8, last)) * DR + col;
    const unsigned o2 = row8(min(base + 16 + r8, last)) * DR + col;
    const unsigned o3 = row8(min(base + 24 + r8, last)) * DR + col;
    t.k0 = ld_stream16(K8 + o0);
    t.v0 = ld_stream16(V8 + o0);
    t.k1 = ld_stream16(K8 + o1);
    t.v1 = ld_stream16(V8 + o1);
    t.k2 = ld_stream16(K8 + o2);
    t.v2 = ld_stream16(V8 + o2);
    t.k3 = ld_stream16(K8 + o3);
    t.v3 = ld_stream16(V8 + o3);
    if constexpr (!kChan) {
      const unsigned j0 = row8(min(base + t16, last));
      const unsigned j1 = row8(min(base + 16 + t16, last));
      t.ks0 = ld_stream((const unsigned short *)KS + j0);
      t.vs0 = ld_stream((const unsigned short *)VS + j0);
      t.ks1 = ld_stream((const unsigned short *)KS + j1);
      t.vs1 = ld_stream((const unsigned short *)VS + j1);
    } else {
      t.ks0 = t.ks1 = t.vs0 = t.vs1 = 0;
    }
    return t;
  };
  TileRegs tr = {};
  // the first INT8 tile is requested before anything else: its latency covers the append and
  // the query loads
  if (w < ntiles) tr = load_tile(w);
  TS(3);
  append_new_token<DR, false>(cv, a, sl, ns);
  const float NEG = -INFINITY;
  const float sm = a.sm_scale;
  TS(1);

  // ---------------- INT8 slots on the matrix cores ----------------
  uint8_t *Kt = (uint8_t *)tiles + (size_t)w * kTileBytes;   // [32][kKRow]
  uint8_t *Vt = Kt + kTile * kKRow;                           // [128][kVRow], slots permuted
  _Float16 *Pb = (_Float16 *)(Vt + kVBytes);                  // [16][kPRow], rows >= G stay 0
  for (int i = lane; i < 16 * kPRow / 2; i += kWave) ((unsigned *)Pb)[i] = 0u;

  // A operand of the score contraction: Q padded to 16 rows; k-step s covers channels
  // g4*32 + 8s + [0,8), matching the K bytes this lane reads from the tile below.
  half8_t qa[4];
  {
    // row t16 = (token, head) of the call's [B][tq][Hq][D] queries
    const int q_tok = t16 / gq, q_head = t16 - q_tok * gq;
    const __half *qrow = a.q + ((((size_t)sl.b * a.q_tokens + q_tok) * cv.Hkv + sl.g) * gq + q_head) * DR;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      int4 raw = make_int4(0, 0, 0, 0);
      // (a 64-channel head: two k-steps, step s of lane group g4 covers channels 16 g4 + 8 s + [0, 8))
      if (t16 < G && q_tok < tq && s < kSteps) raw = *(const int4 *)(qrow + g4 * (8 * kSteps) + 8 * s);
      qa[s] = __builtin_bit_cast(half8_t, raw);
    }
  }
  // Per-channel scales: A operand of the INT8 scores = q * s_k * 2^8 as head + tail in fp16
  // (the power of two keeps the tail of every term that matters a normal number; it is taken
  // back in the score factor), and this lane's eight V scales (channels 16 nt + t16).
  constexpr float kFoldUp = 256.0f;
  half8_t qh[kChan ? 4 : 1], ql[kChan ? 4 : 1];
  float vch[kChan ? 8 : 1];
  if constexpr (kChan) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const half8_t ksv = __builtin_bit_cast(half8_t, *(const int4 *)(KS + g4 * 32 + 8 * s));
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float prod = (float)qa[s][e] * (float)ksv[e] * kFoldUp;
        const _Float16 hi = (_Float16)prod;
        qh[s][e] = hi;
        ql[s][e] = (_Float16)(prod - (float)hi);
      }
    }
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) vch[nt] = __half2float(VS[16 * nt + t16]);
  }
  floatx4_t O[8];
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) O[nt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  // running softmax state in the regrouped layout: reference, normaliser (per-lane partial
  // sum) and the sum of the fp16 probabilities that met biased INT8 values
  constexpr int NV = RowMap<G>::NV;
  float mrun[NV], lrun[NV], pbias[NV];
  int hd[NV];                                    // head of value j of this lane
#pragma unroll
  for (int j = 0; j < NV; ++j) { mrun[j] = NEG; lrun[j] = 0.f; pbias[j] = 0.f; hd[j] = RowMap<G>::head(j, g4); }
  // causal order inside the call: the row of token t sees slots below n - tq + t + 1 (every
  // slot of the unit when the call has one token)
  int seen[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) seen[j] = sl.n - tq + hd[j] / gq + 1;

  // ---------------- the slice as a list of work items ----------------
  // Items 0 .. ntiles-1 are the 32-slot INT8 tiles, the rest the 16-slot FP16 tiles (the same
  // 8 KB of rows each).  Wavefront w takes items w, w + 8, ..; the rows of its next item are
  // requested as soon as the current ones have left the registers for LDS, so one item per
  // wavefront is always in flight.
  const int base16 = sl.lo16;
  const int ntiles16 = (sl.hi16 - sl.lo16 + 15) / 16;
  const int nitems = ntiles + ntiles16;
  const __half *K16 = cv.k16 + (size_t)sl.u * cv.cap16 * DR;
  const __half *V16 = cv.v16 + (size_t)sl.u * cv.cap16 * DR;
  const int c16 = lane & 15, r4 = lane >> 4;     // FP16 load coordinates: 16-byte piece, row
  auto load_tile16 = [&](int f) -> TileRegs {
    TileRegs t;
    const int base = base16 + 16 * f, last = sl.hi16 - 1;
    const int h16 = sl.h16, cap16 = cv.cap16, n8 = sl.n8;
    const unsigned col = (unsigned)(c16 & (DR / 8 - 1)) * 8u;
    const unsigned o0 = (unsigned)ring_row(h16, min(base + r4, last) - n8, cap16) * DR + col;
    const unsigned o1 = (unsigned)ring_row(h16, min(base + 4 + r4, last) - n8, cap16) * DR + col;
    const unsigned o2 = (unsigned)ring_row(h16, min(base + 8 + r4, last) - n8, cap16) * DR + col;
    const unsigned o3 = (unsigned)ring_row(h16, min(base + 12 + r4, last) - n8, cap16) * DR + col;
    // the call's own tokens (slots n - tq .. n - 1, at the end of the unit's last split) are
    // taken from the call's arguments, not read back from the ring: no wait on the append's stores
    // (an observation call appends nothing: every row comes from the ring)
    const int first_new = a.observe_first >= 0 ? 0x3fffffff : sl.n - tq;
    const size_t tok = (size_t)cv.Hkv * DR;                     // [B][tq][Hkv][D]: stride of a token
    const __half *kn = a.knew + ((size_t)sl.b * tq * cv.Hkv + sl.g) * DR + col;
    const __half *vn = a.vnew + ((size_t)sl.b * tq * cv.Hkv + sl.g) * DR + col;
    const int s0 = min(base + r4, last) - first_new, s1 = min(base + 4 + r4, last) - first_new;
    const int s2 = min(base + 8 + r4, last) - first_new, s3 = min(base + 12 + r4, last) - first_new;
    t.k0 = ld_stream16(s0 >= 0 ? kn + s0 * tok : K16 + o0);
    t.v0 = ld_stream16(s0 >= 0 ? vn + s0 * tok : V16 + o0);
    t.k1 = ld_stream16(s1 >= 0 ? kn + s1 * tok : K16 + o1);
    t.v1 = ld_stream16(s1 >= 0 ? vn + s1 * tok : V16 + o1);
    t.k2 = ld_stream16(s2 >= 0 ? kn + s2 * tok : K16 + o2);
    t.v2 = ld_stream16(s2 >= 0 ? vn + s2 * tok : V16 + o2);
    t.k3 = ld_stream16(s3 >= 0 ? kn + s3 * tok : K16 + o3);
    t.v3 = ld_stream16(s3 >= 0 ? vn + s3 * tok : V16 + o3);
    t.ks0 = t.ks1 = t.vs0 = t.vs1 = 0;
    return t;
  };
  auto load_item = [&](int it) -> TileRegs { return it < ntiles ? load_tile(it) : load_tile16(it - ntiles); };
  if (w >= ntiles && w < nitems) tr = load_tile16(w - ntiles);
  // with per-channel scales the accumulator leaves code units once, after the wavefront's last
  // INT8 item (its FP16 items, if any, come after that)
  bool in_code_units = kChan;
  auto leave_code_units = [&]() {
    // the INT8 part is complete: take the code bias out and go from code units to values
    float pb[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) { pb[j] = row16_sum(pbias[j]) * kCodeBias; pbias[j] = 0.f; }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float bias = rows_to_tile<G>(pb, i, g4);
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) O[nt][i] = (O[nt][i] - bias) * vch[nt];
    }
    in_code_units = false;
  };
  int tix = 0;
  for (int item = w; item < nitems; item += kAttWaves) {
    if (item >= ntiles) {
      // ---- an FP16 tile ----
      if constexpr (kChan) {
        if (in_code_units) leave_code_units();
      }
      const int base = base16 + 16 * (item - ntiles);
      // K rows as they are (row stride kKRow16 bytes), V transposed to [channel][slot]
      *(int4 *)(Kt + (r4)*kKRow16 + c16 * 16) = tr.k0;
      *(int4 *)(Kt + (4 + r4) * kKRow16 + c16 * 16) = tr.k1;
      *(int4 *)(Kt + (8 + r4) * kKRow16 + c16 * 16) = tr.k2;
      *(int4 *)(Kt + (12 + r4) * kKRow16 + c16 * 16) = tr.k3;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const unsigned x0 = dword_of(tr.v0, q4), x1 = dword_of(tr.v1, q4);
        const unsigned x2 = dword_of(tr.v2, q4), x3 = dword_of(tr.v3, q4);
        // half r of each pair is slot 4r + r4; it lands at column 4*r4 + r
        unsigned *dst = (unsigned *)(Vt + (8 * c16 + 2 * q4) * kVRow + kVSkew(c16 >> 1) + 8 * r4);
        dst[0] = __builtin_amdgcn_perm(x1, x0, 0x05040100u);
        dst[1] = __builtin_amdgcn_perm(x3, x2, 0x05040100u);
        dst[kVRow / 4] = __builtin_amdgcn_perm(x1, x0, 0x07060302u);
        dst[kVRow / 4 + 1] = __builtin_amdgcn_perm(x3, x2, 0x07060302u);
      }
      wave_lds_sync();
      if (item + kAttWaves < nitems) tr = load_item(item + kAttWaves);
      const uint8_t *krow = Kt + t16 * kKRow16 + g4 * (16 * kSteps);
      floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < kSteps; ++s)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[s], *(const half8_t *)(krow + 16 * s), acc, 0, 0, 0);
      const bool valid = base + t16 < sl.hi16;
      float z[NV], corr[NV];
      regroup_rows<G>(acc, z);
      bool changed = false;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const bool real = valid && hd[j] < G && base + t16 < seen[j];
        const float sv = real ? z[j] * sm : NEG;
        if (valid && hd[j] < G) stash[hd[j] * S + sl.cnt8 + (base + t16 - sl.lo16)] = sv;
        const float mn = fmaxf(mrun[j], row16_max(sv));
        corr[j] = (mn == NEG) ? 1.f : __expf(mrun[j] - mn);
        changed |= (mn != mrun[j]);
        mrun[j] = mn;
        const float p = real ? __expf(sv - mn) : 0.f;
        if (hd[j] < G) Pb[hd[j] * kPRow + 4 * (t16 & 3) + (t16 >> 2)] = (_Float16)p;
        lrun[j] = fmaf(lrun[j], corr[j], p);
        pbias[j] *= corr[j];
      }
      if (__builtin_amdgcn_ballot_w64(changed)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float c = rows_to_tile<G>(corr, i, g4);
#pragma unroll
          for (int nt = 0; nt < 8; ++nt) O[nt][i] *= c;
        }
      }
      wave_lds_sync();
      const half4_t pa = *(const half4_t *)(Pb + t16 * kPRow + 4 * g4);
      // (a 64-channel head has four real channel groups: the copies in groups 4..7 are not multiplied)
#pragma unroll
      for (int nt = 0; nt < DR / 16; ++nt) {
        const unsigned *vb = (const unsigned *)(Vt + (16 * nt + t16) * kVRow + kVSkew(nt) + 8 * g4);
        const uint2 v2 = make_uint2(vb[0], vb[1]);
        O[nt] = __builtin_amdgcn_mfma_f32_16x16x16f16(pa, __builtin_bit_cast(half4_t, v2), O[nt], 0, 0, 0);
      }
      wave_lds_sync();
      continue;
    }
    const int base = sl.lo8 + item * kTile;
    if (tix < 6) TS(4 + 2 * tix);
    // ---- registers -> LDS: K rows as they are, V transposed to [channel][slot] ----
    *(int4 *)(Kt + (r8)*kKRow + c8 * 16) = tr.k0;
    *(int4 *)(Kt + (8 + r8) * kKRow + c8 * 16) = tr.k1;
    *(int4 *)(Kt + (16 + r8) * kKRow + c8 * 16) = tr.k2;
    *(int4 *)(Kt + (24 + r8) * kKRow + c8 * 16) = tr.k3;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const unsigned x0 = dword_of(tr.v0, q4), x1 = dword_of(tr.v1, q4);
      const unsigned x2 = dword_of(tr.v2, q4), x3 = dword_of(tr.v3, q4);
      const unsigned t0 = __builtin_amdgcn_perm(x1, x0, 0x05010400u), t1 = __builtin_amdgcn_perm(x1, x0, 0x07030602u);
      const unsigned t2 = __builtin_amdgcn_perm(x3, x2, 0x05010400u), t3 = __builtin_amdgcn_perm(x3, x2, 0x07030602u);
      const unsigned o0 = __builtin_amdgcn_perm(t2, t0, 0x05040100u), o1 = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
      const unsigned o2 = __builtin_amdgcn_perm(t3, t1, 0x05040100u), o3 = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
      // byte r of o_e is slot 8r + r8 at channel 16*c8 + 4*q4 + e; it lands at column 4*r8 + r
      uint8_t *dst = Vt + (16 * c8 + 4 * q4) * kVRow + kVSkew(c8) + 4 * r8;
      *(unsigned *)(dst) = o0;
      *(unsigned *)(dst + kVRow) = o1;
      *(unsigned *)(dst + 2 * kVRow) = o2;
      *(unsigned *)(dst + 3 * kVRow) = o3;
    }
    const float kscale[2] = {kChan ? sm * (1.0f / kFoldUp) : __half2float(__ushort_as_half(tr.ks0)) * sm,
                             kChan ? sm * (1.0f / kFoldUp) : __half2float(__ushort_as_half(tr.ks1)) * sm};
    const float vscale[2] = {kChan ? 1.0f : __half2float(__ushort_as_half(tr.vs0)),
                             kChan ? 1.0f : __half2float(__ushort_as_half(tr.vs1))};
    wave_lds_sync();
    if (tix < 6) TS(5 + 2 * tix);
    ++tix;
    // the registers are free again: fetch this wavefront's next tile while computing
    if (item + kAttWaves < nitems) tr = load_item(item + kAttWaves);

    // ---- scores: S[head][slot] for the two 16-slot halves of the tile ----
    float sc[2][NV];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      const uint8_t *krow = Kt + (16 * sb + t16) * kKRow + g4 * (8 * kSteps);
      const int4 b0 = *(const int4 *)(krow);
      int4 b1 = b0;
      if constexpr (kSteps == 4) b1 = *(const int4 *)(krow + 16);
      floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
      if constexpr (kSteps == 2) {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[0], cvt_i8x8_f16x8(b0.x, b0.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[1], cvt_i8x8_f16x8(b0.z, b0.w), acc, 0, 0, 0);
      } else if constexpr (kChan) {
        const half8_t kb[4] = {cvt_i8x8_f16x8(b0.x, b0.y), cvt_i8x8_f16x8(b0.z, b0.w),
                               cvt_i8x8_f16x8(b1.x, b1.y), cvt_i8x8_f16x8(b1.z, b1.w)};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ql[s], kb[s], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qh[s], kb[s], acc, 0, 0, 0);
        }
      } else {
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[0], cvt_i8x8_f16x8(b0.x, b0.y), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[1], cvt_i8x8_f16x8(b0.z, b0.w), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[2], cvt_i8x8_f16x8(b1.x, b1.y), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[3], cvt_i8x8_f16x8(b1.z, b1.w), acc, 0, 0, 0);
      }
      const bool valid = base + 16 * sb + t16 < sl.hi8;
      float z[NV];
      regroup_rows<G>(acc, z);
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const bool real = valid && hd[j] < G;
        // an INT8 slot is ahead of a query only in an observation call (appended tokens are FP16)
        const bool ahead = G > 8 && base + 16 * sb + t16 >= seen[j];
        const float sv = ahead ? NEG : z[j] * kscale[sb];
        sc[sb][j] = real ? sv : NEG;
        if (real) stash[hd[j] * S + (base + 16 * sb + t16 - sl.lo8)] = sv;
      }
    }
    if (tix <= 2) TS(24 + (tix - 1) * 3);
    // ---- online softmax per head ----
    // The running reference m only has to stay within a few units of the true maximum (the
    // merge is exact for any reference), so the row reduction and the rescale of O run only
    // when some score of the tile exceeds the reference by more than kSlack; e^kSlack times
    // the largest fp16 value scale still fits fp16.
    constexpr float kSlack = 4.0f;
    float lm[NV];
    bool grow = false;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      lm[j] = fmaxf(sc[0][j], sc[1][j]);
      grow |= lm[j] > mrun[j] + kSlack;             // also true on the first tile (m = -inf)
    }
    if (__builtin_amdgcn_ballot_w64(grow)) {
      float corr[NV];
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const float mn = fmaxf(mrun[j], row16_max(lm[j]));
        corr[j] = (mn == NEG) ? 1.f : __expf(mrun[j] - mn);
        mrun[j] = mn;
        lrun[j] *= corr[j];
        pbias[j] *= corr[j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float c = rows_to_tile<G>(corr, i, g4);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) O[nt][i] *= c;
      }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const float p = (sc[sb][j] == NEG) ? 0.f : __expf(sc[sb][j] - mrun[j]);
        lrun[j] += p;
        const _Float16 ph = (_Float16)(p * vscale[sb]);
        pbias[j] += (float)ph;                             // exactly what the matrix core will see
        const int tau = 16 * sb + t16;                     // slot within the tile
        if (hd[j] < G) Pb[hd[j] * kPRow + 4 * (tau & 7) + (tau >> 3)] = ph;
      }
    }
    wave_lds_sync();
    if (tix <= 2) TS(25 + (tix - 1) * 3);
    // ---- output: O[head][channel] += P[head][slot] V[slot][channel] ----
    const half8_t pa = *(const half8_t *)(Pb + t16 * kPRow + 8 * g4);
#pragma unroll
    for (int nt = 0; nt < DR / 16; ++nt) {
      const unsigned *vb = (const unsigned *)(Vt + (16 * nt + t16) * kVRow + kVSkew(nt) + 8 * g4);   // 4-byte aligned
      O[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, cvt_i8x8_f16x8_biased(vb[0], vb[1]), O[nt], 0, 0, 0);
    }
    wave_lds_sync();
  }
  if constexpr (kChan) {
    if (in_code_units) leave_code_units();
  }
  TS(16);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    lrun[j] = row16_sum(lrun[j]);
    pbias[j] = row16_sum(pbias[j]) * kCodeBias;     // what the biased INT8 values added per channel
  }

  // the wavefront's matrix-core partial goes into its own (now idle) tile buffer
  float *wo_w = tiles + w * (kTileBytes / 4);
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (t16 == 0 && hd[j] < G) { wm[w * G + hd[j]] = mrun[j]; wl[w * G + hd[j]] = lrun[j]; }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int h = 4 * g4 + i;
    const float bias = rows_to_tile<G>(pbias, i, g4);
    if (h < G) {
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) wo_w[h * D + 16 * nt + t16] = O[nt][i] - bias;
    }
  }

  TS(17);
  __syncthreads();
  TS(18);
  attend_epilogue<D, G, NP, kTileBytes / 4, kSpill ? 1 : 0, DR>(cv, a, sl, ns, S, stash, wm, wl, wo, gm, ginv, &s_ok);
  TS_DUMP();
}

#include "attend_wide.h"

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------

typedef void (*AttendFn)(const int32_t *, const int32_t *, const int32_t *, const int32_t *, int, int, int, CacheView,
                         AttendLaunch, int, int);

static std::atomic<bool> g_use_mfma{true};

static AttendFn attend_fn_valu(int D, int G) {
#define CONFKV_CASE(d, g) \
  if (D == d && G == g) return attend_kernel<d, g>;
  CONFKV_CASE(64, 1) CONFKV_CASE(64, 2) CONFKV_CASE(64, 3) CONFKV_CASE(64, 4) CONFKV_CASE(64, 5)
  CONFKV_CASE(64, 6) CONFKV_CASE(64, 7) CONFKV_CASE(64, 8)
  CONFKV_CASE(128, 1) CONFKV_CASE(128, 2) CONFKV_CASE(128, 3) CONFKV_CASE(128, 4) CONFKV_CASE(128, 5)
  CONFKV_CASE(128, 6) CONFKV_CASE(128, 7) CONFKV_CASE(128, 8)
#undef CONFKV_CASE
  return nullptr;
}

static AttendFn attend_fn_spill(int D, int G, bool finish) {
#define CONFKV_CASE(d, g) \
  if (D == d && G == g) return finish ? (AttendFn)attend_finish_kernel<d, g> : (AttendFn)attend_kernel<d, g, true>;
  CONFKV_CASE(64, 1) CONFKV_CASE(64, 2) CONFKV_CASE(64, 3) CONFKV_CASE(64, 4) CONFKV_CASE(64, 5)
  CONFKV_CASE(64, 6) CONFKV_CASE(64, 7) CONFKV_CASE(64, 8)
  CONFKV_CASE(128, 1) CONFKV_CASE(128, 2) CONFKV_CASE(128, 3) CONFKV_CASE(128, 4) CONFKV_CASE(128, 5)
  CONFKV_CASE(128, 6) CONFKV_CASE(128, 7) CONFKV_CASE(128, 8)
#undef CONFKV_CASE
  // multi-token calls: only the second launch exists for 16 rows (the first is the matrix-core body)
  if (D == 128 && G == kChunkRows && finish) return (AttendFn)attend_finish_kernel<128, kChunkRows>;
  return nullptr;
}

// Second launch behind the matrix-core body at D = 64: the partials are 128 channels wide.
static AttendFn attend_fn_finish_padded(int G) {
#define CONFKV_CASE(g) \
  case g: return (AttendFn)attend_finish_kernel<128, g, 64>;
  switch (G) {
    CONFKV_CASE(2) CONFKV_CASE(3) CONFKV_CASE(4) CONFKV_CASE(5) CONFKV_CASE(6) CONFKV_CASE(7) CONFKV_CASE(8)
    default: return nullptr;
  }
#undef CONFKV_CASE
}

static AttendFn attend_fn_mfma(int D, int G, bool chan) {
  if (D == 64 && !chan) {
#define CONFKV_CASE(g) \
  case g: return (AttendFn)attend_mfma_kernel<g, false, false, 64>;
    switch (G) {
      CONFKV_CASE(2) CONFKV_CASE(3) CONFKV_CASE(4) CONFKV_CASE(5) CONFKV_CASE(6) CONFKV_CASE(7) CONFKV_CASE(8)
      default: return nullptr;
    }
#undef CONFKV_CASE
  }
  if (D != 128) return nullptr;
#define CONFKV_CASE(g) \
  case g: return chan ? (AttendFn)attend_mfma_kernel<g, true> : (AttendFn)attend_mfma_kernel<g, false>;
  switch (G) {
    CONFKV_CASE(2) CONFKV_CASE(3) CONFKV_CASE(4) CONFKV_CASE(5) CONFKV_CASE(6) CONFKV_CASE(7) CONFKV_CASE(8)
    CONFKV_CASE(kChunkRows)
    default: return nullptr;
  }
#undef CONFKV_CASE
}

static AttendFn attend_fn_mfma_spill(int D, int G, bool chan) {
  if (D == 64 && !chan) {
#define CONFKV_CASE(g) \
  case g: return (AttendFn)attend_mfma_kernel<g, false, true, 64>;
    switch (G) {
      CONFKV_CASE(2) CONFKV_CASE(3) CONFKV_CASE(4) CONFKV_CASE(5) CONFKV_CASE(6) CONFKV_CASE(7) CONFKV_CASE(8)
      default: return nullptr;
    }
#undef CONFKV_CASE
  }
  if (D != 128) return nullptr;
#define CONFKV_CASE(g) \
  case g: return chan ? (AttendFn)attend_mfma_kernel<g, true, true> : (AttendFn)attend_mfma_kernel<g, false, true>;
  switch (G) {
    CONFKV_CASE(2) CONFKV_CASE(3) CONFKV_CASE(4) CONFKV_CASE(5) CONFKV_CASE(6) CONFKV_CASE(7) CONFKV_CASE(8)
    CONFKV_CASE(kChunkRows)
    default: return nullptr;
  }
#undef CONFKV_CASE
}

// The matrix-core kernel serves every grouped-query shape, FP16-only caches included (at G >= 4
// the vector-ALU body runs out of registers); at D = 64 it pads the head to its 128-channel tiles.
static bool wants_mfma(int D, int G, bool /*has_int8*/) {
  return g_use_mfma && attend_fn_mfma(D, G, false) != nullptr;
}

// Groups of 9 to 16 query heads run as a one-token call of the 16-row matrix-core kernel (D = 128).
bool attend_supported(int D, int G) {
  return attend_fn_valu(D, G) != nullptr || (D == 128 && G > 8 && G <= kChunkRows);
}

static size_t attend_lds_bytes(int D, int G, int S, bool mfma) {
  if (mfma) {
    const int NP = kAttWaves;
    size_t floats = (size_t)G * S + G + 2 + 2 * NP * G;
    size_t tiles = std::max<size_t>((size_t)kAttWaves * kTileBytes, (size_t)NP * G * 128 * sizeof(float));
    return (floats * sizeof(float) + (size_t)2 * G * sizeof(double) + tiles + 32 + 15) / 16 * 16;
  }
  size_t floats = (size_t)G * S + (size_t)kAttWaves * G * D + 2 * kAttWaves * G + G + 2;
  return floats * sizeof(float) + (size_t)2 * G * sizeof(double) + 16;
}

struct DeviceLimits {
  int cus = 0;
  size_t max_lds = 0;
  bool ok = false;
};

// The two caches below are shared by every handle of the process; handles may live on
// different host threads, so both are guarded.
static std::mutex g_plan_mutex;

static const DeviceLimits &device_limits() {
  static DeviceLimits lim;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  if (!lim.ok) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
      lim.cus = prop.multiProcessorCount;
      lim.max_lds = prop.sharedMemPerBlockOptin ? prop.sharedMemPerBlockOptin
                                                : prop.sharedMemPerBlock;
      if (lim.max_lds > 160 * 1024) lim.max_lds = 160 * 1024;
      lim.ok = lim.cus > 0;
      if (const char *e = getenv("CONF_KV_NO_MFMA")) g_use_mfma = atoi(e) == 0;
    }
  }
  return lim;
}

// Resident workgroups per CU of a kernel with `lds` bytes of dynamic LDS.
static int attend_occupancy(AttendFn fn, size_t lds) {
  static std::map<std::tuple<const void *, size_t>, int> cache;
  std::lock_guard<std::mutex> lock(g_plan_mutex);
  auto key = std::make_tuple((const void *)fn, lds);
  auto it = cache.find(key);
  if (it != cache.end()) return it->second;
  int nb = 0;
  // The dynamic-LDS ceiling of a kernel is raised once, to the most any plan can ask for: a
  // ceiling set per plan would be lowered again by a later, smaller plan of the same kernel.
  static std::set<const void *> raised;
  if (lds > 64 * 1024 && raised.insert((const void *)fn).second) {
    hipFuncAttributes fa;
    size_t fixed = 0;                            // LDS the kernel declares itself counts against the same limit
    if (hipFuncGetAttributes(&fa, (const void *)fn) == hipSuccess) fixed = fa.sharedSizeBytes;
    (void)hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(160 * 1024 - std::min<size_t>(fixed, 64 * 1024)));
  }
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void *)fn, kAttThreads, lds) !=
      hipSuccess)
    nb = 0;
  cache[key] = nb;
  return nb;
}

bool attend_plan(int D, int G, bool chan, bool chunk, int units_per_layer, int n_ub, int n16_ub, int forced_splits,
                 bool force_two_launch, size_t extra_lds, AttendPlan *plan) {
  const DeviceLimits &lim = device_limits();
  if (!lim.ok) return false;
  if (chunk ? attend_fn_mfma(D, G, chan) == nullptr : attend_fn_valu(D, G) == nullptr) return false;
  const bool mfma = chunk || wants_mfma(D, G, n16_ub < n_ub);
  AttendFn fn = mfma ? attend_fn_mfma(D, G, chan) : attend_fn_valu(D, G);
  const long long nv = (long long)n_ub + n16_ub;
  // One workgroup per CU measured best: the exchange between the splits of a unit (statistics
  // and partial gather) gets slower with more participants, and a grid that is not a
  // whole number of waves over the CUs leaves a straggler round.  Two per CU only when a
  // single split per unit would leave half of the chip idle.
  int want = lim.cus / units_per_layer;
  if (want < 1) want = 1;
  if (want == 1 && 2 * units_per_layer <= 2 * lim.cus && units_per_layer > lim.cus / 2) want = 2;
  // Measured on 8- and 12-unit layers of 500 to 32768 slots: a unit below about 192 KB is
  // fastest on one workgroup (no exchange at all); above, splits down to about 32 KB each
  // (one 32-slot tile per wavefront) still pay.
  const long long unit_bytes = (long long)(n_ub - n16_ub) * (2 * D + 4) + (long long)n16_ub * 4 * D;
  want = unit_bytes <= 192 * 1024 ? 1 : (int)std::min<long long>(want, unit_bytes / (32 * 1024));
  if (forced_splits > 0) want = std::min<long long>(forced_splits, std::max<long long>(1, nv / 128));
  want = std::max(1, std::min(want, kAttendMaxSplits));
  // preference order: want, want-1, .., 1 (fewer, always co-resident), then want+1, .. (more
  // splits shrink the LDS stash when a long unit does not fit otherwise)
  plan->two_launch = false;
  plan->wide_rb = 0;
  for (int k = 0; k < kAttendMaxSplits && !force_two_launch; ++k) {
    const int ns = k < want ? want - k : k + 1;
    // LDS is sized in steps of 256 slots so the occupancy query is cached across calls
    const int need = (n_ub + ns - 1) / ns + (n16_ub + ns - 1) / ns + 34;
    int S = (need + 255) / 256 * 256;
    size_t lds = attend_lds_bytes(D, G, S, mfma) + extra_lds;
    if (lds > lim.max_lds) {                    // a tight fit: give the rounding up
      S = (need + 31) / 32 * 32;
      lds = attend_lds_bytes(D, G, S, mfma) + extra_lds;
    }
    if (lds > lim.max_lds) continue;
    if (ns > 1) {
      int occ = attend_occupancy(fn, lds);
      if ((long long)occ * lim.cus < (long long)ns * units_per_layer) continue;
    } else if (lds > 64 * 1024) {
      (void)attend_occupancy(fn, lds);          // raises the dynamic-LDS limit
    }
    plan->splits = ns;
    plan->stash_tokens = S;
    plan->lds_bytes = lds;
    plan->mfma = mfma;
    return true;
  }
  // No single-kernel plan: the splits of a unit cannot all be resident (many long units), or
  // the slice's scores do not fit LDS.  Two launches then: the first streams and publishes
  // partials, keeping the raw scores in device scratch; the second merges and updates the EMA.
  // Nothing waits inside a kernel, so any split count works.
  {
    // same split count as the single-kernel plan would like (measured on 64 units of 4096
    // slots: 4 splits 40 us, 16 splits 80 us -- the second launch grows with the split count)
    const int ns = want;
    int S = (n_ub + ns - 1) / ns + (n16_ub + ns - 1) / ns + 34;
    S = (S + 255) / 256 * 256;
    const size_t lds = attend_lds_bytes(D, G, 0, mfma) + extra_lds;
    if (lds > lim.max_lds) return false;
    if (lds > 64 * 1024) (void)attend_occupancy(attend_fn_mfma_spill(D, G, chan), lds);   // raises the dynamic-LDS limit
    plan->splits = ns;
    plan->stash_tokens = S;
    plan->lds_bytes = lds;
    plan->mfma = mfma;
    plan->two_launch = true;
    return true;
  }
}

// Calls with more than 16 query rows per unit: row blocks (a power of two) and split count.  The
// splits of a unit exchange partials inside the launch, so with more than one split the whole grid
// must be resident (one workgroup per CU: the tile buffers take most of the LDS).
bool attend_wide_plan(int rows, int units_per_layer, int n_ub, int forced_splits, AttendPlan *plan) {
  const DeviceLimits &lim = device_limits();
  if (!lim.ok || rows <= kChunkRows || rows > kWideMaxRows) return false;
  int rb = 2;
  while (rb * 16 < rows) rb *= 2;
  int ns = 1;
  while (ns * 2 <= kWideMaxSplits && ns * 2 * units_per_layer <= lim.cus && n_ub / (ns * 2) >= 256) ns *= 2;
  if (forced_splits > 0) {
    ns = 1;
    while (ns * 2 <= std::min(forced_splits, kWideMaxSplits) && ns * 2 * units_per_layer <= lim.cus && n_ub / (ns * 2) >= 64) ns *= 2;
  }
  AttendFn fn = rb == 2 ? (AttendFn)attend_wide_kernel<2> : rb == 4 ? (AttendFn)attend_wide_kernel<4> : (AttendFn)attend_wide_kernel<8>;
  const size_t lds = attend_wide_lds_bytes(rb * 16, ns);
  if (lds > lim.max_lds || attend_occupancy(fn, lds) < 1) return false;
  plan->splits = ns;
  plan->stash_tokens = 0;
  plan->lds_bytes = lds;
  plan->mfma = true;
  plan->two_launch = false;
  plan->wide_rb = rb;
  return true;
}

size_t attend_spill_floats(int units_per_layer, int G, int cap) {
  // splits * S <= n + n16 + splits * (2 + 34 + 255) with n, n16 <= cap
  return (size_t)units_per_layer * G * (2 * (size_t)cap + (size_t)kAttendMaxSplits * 291);
}

hipError_t launch_attend(const CacheView &cv, const AttendLaunch &a_in, const AttendPlan &plan,
                         hipStream_t stream) {
  AttendLaunch a = a_in;
  if (plan.two_launch || !plan.mfma) a.dbg = nullptr;      // only the single matrix-core kernel is traced
  const dim3 grid = a.kv_major ? dim3(cv.Hkv, plan.splits, cv.B) : dim3(plan.splits, cv.Hkv, cv.B);
  if (plan.two_launch) {
    const bool rows16 = a.tq > 1 || a.observe_first >= 0 || cv.G > 8;
    const int rows2 = rows16 ? kChunkRows : cv.G;                   // query rows per unit
    if (rows16 && !plan.mfma) return hipErrorInvalidValue;
    AttendFn first = plan.mfma ? attend_fn_mfma_spill(cv.D, rows2, cv.chan != 0) : attend_fn_spill(cv.D, cv.G, false);
    AttendFn second = plan.mfma && cv.D == 64 ? attend_fn_finish_padded(rows2) : attend_fn_spill(cv.D, rows2, true);
    if (!first || !second || !a.spill) return hipErrorInvalidValue;
    hipLaunchKernelGGL(first, grid, dim3(kAttThreads), plan.lds_bytes, stream, cv.len, cv.n8, cv.head16, cv.head8, a.layer * cv.B * cv.Hkv, cv.Hkv, a.kv_major, cv, a, plan.splits,
                       plan.stash_tokens);
    const size_t lds2 = ((size_t)plan.splits * rows2 * 2 + rows2 + 2) * sizeof(float) + 2 * rows2 * sizeof(double);
    hipLaunchKernelGGL(second, grid, dim3(kAttThreads), lds2, stream, cv.len, cv.n8, cv.head16, cv.head8, a.layer * cv.B * cv.Hkv, cv.Hkv, a.kv_major, cv, a, plan.splits,
                       plan.stash_tokens);
    return hipGetLastError();
  }
  if (plan.wide_rb) {
    AttendFn wide = plan.wide_rb == 2 ? (AttendFn)attend_wide_kernel<2>
                    : plan.wide_rb == 4 ? (AttendFn)attend_wide_kernel<4> : (AttendFn)attend_wide_kernel<8>;
    a.dbg = nullptr;
    a.max_splits = kWideMaxSplits;
    hipLaunchKernelGGL(wide, grid, dim3(kAttThreads), plan.lds_bytes, stream, cv.len, cv.n8, cv.head16, cv.head8, a.layer * cv.B * cv.Hkv, cv.Hkv, a.kv_major, cv, a, plan.splits, 0);
    return hipGetLastError();
  }
  const bool rows16 = a.tq > 1 || a.observe_first >= 0 || cv.G > 8;
  const int rows = rows16 ? kChunkRows : cv.G;
  if (rows16 && !plan.mfma) return hipErrorInvalidValue;
  AttendFn fn = plan.mfma ? attend_fn_mfma(cv.D, rows, cv.chan != 0) : attend_fn_valu(cv.D, cv.G);
  if (!fn) return hipErrorInvalidValue;
#ifdef CONFKV_TRACE
  if (a.dbg && plan.mfma) {             // time stamps live in LDS behind the kernel's own
    AttendLaunch at = a;
    at.trace_off = (int)((plan.lds_bytes + 15) / 16 * 16);
    const size_t lds = at.trace_off + kAttWaves * 32 * 8;
    (void)hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(fn, grid, dim3(kAttThreads), lds, stream, cv.len, cv.n8, cv.head16, cv.head8, a.layer * cv.B * cv.Hkv, cv.Hkv, a.kv_major, cv, at, plan.splits, plan.stash_tokens);
    return hipGetLastError();
  }
#endif
  hipLaunchKernelGGL(fn, grid, dim3(kAttThreads), plan.lds_bytes, stream, cv.len, cv.n8, cv.head16, cv.head8, a.layer * cv.B * cv.Hkv, cv.Hkv, a.kv_major, cv, a, plan.splits,
                     plan.stash_tokens);
  return hipGetLastError();
}

}  // namespace confkv

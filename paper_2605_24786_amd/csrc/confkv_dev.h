// Device-side view of the cache state and small wavefront / workgroup helpers shared by
// the kernels of the Conf-KV decode-step library.  gfx950 only: 64-lane wavefronts.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace confkv {

constexpr int kWave = 64;
constexpr int kMaxLayers = 256;

// Indices into the device statistics block (unsigned long long each).
enum StatSlot { kStatEvicted = 0, kStatDemoted = 1, kStatTight = 2, kStatLoose = 3,
                kStatDeviceErr = 4, kStatSlots = 8 };

// All planes of the cache, for every unit u = (layer * B + b) * Hkv + kv_head.
//   k8, v8   int8  [U][cap8][D]   INT8 ring; slot i < n8[u] lives in ring row
//                                 (head8[u] + i) mod cap8
//   ks, vs   fp16  [U][cap8]      per-token scales of those rows (same ring index); with
//                                 per-channel scales (chan != 0): [U][D], one scale per channel
//   k16, v16 fp16  [U][cap16][D]  FP16 ring; slot i >= n8[u] lives in ring row
//                                 (head16[u] + i - n8[u]) mod cap16
//   ema      fp32  [U][cap]       EMA of attention mass; slot i lives at (head8[u] + i) mod cap
//   pos      int32 [U][cap]       original position (strictly increasing over the slots), same index
//   len, n8, head16, head8  int32 [U]  committed length, INT8 count, ring heads.  head8 is the
//                                 head of every ring anchored at the oldest slot: EMA, position
//                                 and, in mixed caches (cap8 = cap), the INT8 rows and scales
//   budget   int32 [L][B]         N selected by the last confidence step
//   unit_evicted, unit_demoted  uint32 [U]  tokens evicted / demoted so far, per unit
//   unit_moved  uint64 [U]        bytes read + written by compaction moves so far, per unit
struct CacheView {
  int8_t *k8, *v8;
  __half *ks, *vs;
  __half *k16, *v16;
  float *ema;
  int32_t *pos;
  int32_t *len, *n8, *head16, *head8, *budget;
  const int32_t *n_tight, *n_loose;
  unsigned long long *stats;
  unsigned *unit_evicted, *unit_demoted;   // [U] per-unit event counts
  unsigned long long *unit_moved;          // [U] per-unit compaction traffic
  int32_t L, B, Hkv, G, D, cap, cap8, cap16, W, P;
  int32_t chan;                            // INT8 scales are per (unit, channel), not per token
  // Paged layout (page_lg > 0): the INT8 slots of a unit live in pages of 2^page_lg rows of the
  // INT8 planes, reached through the unit's block table pt[u][0 .. npages): entries
  // [0, ceil(n8 / page)) are the live pages in slot order, the rest the free ones, so the table
  // is always a permutation of the physical pages.  Slot i < n8 (codes, scales, EMA, position)
  // lives in row pt[u][i >> page_lg] * page + (i & (page - 1)); the EMA and position of an FP16
  // slot i >= n8 live in row cap - cap16 + (its FP16 ring row); head8 stays 0.
  int32_t *pt;
  int32_t page_lg, npages;
  // Step state the kernels advance themselves, so that no launch argument changes from one
  // decode step to the next (see CtlSlot), and the epoch-tagged exchange words of the attention
  // and confidence kernels (all of them, for the clearing before the tags start over).
  unsigned *ctl;
  unsigned long long *tagged;
  unsigned long long n_tagged;
};

// cv.ctl: [kCtlTag] tags handed out to attention launches up to the last commit (a launch's tag
// is this plus its number since then, so never 0), [kCtlConfTag] the same for the confidence
// kernel, [kCtlClear] 1 = the bases are near the end of their range: the next commit clears the
// tagged words and starts both over, [kCtlPos + l] position the next token appended to layer l gets.
enum CtlSlot { kCtlTag = 0, kCtlConfTag = 1, kCtlClear = 2, kCtlPos = 4 };
constexpr unsigned kTagRestart = 0xFF000000u;      // a base above this asks for the clearing
constexpr unsigned kTagLaunchesMax = 1u << 23;     // launches between two commits (host-enforced)

// Row of slot i in the planes anchored at the oldest slot (EMA, position; for i < n8 also the
// INT8 codes and per-token scales), in either layout.  tab: the unit's block table.
__device__ __forceinline__ int slot_row(const CacheView &cv, const int32_t *tab, int h8, int n8, int h16, int i) {
  if (cv.page_lg == 0) {
    const unsigned r = (unsigned)(h8 + i);
    return (int)min(r, r - (unsigned)cv.cap);
  }
  if (i < n8) return (tab[i >> cv.page_lg] << cv.page_lg) | (i & ((1 << cv.page_lg) - 1));
  int r = h16 + (i - n8);
  r = r >= cv.cap16 ? r - cv.cap16 : r;
  return cv.cap - cv.cap16 + r;
}

// Per layer: tokens appended by conf_kv_attend / conf_kv_attend_chunk since the last commit.
struct LayerMask {
  unsigned char c[kMaxLayers];
  __host__ __device__ int get(int l) const { return c[l]; }
  __host__ __device__ void set(int l, int count) { c[l] = (unsigned char)count; }
};

__device__ __forceinline__ int ring_row(int head, int idx, int cap16) {
  int r = head + idx;
  return r >= cap16 ? r - cap16 : r;
}
// Same for 0 <= head + idx < 2 * cap in two instructions: the subtraction wraps to a huge
// unsigned value exactly when no wrap of the ring is due.
__device__ __forceinline__ int ring_row_u(int head, int idx, int cap) {
  const unsigned r = (unsigned)(head + idx);
  return (int)min(r, r - (unsigned)cap);
}

// Streaming (non-temporal) accesses for data a kernel touches once: cache rows, logits, per-slot
// planes.  They leave the caches to data that is used again, and they are measurably faster
// here: the attention kernel's tile loads alone take 1.4 us off a 20.5 us launch.
typedef int confkv_v4i __attribute__((ext_vector_type(4)));
typedef unsigned confkv_v2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ int4 ld_stream16(const void *p) {
  const confkv_v4i v = __builtin_nontemporal_load((const confkv_v4i *)p);
  return make_int4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream16(void *p, const int4 &v) {
  __builtin_nontemporal_store(confkv_v4i{v.x, v.y, v.z, v.w}, (confkv_v4i *)p);
}
__device__ __forceinline__ void st_stream8(void *p, const uint2 &v) {
  __builtin_nontemporal_store(confkv_v2u{v.x, v.y}, (confkv_v2u *)p);
}
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v) { __builtin_nontemporal_store(v, p); }

// ---- wavefront reductions (all 64 lanes end with the result) ----
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fminf(v, __shfl_xor(v, m, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
__device__ __forceinline__ double wave_min(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmin(v, __shfl_xor(v, m, kWave));
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmax(v, __shfl_xor(v, m, kWave));
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = min(v, __shfl_xor(v, m, kWave));
  return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = max(v, __shfl_xor(v, m, kWave));
  return v;
}

// Inclusive prefix sum across the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_scan_incl(int v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int t = __shfl_up(v, d, kWave);
    if (lane >= d) v += t;
  }
  return v;
}

// Exclusive prefix sum over a 256-thread workgroup; *total gets the workgroup sum.
// `tmp` is 4 ints of LDS.  Contains two barriers; all 256 threads must call it.
__device__ __forceinline__ int block256_scan_excl(int v, int *tmp, int *total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
  int inc = wave_scan_incl(v);
  __syncthreads();                       // tmp may still be read from a previous call
  if (lane == kWave - 1) tmp[w] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    int t = tmp[k];
    if (k < w) off += t;
    tot += t;
  }
  *total = tot;
  return off + inc - v;
}

}  // namespace confkv

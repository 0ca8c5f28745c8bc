// Ranker, top-k eviction, in-place compaction and FP16 -> INT8 demotion, plus the prompt
// loader (paper: "Budget and ranker" -- composite score of min-max-normalised EMA mass and
// recency over the non-protected candidates, evict the lowest until the budget holds,
// always keep the newest P; "Cache manager" -- gather survivors into contiguous storage;
// "Tiled attention and mixed precision" -- symmetric INT8 with scale max|x|/127 outside
// the FP16 window; Algorithm 1, per-layer tail).
//
// Three launches cover every layer:
//   rank_select   one 1024-thread workgroup per unit: float64 scores, radix select of the eviction
//                 cut-off, ordered survivor list
//   compact       one workgroup per (unit, plane): in-place, order-preserving gather
//   demote        one wavefront per unit: quantise the FP16 slots that left the window,
//                 commit the new lengths
#include "confkv_dev.h"
#include "launch.h"

namespace confkv {

constexpr int kEvThreads = 256;

// ---------------------------------------------------------------------------------------
// Quantiser shared by the prompt loader and the demotion kernel.
// One wavefront quantises one D-vector: scale = fl16(fl32(amax / 127)),
// code = clamp(rint(x / scale), -127, 127) with IEEE fp32 division and round-half-even.
// ---------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void quantize_row_wave(const __half *__restrict__ src,
                                                  int8_t *__restrict__ dst_codes,
                                                  __half *__restrict__ dst_scale, int lane) {
  constexpr int EPL = D / kWave;                 // elements per lane (1 or 2)
  float x[EPL];
  if constexpr (EPL == 2) {
    const __half2 v = ((const __half2 *)src)[lane];
    x[0] = __low2float(v);
    x[1] = __high2float(v);
  } else {
    x[0] = __half2float(src[lane]);
  }
  float amax = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) amax = fmaxf(amax, fabsf(x[e]));
  amax = wave_max(amax);
  const __half hs = __float2half_rn(__fdiv_rn(amax, 127.0f));
  const float sf = __half2float(hs);
  const bool dead = !(sf > 0.f) || isinf(sf);
  int code[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    float r = dead ? 0.f : rintf(__fdiv_rn(x[e], sf));
    r = fminf(fmaxf(r, -127.f), 127.f);
    code[e] = (int)r;
  }
  if constexpr (EPL == 2) {
    ((unsigned short *)dst_codes)[lane] = (unsigned short)((code[0] & 0xff) | ((code[1] & 0xff) << 8));
  } else {
    dst_codes[lane] = (int8_t)code[0];
  }
  if (lane == 0) *dst_scale = dead ? __float2half_rn(0.f) : hs;
}

// The same with fixed per-channel scales ("Tiled attention and mixed precision": per head and
// channel): code_d = clamp(rint(x_d / s_d), -127, 127); a channel whose scale is 0 gets code 0.
template <int D>
__device__ __forceinline__ void quantize_row_channels(const __half *__restrict__ src,
                                                      int8_t *__restrict__ dst_codes,
                                                      const __half *__restrict__ scales, int lane) {
  constexpr int EPL = D / kWave;
  static_assert(EPL == 2, "per-channel scales are built for D = 128");
  const __half2 v = ((const __half2 *)src)[lane];
  const __half2 sc = ((const __half2 *)scales)[lane];
  const float x[2] = {__low2float(v), __high2float(v)};
  const float sf[2] = {__low2float(sc), __high2float(sc)};
  int code[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    float r = (sf[e] > 0.f) ? rintf(__fdiv_rn(x[e], sf[e])) : 0.f;
    r = fminf(fmaxf(r, -127.f), 127.f);
    code[e] = (int)r;
  }
  ((unsigned short *)dst_codes)[lane] = (unsigned short)((code[0] & 0xff) | ((code[1] & 0xff) << 8));
}

// ---------------------------------------------------------------------------------------
// Channel scales of a prompt: grid (B * Hkv, 2), plane 0 = K, 1 = V; 1024 threads.  Thread t
// owns the 8 channels of 16-byte piece t % 16 on the rows t / 16, t / 16 + 64, ...;
// scale_d = fl16(fl32(max_t |x_{t,d}| / 127)), 0 when that is not finite.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void channel_scales_kernel(CacheView cv, int layer,
                                                              const __half *__restrict__ k16,
                                                              const __half *__restrict__ v16, int T0) {
  constexpr int D = 128, PIECES = D / 8, ROWS = 1024 / PIECES;
  __shared__ unsigned short part[ROWS][D];
  const int ul = blockIdx.x, tid = threadIdx.x;
  const int u = layer * cv.B * cv.Hkv + ul;
  const int c = tid % PIECES, r0 = tid / PIECES;
  const __half *src = (blockIdx.y ? v16 : k16) + (size_t)ul * T0 * D;
  // |x| as fp16 bits with the sign cleared: for finite values and infinities the bit patterns
  // order like the magnitudes, so the maximum is taken on 16-bit integers
  unsigned short m[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int t = r0; t < T0; t += ROWS) {
    const int4 raw = *(const int4 *)(src + (size_t)t * D + c * 8);
    const unsigned w[4] = {(unsigned)raw.x, (unsigned)raw.y, (unsigned)raw.z, (unsigned)raw.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      m[2 * e] = max(m[2 * e], (unsigned short)(w[e] & 0x7fffu));
      m[2 * e + 1] = max(m[2 * e + 1], (unsigned short)((w[e] >> 16) & 0x7fffu));
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[r0][c * 8 + e] = m[e];
  __syncthreads();
  if (tid < D) {
    unsigned short best = 0;
    for (int r = 0; r < ROWS; ++r) best = max(best, part[r][tid]);
    const float amax = __half2float(__ushort_as_half(best));      // NaN patterns stay NaN
    const __half hs = __float2half_rn(__fdiv_rn(amax, 127.0f));
    const float sf = __half2float(hs);
    const bool dead = !(sf > 0.f) || isinf(sf);
    ((blockIdx.y ? cv.vs : cv.ks) + (size_t)u * D)[tid] = dead ? __float2half_rn(0.f) : hs;
  }
}

// ---------------------------------------------------------------------------------------
// Prompt loader: grid (ceil(T0 / RW), B * Hkv), 256 threads.  D / 8 lanes own one token row in
// 16-byte pieces (eight fp16 values each), so a workgroup takes RW = 2048 / D tokens and every
// load and store instruction covers whole rows.  Same arithmetic per element as
// quantize_row_wave (the maximum does not depend on the order it is taken in), so the stored
// bits are those of the one-row-per-wavefront quantiser the demotion kernel uses.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void unpack_h8(const int4 &raw, float (&x)[8]) {
  const unsigned w[4] = {(unsigned)raw.x, (unsigned)raw.y, (unsigned)raw.z, (unsigned)raw.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    x[2 * e] = __half2float(__ushort_as_half((unsigned short)(w[e] & 0xffffu)));
    x[2 * e + 1] = __half2float(__ushort_as_half((unsigned short)(w[e] >> 16)));
  }
}
__device__ __forceinline__ uint2 pack_codes8(const int (&code)[8]) {
  uint2 r;
  r.x = (unsigned)(code[0] & 0xff) | ((unsigned)(code[1] & 0xff) << 8) | ((unsigned)(code[2] & 0xff) << 16) |
        ((unsigned)(code[3] & 0xff) << 24);
  r.y = (unsigned)(code[4] & 0xff) | ((unsigned)(code[5] & 0xff) << 8) | ((unsigned)(code[6] & 0xff) << 16) |
        ((unsigned)(code[7] & 0xff) << 24);
  return r;
}
// Eight values of a row per lane, LPR lanes per row: per-token scale of the row and the codes.
template <int LPR>
__device__ __forceinline__ uint2 quantize_piece(const int4 &raw, __half *scale_out) {
  float x[8];
  unpack_h8(raw, x);
  float amax = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, kWave));
  const __half hs = __float2half_rn(__fdiv_rn(amax, 127.0f));
  const float sf = __half2float(hs);
  const bool dead = !(sf > 0.f) || isinf(sf);
  int code[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float r = dead ? 0.f : rintf(__fdiv_rn(x[e], sf));
    r = fminf(fmaxf(r, -127.f), 127.f);
    code[e] = (int)r;
  }
  *scale_out = dead ? __float2half_rn(0.f) : hs;
  return pack_codes8(code);
}
// The same piece against fixed per-channel scales (eight fp16 scales of the lane's channels).
__device__ __forceinline__ uint2 quantize_piece_channels(const int4 &raw, const int4 &scales) {
  float x[8], sf[8];
  unpack_h8(raw, x);
  unpack_h8(scales, sf);
  int code[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float r = (sf[e] > 0.f) ? rintf(__fdiv_rn(x[e], sf[e])) : 0.f;
    r = fminf(fmaxf(r, -127.f), 127.f);
    code[e] = (int)r;
  }
  return pack_codes8(code);
}

template <int D>
__global__ __launch_bounds__(kEvThreads) void load_prefill_kernel(
    CacheView cv, int layer, const __half *__restrict__ k16, const __half *__restrict__ v16, int T0,
    const float *__restrict__ ema0) {
  constexpr int LPR = D / 8, RW = kEvThreads / LPR;
  const int c = threadIdx.x % LPR;
  const int ul = blockIdx.y;
  const int u = layer * cv.B * cv.Hkv + ul;
  const int t = blockIdx.x * RW + threadIdx.x / LPR;
  const int n8 = (cv.W < 0) ? 0 : max(0, T0 - cv.W);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    cv.len[u] = T0;
    cv.n8[u] = n8;
    cv.head16[u] = 0;
    cv.head8[u] = 0;
    if (ul == 0) cv.ctl[kCtlPos + layer] = (unsigned)T0;      // the first decode token's position
  }
  if (cv.page_lg && blockIdx.x == 0)                // paged layout: the block table starts over as the identity
    for (int i = threadIdx.x; i < cv.npages; i += kEvThreads) cv.pt[(size_t)u * cv.npages + i] = i;
  if (t >= T0) return;                              // (the LPR lanes of a row leave together)
  // the prompt is read once and the cache rows are not read again before gigabytes of other
  // traffic: streaming loads and stores, so the loader leaves the caches to the decode kernels
  typedef int v4i_t __attribute__((ext_vector_type(4)));
  typedef unsigned v2u_t __attribute__((ext_vector_type(2)));
  const v4i_t kl = __builtin_nontemporal_load((const v4i_t *)(k16 + ((size_t)ul * T0 + t) * D + c * 8));
  const v4i_t vl = __builtin_nontemporal_load((const v4i_t *)(v16 + ((size_t)ul * T0 + t) * D + c * 8));
  const int4 kraw = make_int4(kl.x, kl.y, kl.z, kl.w), vraw = make_int4(vl.x, vl.y, vl.z, vl.w);
  if (c == 0) {
    // (identity table, ring heads 0: INT8 slot t sits in row t, FP16 slot t in metadata row t - n8)
    const int mrow = (cv.page_lg && t >= n8) ? cv.cap - cv.cap16 + (t - n8) : t;
    cv.pos[(size_t)u * cv.cap + mrow] = t;
    cv.ema[(size_t)u * cv.cap + mrow] = ema0 ? ema0[(size_t)ul * T0 + t] : 0.f;
  }
  if (t < n8) {
    const size_t row = (size_t)u * cv.cap8 + t;
    uint2 kc, vc;
    if (D == 128 && cv.chan) {                      // scales were fixed by channel_scales_kernel
      kc = quantize_piece_channels(kraw, *(const int4 *)(cv.ks + (size_t)u * D + c * 8));
      vc = quantize_piece_channels(vraw, *(const int4 *)(cv.vs + (size_t)u * D + c * 8));
    } else {
      __half ksc, vsc;
      kc = quantize_piece<LPR>(kraw, &ksc);
      vc = quantize_piece<LPR>(vraw, &vsc);
      if (c == 0) { cv.ks[row] = ksc; cv.vs[row] = vsc; }
    }
    __builtin_nontemporal_store(v2u_t{kc.x, kc.y}, (v2u_t *)(cv.k8 + row * D + c * 8));
    __builtin_nontemporal_store(v2u_t{vc.x, vc.y}, (v2u_t *)(cv.v8 + row * D + c * 8));
  } else {
    const size_t row = (size_t)u * cv.cap16 + (t - n8);   // both ring heads are 0 after a load
    __builtin_nontemporal_store(kl, (v4i_t *)(cv.k16 + row * D + c * 8));
    __builtin_nontemporal_store(vl, (v4i_t *)(cv.v16 + row * D + c * 8));
  }
}

// ---------------------------------------------------------------------------------------
// Correctly rounded float64 quotients n / d for many numerators and one denominator.
// The compiler's own division is rcp, two Newton steps on the reciprocal, then
// q0 = n y, r = fma(-d, q0, n), q = fma(r, y, q0) (plus range scaling that only acts outside
// the ranges met here: d and n are differences of float32 values or of int32 positions, so
// d lies in [2^-149, 2^129] and n in {0} or [2^-149, d]).  The reciprocal part depends on d
// alone and is done once per unit; the three per-numerator operations are the same ones, so
// the quotient has the same bits as n / d.
// ---------------------------------------------------------------------------------------
struct Divisor {
  double d, y;
};
__device__ __forceinline__ Divisor make_divisor(double d) {
  double y = __builtin_amdgcn_rcp(d);
  double e = __builtin_fma(-d, y, 1.0);
  y = __builtin_fma(y, e, y);
  e = __builtin_fma(-d, y, 1.0);
  y = __builtin_fma(y, e, y);
  return Divisor{d, y};
}
__device__ __forceinline__ double quotient(double n, const Divisor &dv) {
  const double q0 = __dmul_rn(n, dv.y);
  const double r = __builtin_fma(-dv.d, q0, n);
  return __builtin_fma(r, dv.y, q0);
}

// ---------------------------------------------------------------------------------------
// Outcome of one unit's selection.  Every plane is a ring, so the survivors can close the
// holes from either side: slots behind the first hole shift left (heads stay), or slots in
// front of the last hole shift right (the head of the rings anchored at the oldest slot
// advances by the number of evictions).  The side with fewer rows to move is taken; in steady
// state the evicted slot is old, so the right shift moves next to nothing.  The right shift is
// open when all holes lie in one payload ring: all INT8 in a mixed cache (the FP16 slots, newer
// than every hole, then keep their rows), any in an FP16-only cache.
// `last_hole` is the newest evicted slot of that ring (-1: none).
// ---------------------------------------------------------------------------------------
struct ShiftPlan {
  int right;        // 1: slots in front of the last hole shift right
  int left_rows;    // payload rows a left shift would move
  int right_rows;   // payload rows (= slots) a right shift would move
  int lo, hi;       // new slot numbers [lo, hi) that move, i.e. whose source slot the compaction looks up
};
__device__ __forceinline__ ShiftPlan shift_plan(const CacheView &cv, int n_new, int n8_old, int n8_new,
                                                int first_hole, int evicted, int last_hole) {
  const bool fp16_only = cv.cap8 == 0;
  const int e8 = n8_old - n8_new;
  const int span = fp16_only ? n_new : n8_new;       // survivors of the ring the holes lie in
  ShiftPlan p;
  p.left_rows = span - min(first_hole, span);
  p.right_rows = last_hole + 1 - (fp16_only ? evicted : e8);   // survivors in front of the last hole
  p.right = (fp16_only ? evicted > 0 : (e8 > 0 && evicted == e8)) && p.right_rows < p.left_rows;
  p.lo = p.right ? 0 : min(first_hole, n_new);
  p.hi = p.right ? p.right_rows : n_new;
  return p;
}

__device__ __forceinline__ void write_selection(const CacheView &cv, int u, int32_t *sel, int n_new,
                                                int n8_old, int n8_new, int first_hole, int evicted,
                                                int last_hole) {
  const bool fp16_only = cv.cap8 == 0;
  const int h0 = cv.head8[u];
  const int e8 = n8_old - n8_new;
  const ShiftPlan sp = shift_plan(cv, n_new, n8_old, n8_new, first_hole, evicted, last_hole);
  const int right = sp.right, left_rows = sp.left_rows, right_rows = sp.right_rows;
  sel[0] = n_new;
  sel[1] = n8_new;
  sel[2] = first_hole;
  sel[3] = evicted;
  sel[4] = last_hole;
  sel[5] = cv.page_lg ? 0 : right;
  sel[6] = cv.page_lg ? 0 : (right ? ring_row(h0, fp16_only ? evicted : e8, cv.cap) : h0);
  sel[7] = 1;                                        // this unit's selection is final
  if (evicted > 0 && cv.page_lg) {
    // paged layout: whole pages leave, the block table is rewritten, no row moves
    cv.unit_moved[u] += 2ull * 4ull * (unsigned long long)((n8_old + (1 << cv.page_lg) - 1) >> cv.page_lg);
  } else if (evicted > 0) {
    // traffic of the moves the compaction kernel will make (each row is read and written once)
    const long long meta = right ? right_rows : n_new - min(first_hole, n_new);
    long long rows8 = 0, rows16 = 0;
    if (fp16_only) {
      rows16 = right ? right_rows : left_rows;
    } else {
      rows8 = right ? right_rows : left_rows;
      rows16 = (evicted > e8) ? n_new - max(first_hole, n8_new) : 0;
    }
    const int scale_bytes = cv.chan ? 0 : 4;           // per-token scales travel with their rows
    cv.unit_moved[u] += 2ull * (unsigned long long)(rows8 * (2 * cv.D + scale_bytes) + rows16 * 4 * cv.D + meta * 8);
  }
}

// ---------------------------------------------------------------------------------------
// rank_select: grid (U), 256 threads (1024 for long units, which would otherwise take
// dozens of chunk rounds).
//
// score_i = alpha * a_hat_i + (1 - alpha) * r_hat_i in float64 with every operation
// rounded separately (no fused multiply-add), so equal inputs give bit-equal scores on
// any IEEE machine.  The e lowest (score, slot) pairs are evicted: an 8-bit-digit radix
// select over the score's bit pattern (non-negative doubles order like unsigned integers)
// finds the cut-off, stopping as soon as the cut-off bucket is evicted whole; slots that
// tie with the cut-off go oldest first (this needs a second prefix sum only when the
// select ran to the last digit and equal scores straddle the cut-off).
// ---------------------------------------------------------------------------------------

// Exclusive prefix sum over a workgroup of kRsWaves wavefronts (<= 16); *total gets the
// workgroup sum.  `tmp` is kRsWaves ints of LDS.  Contains barriers; all threads must call it.
template <int kRsWaves>
__device__ __forceinline__ int block_scan_excl(int v, int *tmp, int *total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
  const int inc = wave_scan_incl(v);
  __syncthreads();                       // tmp may still be read from a previous call
  if (lane == kWave - 1) tmp[w] = inc;
  __syncthreads();
  int mine = lane < kRsWaves ? tmp[lane] : 0;
  const int incw = wave_scan_incl(mine);                 // every wave scans the 16 wave totals
  const int off = __shfl(incw - mine, w, kWave);         // exclusive offset of this wave
  *total = __shfl(incw, kRsWaves - 1, kWave);
  return off + inc - v;
}

// SplitMix64 (Steele, Lea, Flood 2014): one output for state x.
__device__ __forceinline__ unsigned long long splitmix64(unsigned long long x) {
  unsigned long long z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Random ranker: the score of a slot is a counter-based uniform draw keyed by (seed, unit or
// (layer, sequence), original position), as the bits of the double it is: exact (53 bits, a
// power-of-two scale), so it orders like the oracle's draw.
struct RandomRank {
  int on;                      // 0: the composite score
  int layer_scope;             // the kv-heads of a (layer, sequence) draw the same numbers
  unsigned long long seed;
};
__device__ __forceinline__ unsigned long long random_unit_key(const CacheView &cv, const RandomRank &rr, int u) {
  return rr.layer_scope ? (1ull << 40) + (unsigned long long)(u / cv.Hkv) : (unsigned long long)u;
}
__device__ __forceinline__ unsigned long long random_key(const RandomRank &rr, unsigned long long unit_key, int pos) {
  const unsigned long long r = splitmix64(rr.seed + (unit_key << 32) + (unsigned long long)(long long)pos);
  return (unsigned long long)__double_as_longlong((double)(r >> 11) * 0x1.0p-53);
}

// Layer scope: shared[(layer, b)][slot] = sum over the kv-heads, in kv-head order, of the
// unit's EMA as float64.  Grid (L * B, ceil(cap / 256)).
__global__ __launch_bounds__(kEvThreads) void shared_mass_kernel(CacheView cv, LayerMask appended,
                                                                 double *__restrict__ shared) {
  const int lb = blockIdx.x, i = blockIdx.y * kEvThreads + threadIdx.x;
  const int u0 = lb * cv.Hkv;
  const int n = cv.len[u0] + appended.get(lb / cv.B);
  if (i >= n) return;
  double acc = 0.0;
  for (int g = 0; g < cv.Hkv; ++g)
    acc = __dadd_rn(acc, (double)cv.ema[(size_t)(u0 + g) * cv.cap + ring_row_u(cv.head8[u0 + g], i, cv.cap)]);
  shared[(size_t)lb * cv.cap + i] = acc;
}

// The general kernel also serves the ranker variants: importance shared by the kv-heads of a
// (layer, sequence) -- every unit of the group then ranks the same numbers and reaches the same
// kept set -- and the random ranker.  check_settled = 0 when rank_small_kernel has not run.
template <int kRsThreads>
__global__ __launch_bounds__(kRsThreads) void rank_select_kernel(CacheView cv, LayerMask appended,
                                                                 double alpha, RankOptions opt,
                                                                 int check_settled,
                                                                 double *__restrict__ score_all,
                                                                 int32_t *__restrict__ src_all,
                                                                 int32_t *__restrict__ sel_all) {
  constexpr int kRsWaves = kRsThreads / kWave;
  __shared__ int hist[256];
  __shared__ int s_tmp[kRsWaves];
  __shared__ double s_fmin[kRsWaves], s_fmax[kRsWaves];
  __shared__ unsigned long long s_prefix;
  __shared__ int s_krem, s_done, s_hole[kRsWaves], s_k8[kRsWaves], s_last8[kRsWaves];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int u = blockIdx.x;
  const int UPL = cv.B * cv.Hkv;
  const int layer = u / UPL, b = (u % UPL) / cv.Hkv;
  const int n = cv.len[u] + appended.get(layer);
  const int n8 = cv.n8[u];
  const int N = cv.budget[layer * cv.B + b];
  int32_t *sel = sel_all + (size_t)u * kSelInts;
  if (check_settled && sel[7] != 0) return;           // settled by rank_small_kernel
  const int p_eff = min(cv.P, n);
  const int ncand = n - p_eff;
  const int e = min(n - N, ncand);
  if (n <= N || e <= 0) {
    if (tid == 0) write_selection(cv, u, sel, n, n8, n8, n, 0, -1);
    return;
  }
  const float *ema = cv.ema + (size_t)u * cv.cap;
  const int32_t *pos = cv.pos + (size_t)u * cv.cap;
  const int hm = cv.head8[u];                        // slot i of the per-slot planes: row_of(i)
  const int h16 = cv.head16[u];
  const int32_t *tab = cv.pt + (size_t)u * cv.npages;   // paged layout: the unit's block table
  auto row_of = [&](int i) { return slot_row(cv, tab, hm, n8, h16, i); };
  const int nx = cv.cap8 == 0 ? n : n8;              // slots of the ring a right shift could serve
  double *score = score_all + (size_t)u * cv.cap;
  int32_t *src = src_all + (size_t)u * cv.cap;

  // importance of slot i: the unit's own EMA, or the sum shared by the (layer, sequence)
  const double *shared = opt.shared ? opt.shared + (size_t)(u / cv.Hkv) * cv.cap : nullptr;
  // min / max of the importance over the candidates (float -> double is exact and monotone)
  double fmin_ = INFINITY, fmax_ = -INFINITY;
  for (int i = tid; i < ncand; i += kRsThreads) {
    const double a = shared ? shared[i] : (double)ema[row_of(i)];
    fmin_ = fmin(fmin_, a);
    fmax_ = fmax(fmax_, a);
  }
  fmin_ = wave_min(fmin_);
  fmax_ = wave_max(fmax_);
  if (lane == 0) { s_fmin[w] = fmin_; s_fmax[w] = fmax_; }
  if (tid == 0) { s_prefix = 0ull; s_krem = e; s_done = 0; }
  __syncthreads();
  double a_lo = s_fmin[0], a_hi = s_fmax[0];
#pragma unroll
  for (int k = 1; k < kRsWaves; ++k) { a_lo = fmin(a_lo, s_fmin[k]); a_hi = fmax(a_hi, s_fmax[k]); }
  // slots are position-sorted
  const double p_lo = (double)pos[row_of(0)], p_hi = (double)pos[row_of(ncand - 1)];
  const double a_rng = __dsub_rn(a_hi, a_lo), p_rng = __dsub_rn(p_hi, p_lo);
  const double oma = __dsub_rn(1.0, alpha);
  const Divisor a_div = make_divisor(a_rng == 0.0 ? 1.0 : a_rng), p_div = make_divisor(p_rng == 0.0 ? 1.0 : p_rng);
  const unsigned long long unit_key = shared ? (1ull << 40) + (unsigned long long)(u / cv.Hkv) : (unsigned long long)u;
  for (int i = tid; i < ncand; i += kRsThreads) {
    if (opt.random) {
      const unsigned long long r =
          splitmix64(opt.seed + (unit_key << 32) + (unsigned long long)(long long)pos[row_of(i)]);
      score[i] = (double)(r >> 11) * 0x1.0p-53;     // exact: 53 bits, power-of-two scale
    } else {
      const double a = shared ? shared[i] : (double)ema[row_of(i)];
      const double ah = (a_rng == 0.0) ? 0.0 : quotient(__dsub_rn(a, a_lo), a_div);
      const double rh = (p_rng == 0.0) ? 0.0 : quotient(__dsub_rn((double)pos[row_of(i)], p_lo), p_div);
      score[i] = __dadd_rn(__dmul_rn(alpha, ah), __dmul_rn(oma, rh));
    }
  }
  __syncthreads();                                  // orders the score writes before the reads

  // Coarsened eviction: whole pages of opt.page original positions go.  Slots are
  // position-sorted, so a page is a run of consecutive slots; the thread of its first slot
  // adds up the token scores in slot order, and the page's mean replaces that slot's score.
  // src[] holds, until the survivor list is written into it, the slot count of every page
  // that can go at its first slot (a page with a slot in the protected window cannot),
  // later -1 at every slot that goes, 0 elsewhere.
  const int pg = opt.page;
  bool all_go = false;                              // every page that can go goes: no select
  if (pg > 1) {
    for (int i = tid; i < n; i += kRsThreads) src[i] = 0;
    __syncthreads();
    int can = 0;
    for (int i = tid; i < ncand; i += kRsThreads) {
      const int pid = pos[row_of(i)] / pg;
      if (i == 0 || pos[row_of(i - 1)] / pg != pid) {
        double tot = 0.0;
        int m = i;
        // the page's slots in slot order, eight requested at a time (positions rise with the
        // slots, so the page ends at the first position at or past its upper bound)
        const int pend = (pid + 1) * pg;
        for (bool open = true; open;) {
          int pp[8];
          double sc8[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            pp[k] = pos[row_of(min(m + k, n - 1))];
            sc8[k] = score[min(m + k, ncand - 1)];
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            if (open && m < n && pp[k] < pend) {
              if (m < ncand) tot = __dadd_rn(tot, sc8[k]);
              ++m;
            } else {
              open = false;
            }
          }
        }
        if (m <= ncand) {
          score[i] = __ddiv_rn(tot, (double)(m - i));
          src[i] = m - i;
          can += m - i;
        }
      }
    }
    can = wave_sum(can);
    if (lane == 0) s_tmp[w] = can;
    __syncthreads();
    can = 0;
#pragma unroll
    for (int k = 0; k < kRsWaves; ++k) can += s_tmp[k];
    __syncthreads();                                // s_tmp is reused by the scans below
    if (can == 0) {
      if (tid == 0) write_selection(cv, u, sel, n, n8, n8, n, 0, -1);
      return;
    }
    all_go = can <= e;
  }

  // radix select of the e-th smallest score (of the page whose slots take the count to e)
  unsigned long long mask = 0ull;
  for (int shift = 56; shift >= 0 && !all_go; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const unsigned long long prefix = s_prefix;
    for (int i = tid; i < ncand; i += kRsThreads) {
      const int wgt = pg > 1 ? src[i] : 1;
      if (wgt > 0) {                                  // (with pages only a page's first slot carries a score)
        const unsigned long long key = (unsigned long long)__double_as_longlong(score[i]);
        if ((key & mask) == prefix) atomicAdd(&hist[(int)((key >> shift) & 255ull)], wgt);
      }
    }
    __syncthreads();
    const int cnt = tid < 256 ? hist[tid] : 0;
    int total;
    const int before = block_scan_excl<kRsWaves>(cnt, s_tmp, &total);
    const int krem = s_krem;
    __syncthreads();                                // every thread has read s_krem
    if (tid < 256 && before < krem && krem <= before + cnt) {   // exactly one bin holds the cut-off
      s_prefix = prefix | ((unsigned long long)tid << shift);
      s_krem = krem - before;
      s_done = (krem - before == cnt);              // the whole bucket goes
    }
    mask |= 255ull << shift;
    __syncthreads();
    if (s_done) break;
  }
  const unsigned long long prefix = s_prefix;
  const int krem = s_krem;
  const bool whole_bucket = s_done != 0;            // no tie ranking needed

  int carry_keep = 0, carry_tie = 0, kept8 = 0, hole = n, last8 = -1;
  if (pg > 1) {
    // page decisions, in slot order (pages that tie with the cut-off go oldest first until the
    // count is reached); the thread of a page's first slot marks all its slots
    for (int base = 0; base < ncand; base += kRsThreads) {
      const int i = base + tid;
      const int wgt = i < ncand ? max(src[i], 0) : 0;
      int tie = 0, below = 0;
      if (wgt > 0) {
        const unsigned long long km = (unsigned long long)__double_as_longlong(score[i]) & mask;
        below = km < prefix;
        tie = km == prefix;
      }
      int go;
      if (all_go) {
        go = wgt > 0;
      } else if (whole_bucket) {
        go = below | tie;
      } else {
        int tot_tie;
        const int before = carry_tie + block_scan_excl<kRsWaves>(tie ? wgt : 0, s_tmp, &tot_tie);
        carry_tie += tot_tie;
        go = below | (tie & (before < krem));
      }
      if (wgt > 0)
        for (int m = i; m < i + wgt; ++m) src[m] = go ? -1 : 0;
      __syncthreads();                              // marks may land in the next chunk's slots
    }
  }
  // survivor list in slot order; ties with the cut-off are evicted oldest first
  for (int base = 0; base < n; base += kRsThreads) {
    const int i = base + tid;
    int tie = 0, below = 0;
    if (pg <= 1 && i < ncand) {
      const unsigned long long km = (unsigned long long)__double_as_longlong(score[i]) & mask;
      below = km < prefix;
      tie = km == prefix;
    }
    int evict;
    if (pg > 1) {
      evict = i < ncand && src[i] < 0;              // read before the scan's barriers, overwritten after
    } else if (whole_bucket) {
      evict = below | tie;
    } else {
      int tot_tie;
      const int tie_rank = carry_tie + block_scan_excl<kRsWaves>(tie, s_tmp, &tot_tie);
      carry_tie += tot_tie;
      evict = below | (tie & (tie_rank < krem));
    }
    const int keep = (i < n) & !evict;
    int tot_keep;
    const int j = carry_keep + block_scan_excl<kRsWaves>(keep, s_tmp, &tot_keep);
    carry_keep += tot_keep;
    if (keep) {
      src[j] = i;
      kept8 += (i < n8);
    }
    if (evict) {
      hole = min(hole, i);
      if (i < nx) last8 = max(last8, i);
    }
  }
  kept8 = wave_sum(kept8);
  hole = wave_min(hole);
  last8 = wave_max(last8);
  if (lane == 0) { s_k8[w] = kept8; s_hole[w] = hole; s_last8[w] = last8; }
  __syncthreads();
  if (tid == 0) {
    int k8 = 0, hl = n, l8 = -1;
#pragma unroll
    for (int k = 0; k < kRsWaves; ++k) { k8 += s_k8[k]; hl = min(hl, s_hole[k]); l8 = max(l8, s_last8[k]); }
    // (n - carry_keep = e, or up to a page more under coarsened eviction)
    write_selection(cv, u, sel, carry_keep, n8, k8, hl, n - carry_keep, l8);
    cv.unit_evicted[u] += (unsigned)(n - carry_keep);   // per-unit counter: no contended atomic
  }
}

// ---------------------------------------------------------------------------------------
// rank_select, register-resident variant: grid (U), T threads; thread t owns the slots
// t, t + T, t + 2T, .. (at most E of them), so every load is coalesced and the scores never
// leave the registers between the select passes.  The survivor list is ranked with
// wavefront ballots: for slot round k, the kept lanes of a wavefront are counted with one
// ballot, the (round, wavefront) counts are prefix-summed once by the workgroup, and each
// kept slot lands at base(round, wavefront) + its rank inside the ballot.  Same arithmetic
// and same decisions as rank_select_kernel; used whenever the longest unit fits (n <= T * E).
// ---------------------------------------------------------------------------------------
// The per-unit words a ranking kernel starts from -- length, INT8 count, ring head, budget and
// the unit's "settled" mark -- in ONE memory round trip: lanes 0..4 of a wavefront read one
// word each with a single load (as separate scalar loads the compiler strings them out between
// the kernel-argument fetches, each waiting for the one before).
struct UnitWords { int len, n8, head, budget, settled; };
__device__ __forceinline__ UnitWords load_unit_words(const CacheView &cv, const int32_t *sel, int u, int layer, int b) {
  const int k = threadIdx.x & 7;
  const int32_t *p = k == 0 ? cv.len + u : k == 1 ? cv.n8 + u : k == 2 ? cv.head8 + u
                   : k == 3 ? cv.budget + (layer * cv.B + b) : sel + 7;
  const int v = *p;
  UnitWords w;
  w.len = __builtin_amdgcn_readlane(v, 0);
  w.n8 = __builtin_amdgcn_readlane(v, 1);
  w.head = __builtin_amdgcn_readlane(v, 2);
  w.budget = __builtin_amdgcn_readlane(v, 3);
  w.settled = __builtin_amdgcn_readlane(v, 4);
  return w;
}

__device__ __forceinline__ int lanes_below(unsigned long long m) {   // set bits of m below this lane
  return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0));
}

// kShared: the importance is the layer-shared float64 sum in shared_all (see rank_small_kernel).
// kRandom: the random ranker's key per slot instead of the composite score (rr says how it is drawn).
template <int T, int E, bool kShared = false, bool kRandom = false>
__global__ __launch_bounds__(T) __attribute__((amdgpu_waves_per_eu(T == 256 && !kShared ? 4 : 1, T == 256 && !kShared ? 4 : 8)))
void rank_select_reg_kernel(CacheView cv, LayerMask appended,
                                                            double alpha,
                                                            int32_t *__restrict__ src_all,
                                                            int32_t *__restrict__ sel_all,
                                                            const double *__restrict__ shared_all, RandomRank rr) {
  typedef typename std::conditional<kShared, double, float>::type Imp;   // importance as stored
  constexpr int kRsWaves = T / kWave;
  // width of the first radix pass: 11 bits where a workgroup has the threads to scan 2048 bins
  // (the one-wavefront instance keeps 8: its many small workgroups share a CU's LDS; so do the
  // layer-scope instances, which measured 6 us slower with the separate first pass: those start
  // with the 8-bit passes below)
  constexpr bool kWide0 = T >= 256 && !kShared;
  constexpr int kRadix0Bits = kWide0 ? 11 : 8, kRadix0Bins = kWide0 ? 1 << kRadix0Bits : 1;
  __shared__ int hist[512];                         // two histograms, used alternately
  __shared__ int hist0[kRadix0Bins];                // the wider histogram of the first pass
  __shared__ int s_tmp[kRsWaves];
  __shared__ int s_cnt[E * kRsWaves];               // tied lanes per (round, wavefront)
  __shared__ int s_keep[E * kRsWaves + 1];          // kept lanes per (round, wavefront), then their prefix sums
  __shared__ Imp s_fmin[kRsWaves], s_fmax[kRsWaves];
  __shared__ unsigned long long s_prefix, s_kmin[kRsWaves], s_kmax[kRsWaves];
  __shared__ int s_krem, s_done, s_hole[kRsWaves], s_k8[kRsWaves], s_last8[kRsWaves];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int u = blockIdx.x;
  // the kernel arguments of the prologue in one fetch
  asm volatile("" ::"s"(cv.len), "s"(cv.n8), "s"(cv.head8), "s"(cv.budget), "s"(cv.ema), "s"(cv.pos), "s"(cv.B),
               "s"(cv.Hkv), "s"(cv.P), "s"(cv.cap), "s"(cv.cap8), "s"(sel_all), "s"(src_all));
  const int UPL = cv.B * cv.Hkv;
  const int layer = u / UPL, b = (u % UPL) / cv.Hkv;
  int32_t *sel = sel_all + (size_t)u * kSelInts;
  const int app = appended.get(layer);
  const UnitWords uw = load_unit_words(cv, sel, u, layer, b);
  if (uw.settled != 0) return;                        // settled by rank_small_kernel
  const int n = uw.len + app;
  const int n8 = uw.n8;
  const int N = uw.budget;
  const int p_eff = min(cv.P, n);
  const int ncand = n - p_eff;
  const int e = min(n - N, ncand);
  if (n <= N || e <= 0) {
    if (tid == 0) write_selection(cv, u, sel, n, n8, n8, n, 0, -1);
    return;
  }
  const float *ema = cv.ema + (size_t)u * cv.cap;
  const int32_t *pos = cv.pos + (size_t)u * cv.cap;
  const int hm = uw.head, cap = cv.cap;              // slot i of the per-slot planes: ring_row_u(hm, i, cap)
  const int nx = cv.cap8 == 0 ? n : n8;              // slots of the ring a right shift could serve
  int32_t *src = src_all + (size_t)u * cv.cap;
  const int Ed = (n + T - 1) / T;                   // rounds in use, <= E (checked by the host)

  // candidate EMA / position of the owned slots, min / max of the EMA
  const double *shared = kShared ? shared_all + (size_t)(u / cv.Hkv) * cv.cap : nullptr;
  Imp av[E];
  int pv[E];
  // slots are position-sorted: first and last candidate position (requested with the rest)
  const int pos_first = pos[hm], pos_last = pos[ring_row_u(hm, ncand - 1, cap)];
  Imp fmin_ = INFINITY, fmax_ = -INFINITY;
  // branch-free loads (indices past the candidates re-read the last one and are masked where
  // the values are used), so that all loads of the unit are in flight before the first wait
#pragma unroll
  for (int k = 0; k < E; ++k) {
    const int slot = min(tid + k * T, ncand - 1);
    const int row = ring_row_u(hm, slot, cap);
    if constexpr (kShared) av[k] = shared[slot];
    else av[k] = ema[row];
    pv[k] = pos[row];
  }
#pragma unroll
  for (int k = 0; k < E; ++k) {
    if (k < Ed && tid + k * T < ncand) {              // (no NaN in an importance: plain compares)
      fmin_ = av[k] < fmin_ ? av[k] : fmin_;
      fmax_ = av[k] > fmax_ ? av[k] : fmax_;
    }
  }
  fmin_ = wave_min(fmin_);
  fmax_ = wave_max(fmax_);
  if (lane == 0) { s_fmin[w] = fmin_; s_fmax[w] = fmax_; }
  if (tid == 0) { s_prefix = 0ull; s_krem = e; s_done = 0; }
  __syncthreads();
  Imp lo_f = s_fmin[0], hi_f = s_fmax[0];
#pragma unroll
  for (int k = 1; k < kRsWaves; ++k) {
    lo_f = s_fmin[k] < lo_f ? s_fmin[k] : lo_f;
    hi_f = s_fmax[k] > hi_f ? s_fmax[k] : hi_f;
  }
  const double a_lo = (double)lo_f, a_hi = (double)hi_f;
  const double p_lo = (double)pos_first, p_hi = (double)pos_last;
  const double a_rng = __dsub_rn(a_hi, a_lo), p_rng = __dsub_rn(p_hi, p_lo);
  const double oma = __dsub_rn(1.0, alpha);
  const Divisor a_div = make_divisor(a_rng == 0.0 ? 1.0 : a_rng), p_div = make_divisor(p_rng == 0.0 ? 1.0 : p_rng);
  unsigned long long key[E];
  unsigned long long kmin = ~0ull, kmax = 0ull;
#pragma unroll
  for (int k = 0; k < E; ++k) {
    const int i = tid + k * T;
    key[k] = 0ull;
    if (k < Ed && i < ncand) {
      const double ah = (a_rng == 0.0) ? 0.0 : quotient(__dsub_rn((double)av[k], a_lo), a_div);
      const double rh = (p_rng == 0.0) ? 0.0 : quotient(__dsub_rn((double)pv[k], p_lo), p_div);
      key[k] = (unsigned long long)__double_as_longlong(__dadd_rn(__dmul_rn(alpha, ah), __dmul_rn(oma, rh)));
      if constexpr (kRandom) key[k] = random_key(rr, random_unit_key(cv, rr, u), pv[k]);
      kmin = key[k] < kmin ? key[k] : kmin;
      kmax = key[k] > kmax ? key[k] : kmax;
    }
  }
  // Keys are taken relative to the smallest candidate key, and the select starts at the top
  // bit in which the candidates differ: the scores live in [0, 1], so the leading sign and
  // exponent bits are the same for almost all of them and would put every candidate into one
  // histogram bin (LDS atomics on one address serialise).
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const unsigned long long a2 = __shfl_xor(kmin, m, kWave), b2 = __shfl_xor(kmax, m, kWave);
    kmin = a2 < kmin ? a2 : kmin;
    kmax = b2 > kmax ? b2 : kmax;
  }
  if (lane == 0) { s_kmin[w] = kmin; s_kmax[w] = kmax; }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kRsWaves; ++k) {
    kmin = s_kmin[k] < kmin ? s_kmin[k] : kmin;
    kmax = s_kmax[k] > kmax ? s_kmax[k] : kmax;
  }
#pragma unroll
  for (int k = 0; k < E; ++k) key[k] -= kmin;          // order-preserving
  const unsigned long long span = kmax - kmin;
  const int top = span ? 63 - __clzll((long long)span) : 0;   // highest differing bit

  // radix select of the e-th smallest key.  The first pass takes 11 bits (or what there is): with
  // a few thousand candidates its bin then holds a handful of keys and the second pass usually
  // ends the search, where 8-bit passes need three.  Every thread scans its share of the 2048
  // bins (contiguous, so that one prefix sum over the workgroup orders them).
  unsigned long long mask = 0ull;
  for (int bin = tid; bin < 512; bin += T) hist[bin] = 0;
  if constexpr (kWide0)
    for (int bin = tid; bin < kRadix0Bins; bin += T) hist0[bin] = 0;
  __syncthreads();
  int hi_bit = top + 1;
  if constexpr (kWide0) {
    const int shift = hi_bit > kRadix0Bits ? hi_bit - kRadix0Bits : 0;
    const unsigned dmask = (1u << (hi_bit - shift)) - 1u;
#pragma unroll
    for (int k = 0; k < E; ++k) {
      if (k < Ed && tid + k * T < ncand) {
        // (lanes that share the first active lane's bin add once: see below)
        const int bin = (int)((unsigned)(key[k] >> shift) & dmask);
        const int b0 = __builtin_amdgcn_readfirstlane(bin);
        const unsigned long long same = __builtin_amdgcn_ballot_w64(bin == b0);
        if (bin != b0) atomicAdd(&hist0[bin], 1);
        else if (lanes_below(same) == 0) atomicAdd(&hist0[b0], __builtin_popcountll(same));
      }
    }
    __syncthreads();
    constexpr int BPT = kRadix0Bins / T;              // bins per thread
    int cnt[BPT], mine = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      cnt[j] = hist0[BPT * tid + j];
      mine += cnt[j];
    }
    int total;
    int before = block_scan_excl<kRsWaves>(mine, s_tmp, &total);
    const int krem = e;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      if (before < krem && krem <= before + cnt[j]) {     // exactly one bin holds the cut-off
        s_prefix = (unsigned long long)(BPT * tid + j) << shift;
        s_krem = krem - before;
        s_done = (krem - before == cnt[j]);               // the whole bucket goes
      }
      before += cnt[j];
    }
    mask = ~0ull << shift;
    hi_bit = shift;
    __syncthreads();
  }
  // the following passes: 8 bits (or what is left) each.  Two barriers
  // per pass: the histogram of the next pass (the other of two buffers) is cleared while this
  // one is filled, and the first wavefront alone scans the 256 bins (four per lane) and picks
  // the bin that holds the cut-off.
  int pass = 0;
  for (; hi_bit > 0 && !s_done; ++pass) {
    const int shift = hi_bit > 8 ? hi_bit - 8 : 0;
    const unsigned dmask = (1u << (hi_bit - shift)) - 1u;
    int *hcur = hist + 256 * (pass & 1), *hnext = hist + 256 * ((pass + 1) & 1);
    const unsigned long long prefix = s_prefix;
    for (int bin = tid; bin < 256; bin += T) hnext[bin] = 0;
#pragma unroll
    for (int k = 0; k < E; ++k) {
      if (k < Ed && tid + k * T < ncand && (key[k] & mask) == prefix) {
        // scores in (0, 1] share their leading exponent bits, so in the first pass most lanes of
        // a wavefront hit one bin: the lanes that share the first active lane's bin add once
        const int bin = (int)((unsigned)(key[k] >> shift) & dmask);
        const int b0 = __builtin_amdgcn_readfirstlane(bin);
        const unsigned long long same = __builtin_amdgcn_ballot_w64(bin == b0);
        if (bin != b0) atomicAdd(&hcur[bin], 1);
        else if (lanes_below(same) == 0) atomicAdd(&hcur[b0], __builtin_popcountll(same));
      }
    }
    __syncthreads();
    if (tid < kWave) {
      int cnt[4], mine = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        cnt[j] = hcur[4 * tid + j];
        mine += cnt[j];
      }
      int before = wave_scan_incl(mine) - mine;
      const int krem = s_krem;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (before < krem && krem <= before + cnt[j]) {   // exactly one bin holds the cut-off
          s_prefix = prefix | ((unsigned long long)(4 * tid + j) << shift);
          s_krem = krem - before;
          s_done = (krem - before == cnt[j]);             // the whole bucket goes
        }
        before += cnt[j];
      }
    }
    mask = ~0ull << shift;
    hi_bit = shift;
    __syncthreads();
    if (s_done) break;
  }
  const unsigned long long prefix = s_prefix;
  const int krem = s_krem;
  const bool whole = s_done != 0;                   // uniform over the workgroup

  // Only part of the cut-off bucket goes: rank the tied slots in slot order (oldest first).
  // tie_rank(round k, lane) = base(k, wavefront) + rank inside the round's ballot.
  if (!whole) {
#pragma unroll
    for (int k = 0; k < E; ++k) {
      if (k < Ed) {
        const bool tie = tid + k * T < ncand && (key[k] & mask) == prefix;
        const unsigned long long bm = __builtin_amdgcn_ballot_w64(tie);
        if (lane == 0) s_cnt[k * kRsWaves + w] = __builtin_popcountll(bm);
      }
    }
    __syncthreads();
    for (int base = 0; base < Ed * kRsWaves; base += T) {       // in-place exclusive scan
      const int idx = base + tid;
      const int v = idx < Ed * kRsWaves ? s_cnt[idx] : 0;
      int tot;
      const int ex = block_scan_excl<kRsWaves>(v, s_tmp, &tot);
      __syncthreads();
      if (idx < Ed * kRsWaves) s_cnt[idx] = ex;                 // one chunk when Ed * waves <= T
    }
    __syncthreads();
  }
  // eviction flags as a bit per round, and in the same walk the survivors per (round,
  // wavefront), the INT8 survivors, the first hole and the last hole of the shiftable ring
  unsigned long long evbits = 0ull;                 // E <= 64
  int kept8 = 0, hole = n, last8 = -1;
#pragma unroll
  for (int k = 0; k < E; ++k) {
    if (k < Ed) {
      const int i = tid + k * T;
      bool ev = false;
      bool tie = false;
      if (i < ncand) {
        const unsigned long long km = key[k] & mask;
        ev = km < prefix;
        tie = km == prefix;
      }
      if (whole) {
        ev |= tie;
      } else {
        const unsigned long long bm = __builtin_amdgcn_ballot_w64(tie);
        if (tie) ev = s_cnt[k * kRsWaves + w] + lanes_below(bm) < krem;
      }
      if (ev) evbits |= 1ull << k;
      const bool keep = i < n && !ev;
      const unsigned long long kb = __builtin_amdgcn_ballot_w64(keep);
      if (lane == 0) s_keep[k * kRsWaves + w] = __builtin_popcountll(kb);
      kept8 += keep && i < n8;
      if (ev) {
        hole = min(hole, i);
        if (i < nx) last8 = max(last8, i);
      }
    }
  }
  kept8 = wave_sum(kept8);
  hole = wave_min(hole);
  last8 = wave_max(last8);
  if (lane == 0) { s_k8[w] = kept8; s_hole[w] = hole; s_last8[w] = last8; }
  __syncthreads();
  int k8 = 0, hl = n, l8 = -1;
#pragma unroll
  for (int k = 0; k < kRsWaves; ++k) { k8 += s_k8[k]; hl = min(hl, s_hole[k]); l8 = max(l8, s_last8[k]); }
  int tot_keep = 0;
  {
    // Ed * waves <= T for every instantiation's limits: one scan
    const int v = tid < Ed * kRsWaves ? s_keep[tid] : 0;
    const int ex = block_scan_excl<kRsWaves>(v, s_tmp, &tot_keep);
    __syncthreads();
    if (tid < Ed * kRsWaves) s_keep[tid] = ex;
    if (tid == 0) s_keep[Ed * kRsWaves] = tot_keep;
  }
  __syncthreads();
  // the compaction only looks up the source of the slots that move
  const ShiftPlan sp = shift_plan(cv, tot_keep /* = n - e */, n8, k8, hl, e, l8);
#pragma unroll
  for (int k = 0; k < E; ++k) {
    if (k < Ed) {
      // new slots [first, next) come from this wavefront's lanes of round k; most rounds lie
      // wholly outside the moving range and are skipped
      const int first = s_keep[k * kRsWaves + w], next = s_keep[k * kRsWaves + w + 1];
      if (first < sp.hi && next > sp.lo) {
        const int i = tid + k * T;
        const bool keep = i < n && !((evbits >> k) & 1ull);
        const unsigned long long bm = __builtin_amdgcn_ballot_w64(keep);
        const int j = first + lanes_below(bm);
        if (keep && j >= sp.lo && j < sp.hi) src[j] = i;
      }
    }
  }
  if (tid == 0) {
    write_selection(cv, u, sel, tot_keep, n8, k8, hl, e, l8);
    cv.unit_evicted[u] += (unsigned)e;
  }
}

// ---------------------------------------------------------------------------------------
// rank_small: grid (U / 4), one wavefront per unit.  Runs first and settles every unit that
// evicts nothing or at most kSmallE slots -- the steady state of a decode loop, where a unit
// is one token over its budget: the e lowest (score, slot) pairs are found by e passes of a
// running lexicographic minimum, with no histogram, no survivor ranking and a handful of
// registers, so many wavefronts fit a SIMD.  Same score arithmetic, same decisions as the
// general kernels, which then skip the settled units (sel[7] = 1) and handle the rest.
// ---------------------------------------------------------------------------------------
constexpr int kSmallE = 4;

// kShared: the importance is the float64 sum over the kv-heads of the (layer, sequence), which
// shared_mass_kernel left in shared_all (indexed by slot, not by ring row).
// kBatch: loads a lane has in flight at a time (8 keeps the registers few enough for thousands of
// units per launch; 32 covers a 2048-slot unit in one round trip per pass when there are few units).
template <bool kShared, int kBatch = 8, bool kRandom = false>
__global__ __launch_bounds__(kEvThreads) void rank_small_kernel(CacheView cv, LayerMask appended,
                                                                double alpha,
                                                                const double *__restrict__ shared_all,
                                                                int32_t *__restrict__ src_all,
                                                                int32_t *__restrict__ sel_all, int U,
                                                                int idle_only, RandomRank rr) {
  const int lane = threadIdx.x & 63;
  const int u = blockIdx.x * (kEvThreads / kWave) + (threadIdx.x >> 6);
  if (u >= U) return;
  asm volatile("" ::"s"(cv.len), "s"(cv.n8), "s"(cv.head8), "s"(cv.budget), "s"(cv.ema), "s"(cv.pos), "s"(cv.B),
               "s"(cv.Hkv), "s"(cv.P), "s"(cv.cap), "s"(cv.cap8), "s"(sel_all), "s"(src_all));
  const int UPL = cv.B * cv.Hkv;
  const int layer = u / UPL, b = (u % UPL) / cv.Hkv;
  int32_t *sel = sel_all + (size_t)u * kSelInts;
  const int app = appended.get(layer);
  const UnitWords uw = load_unit_words(cv, sel, u, layer, b);   // (its "settled" word is not used here)
  const int n = uw.len + app;
  const int n8 = uw.n8;
  const int N = uw.budget;
  const int p_eff = min(cv.P, n);
  const int ncand = n - p_eff;
  const int e = min(n - N, ncand);
  if (n <= N || e <= 0) {
    if (lane == 0) write_selection(cv, u, sel, n, n8, n8, n, 0, -1);
    return;
  }
  // (idle_only: whole pages are the general kernel's; this one then only settles the units that
  // evict nothing, most of them in a decode loop)
  if (e > kSmallE || idle_only) {
    if (lane == 0) sel[7] = 0;                       // left to the general kernel
    return;
  }
  const float *ema = cv.ema + (size_t)u * cv.cap;
  const int32_t *pos = cv.pos + (size_t)u * cv.cap;
  const double *shared = kShared ? shared_all + (size_t)(u / cv.Hkv) * cv.cap : nullptr;
  const int hm = uw.head, cap = cv.cap;                // slot i of the per-slot planes: ring_row_u(hm, i, cap)
  const int nx = cv.cap8 == 0 ? n : n8;              // slots of the ring a right shift could serve
  // loads go out in batches of kBatch (indices past the end re-read the last candidate), so a
  // long unit costs a few memory round trips per pass and not one per 64 slots
  typedef typename std::conditional<kShared, double, float>::type Imp;   // importance as stored
  Imp fmin_ = INFINITY, fmax_ = -INFINITY;
  for (int base = 0; base < ncand; base += kBatch * kWave) {
    Imp a[kBatch];
#pragma unroll
    for (int r = 0; r < kBatch; ++r) {
      const int i = min(base + r * kWave + lane, ncand - 1);
      if constexpr (kShared) a[r] = shared[i];
      else a[r] = ema[ring_row_u(hm, i, cap)];
    }
#pragma unroll
    for (int r = 0; r < kBatch; ++r) {
      fmin_ = a[r] < fmin_ ? a[r] : fmin_;             // (no NaN in an importance: plain compares)
      fmax_ = a[r] > fmax_ ? a[r] : fmax_;
    }
  }
  const double a_lo = (double)wave_min(fmin_), a_hi = (double)wave_max(fmax_);
  // slots are position-sorted
  const double p_lo = (double)pos[hm], p_hi = (double)pos[ring_row_u(hm, ncand - 1, cap)];
  const double a_rng = __dsub_rn(a_hi, a_lo), p_rng = __dsub_rn(p_hi, p_lo);
  const double oma = __dsub_rn(1.0, alpha);
  const Divisor a_div = make_divisor(a_rng == 0.0 ? 1.0 : a_rng), p_div = make_divisor(p_rng == 0.0 ? 1.0 : p_rng);

  int ev[kSmallE];
  unsigned long long prev_key = 0ull;
  int prev_idx = -1;                                 // every (key, slot) pair is above (0, -1)
#pragma unroll
  for (int p = 0; p < kSmallE; ++p) {
    ev[p] = 0x7fffffff;
    if (p < e) {                                     // uniform over the wavefront
      unsigned long long best_key = ~0ull;
      int best_idx = 0x7fffffff;
      for (int base = 0; base < ncand; base += kBatch * kWave) {
        Imp a[kBatch];
        int ps[kBatch];
#pragma unroll
        for (int r = 0; r < kBatch; ++r) {
          const int slot = min(base + r * kWave + lane, ncand - 1);
          const int i = ring_row_u(hm, slot, cap);
          if constexpr (kShared) a[r] = shared[slot];
          else a[r] = ema[i];
          ps[r] = pos[i];
        }
#pragma unroll
        for (int r = 0; r < kBatch; ++r) {
          const int i = base + r * kWave + lane;
          const double ah = (a_rng == 0.0) ? 0.0 : quotient(__dsub_rn((double)a[r], a_lo), a_div);
          const double rh = (p_rng == 0.0) ? 0.0 : quotient(__dsub_rn((double)ps[r], p_lo), p_div);
          const unsigned long long key =
              kRandom ? random_key(rr, random_unit_key(cv, rr, u), ps[r])
                      : (unsigned long long)__double_as_longlong(__dadd_rn(__dmul_rn(alpha, ah), __dmul_rn(oma, rh)));
          const bool above = key > prev_key || (key == prev_key && i > prev_idx);
          if (i < ncand && above && key < best_key) {  // slots rise within a lane: first one wins a tie
            best_key = key;
            best_idx = i;
          }
        }
      }
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) {
        const unsigned long long ok = __shfl_xor(best_key, m, kWave);
        const int oi = __shfl_xor(best_idx, m, kWave);
        if (ok < best_key || (ok == best_key && oi < best_idx)) {
          best_key = ok;
          best_idx = oi;
        }
      }
      ev[p] = best_idx;
      prev_key = best_key;
      prev_idx = best_idx;
    }
  }
  // evicted slots in slot order
#pragma unroll
  for (int x = 1; x < kSmallE; ++x)
#pragma unroll
    for (int y = x; y > 0; --y)
      if (ev[y] < ev[y - 1]) { const int t = ev[y]; ev[y] = ev[y - 1]; ev[y - 1] = t; }
  const int n_new = n - e;
  int gone8 = 0, last8 = -1;
#pragma unroll
  for (int q = 0; q < kSmallE; ++q) {
    if (ev[q] < n8) ++gone8;
    if (ev[q] < nx) last8 = ev[q];                   // unused entries are INT_MAX
  }
  // the compaction only looks up the source of the slots that move
  const ShiftPlan sp = shift_plan(cv, n_new, n8, n8 - gone8, ev[0], e, last8);
  int32_t *src = src_all + (size_t)u * cv.cap;
  for (int j = sp.lo + lane; j < sp.hi; j += kWave) {
    int sidx = j;
#pragma unroll
    for (int q = 0; q < kSmallE; ++q) sidx += (ev[q] <= sidx);   // unused entries are INT_MAX
    src[j] = sidx;
  }
  if (lane == 0) {
    write_selection(cv, u, sel, n_new, n8, n8 - gone8, ev[0], e, last8);
    cv.unit_evicted[u] += (unsigned)e;
  }
}

// ---------------------------------------------------------------------------------------
// compact: grid (U, 2) or (U, 5), 256 threads.  Survivor j (new slot number) comes from old slot
// src[j] >= j.  Left shift (heads stay): a workgroup walks its plane front to back in chunks
// (load a chunk into registers, barrier, store); earlier chunks only wrote below the chunk
// start and later sources all lie at or above it, so nothing is overwritten before it is
// read.  Right shift (the head of the slot-anchored rings advances by the evictions e):
// survivor j moves from ring offset src[j] to offset e + j >= src[j], only the survivors in
// front of the last hole move, and the walk goes back to front; the mirror argument holds.
// Paired form, grid (U, 2), for thousands of units: workgroup 0 of a unit moves the K and V
// rows of the ring the holes lie in, together (one look-up of the sources serves both);
// workgroup 1 moves scales, EMA and position, and then, in a mixed cache, the FP16 rows in the
// rare case that an FP16 slot was evicted.  Most units move a handful of rows there, so the
// kernel's time is workgroups times round trips.  With fewer units every plane gets a workgroup
// of its own, grid (U, 5): 0 = K INT8 rows, 1 = V INT8 rows, 2 = scales + EMA + position,
// 3 = K FP16 rows, 4 = V FP16 rows.
// ---------------------------------------------------------------------------------------

// The rows of one plane, or of two with the same row size and ring (K and V; base2 = null:
// one), ROWB bytes each:
// destination slots [lo, hi) in walk order `right`.  srow(s) gives the ring row of old slot s,
// drow(j) that of new slot j.  Loads are grouped (source slots of all passes, then all rows of
// both planes), so a chunk costs two memory round trips; lanes past the range issue nothing.
template <int ROWB, typename SrcRow, typename DstRow>
__device__ __forceinline__ void move_rows(uint8_t *base_ptr, uint8_t *base2, const int32_t *__restrict__ src,
                                          int lo, int hi, bool right, SrcRow srow, DstRow drow) {
  constexpr int LPR = ROWB / 16, RPP = kEvThreads / LPR, PASSES = 4;
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const int cnt = hi - lo;
  for (int done = 0; done < cnt; done += RPP * PASSES) {
    // four passes written out with scalar variables: as arrays the rows took a detour
    // through scratch memory
    const int k0 = done + r0, k1 = k0 + RPP, k2 = k1 + RPP, k3 = k2 + RPP;   // k-th slots of the walk
    int f0 = 0, f1 = 0, f2 = 0, f3 = 0;
    int4 b0, b1, b2, b3, c0, c1, c2, c3;
    if (k0 < cnt) f0 = src[right ? hi - 1 - k0 : lo + k0];
    if (k1 < cnt) f1 = src[right ? hi - 1 - k1 : lo + k1];
    if (k2 < cnt) f2 = src[right ? hi - 1 - k2 : lo + k2];
    if (k3 < cnt) f3 = src[right ? hi - 1 - k3 : lo + k3];
    if (k0 < cnt) b0 = *(const int4 *)(base_ptr + (size_t)srow(f0) * ROWB + c * 16);
    if (k1 < cnt) b1 = *(const int4 *)(base_ptr + (size_t)srow(f1) * ROWB + c * 16);
    if (k2 < cnt) b2 = *(const int4 *)(base_ptr + (size_t)srow(f2) * ROWB + c * 16);
    if (k3 < cnt) b3 = *(const int4 *)(base_ptr + (size_t)srow(f3) * ROWB + c * 16);
    if (base2 && k0 < cnt) c0 = *(const int4 *)(base2 + (size_t)srow(f0) * ROWB + c * 16);
    if (base2 && k1 < cnt) c1 = *(const int4 *)(base2 + (size_t)srow(f1) * ROWB + c * 16);
    if (base2 && k2 < cnt) c2 = *(const int4 *)(base2 + (size_t)srow(f2) * ROWB + c * 16);
    if (base2 && k3 < cnt) c3 = *(const int4 *)(base2 + (size_t)srow(f3) * ROWB + c * 16);
    __syncthreads();
    if (k0 < cnt) *(int4 *)(base_ptr + (size_t)drow(right ? hi - 1 - k0 : lo + k0) * ROWB + c * 16) = b0;
    if (k1 < cnt) *(int4 *)(base_ptr + (size_t)drow(right ? hi - 1 - k1 : lo + k1) * ROWB + c * 16) = b1;
    if (k2 < cnt) *(int4 *)(base_ptr + (size_t)drow(right ? hi - 1 - k2 : lo + k2) * ROWB + c * 16) = b2;
    if (k3 < cnt) *(int4 *)(base_ptr + (size_t)drow(right ? hi - 1 - k3 : lo + k3) * ROWB + c * 16) = b3;
    if (base2 && k0 < cnt) *(int4 *)(base2 + (size_t)drow(right ? hi - 1 - k0 : lo + k0) * ROWB + c * 16) = c0;
    if (base2 && k1 < cnt) *(int4 *)(base2 + (size_t)drow(right ? hi - 1 - k1 : lo + k1) * ROWB + c * 16) = c1;
    if (base2 && k2 < cnt) *(int4 *)(base2 + (size_t)drow(right ? hi - 1 - k2 : lo + k2) * ROWB + c * 16) = c2;
    if (base2 && k3 < cnt) *(int4 *)(base2 + (size_t)drow(right ? hi - 1 - k3 : lo + k3) * ROWB + c * 16) = c3;
  }
}

// Before the tags of the exchange words start over (the commit of the call before asked for it;
// the flag does not change while this kernel runs), every workgroup clears its share of them.
__device__ __forceinline__ void clear_tagged_if_asked(const CacheView &cv) {
  if (__builtin_amdgcn_readfirstlane(cv.ctl[kCtlClear]) == 0u) return;
  const size_t nwg = (size_t)gridDim.x * gridDim.y, wg = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
  for (size_t i = wg * blockDim.x + threadIdx.x; i < cv.n_tagged; i += nwg * blockDim.x) cv.tagged[i] = 0ull;
}

// kSmall: with the one-pass path for units that move a few slots (below).  The host picks the
// instance without it for the step that follows a prompt load, where every unit moves hundreds of
// rows and the extra path only costs the chunked walk registers and schedule.
template <int D, bool kSmall>
__global__ __launch_bounds__(kEvThreads) void compact_kernel(CacheView cv,
                                                             const int32_t *__restrict__ src_all,
                                                             const int32_t *__restrict__ sel_all, int paired) {
  const int u = blockIdx.x, tid = threadIdx.x;
  clear_tagged_if_asked(cv);
  // what this workgroup moves: the payload rows of the ring the holes lie in (K, V or both),
  // the per-slot planes, the FP16 rows of a mixed cache (K, V or both)
  const int y = blockIdx.y;
  const bool do_k = paired ? y == 0 : (y == 0 || y == 3), do_v = paired ? y == 0 : (y == 1 || y == 4);
  const bool do_meta = paired ? y == 1 : y == 2;
  const bool late16 = paired ? y == 1 : y >= 3;     // FP16 rows of a mixed cache
  const bool main_rows = paired ? y == 0 : y <= 1;
  const int32_t *sel = sel_all + (size_t)u * kSelInts;
  const int n_new = sel[0], n8_new = sel[1], hole = sel[2], evicted = sel[3];
  if (hole >= n_new) return;                          // nothing moves
  const int n8_old = cv.n8[u], h16 = cv.head16[u], h0 = cv.head8[u];
  const int32_t *src = src_all + (size_t)u * cv.cap;
  const int cap = cv.cap, cap8 = cv.cap8, cap16 = cv.cap16;
  const bool fp16_only = cap8 == 0;
  const bool right = sel[5] != 0;
  const int e8 = n8_old - n8_new;
  const int jr = sel[4] + 1 - (fp16_only ? evicted : e8);   // right shift: survivors [0, jr) move
  const int h0_new = sel[6];

  // A mixed cache that moves a few slots and no FP16 row -- a unit of a decode loop in its steady
  // state -- is served by the unit's first workgroup alone, in one pass: the sources of all
  // planes are looked up together, then all rows are requested together, so the unit costs two
  // memory round trips however many planes it has; its other workgroups leave at once.
  if (kSmall && !fp16_only && evicted == e8) {
    constexpr int LPR = D / 16, RPP = kEvThreads / LPR;
    const int lo = right ? 0 : hole, hi_m = right ? jr : n_new, hi_8 = right ? jr : n8_new;
    const int cnt_m = hi_m - lo, cnt_8 = max(0, hi_8 - lo);
    if (cnt_m <= kEvThreads && cnt_8 <= RPP * 4) {
      if (y != 0) return;
      uint8_t *pk = (uint8_t *)(cv.k8 + (size_t)u * cap8 * D), *pv = (uint8_t *)(cv.v8 + (size_t)u * cap8 * D);
      float *ema = cv.ema + (size_t)u * cap;
      int32_t *pos = cv.pos + (size_t)u * cap;
      unsigned short *ks = (unsigned short *)(cv.ks + (size_t)u * cap8), *vs = (unsigned short *)(cv.vs + (size_t)u * cap8);
      const int c = tid % LPR, r0 = tid / LPR;
      // (four passes written out with scalar variables: see move_rows)
      const int k0 = r0, k1 = k0 + RPP, k2 = k1 + RPP, k3 = k2 + RPP;
      const int j0 = right ? hi_8 - 1 - k0 : lo + k0, j1 = right ? hi_8 - 1 - k1 : lo + k1;
      const int j2 = right ? hi_8 - 1 - k2 : lo + k2, j3 = right ? hi_8 - 1 - k3 : lo + k3;
      const int jm = right ? hi_m - 1 - tid : lo + tid;
      int f0 = 0, f1 = 0, f2 = 0, f3 = 0, fm = 0;
      if (k0 < cnt_8) f0 = src[j0];
      if (k1 < cnt_8) f1 = src[j1];
      if (k2 < cnt_8) f2 = src[j2];
      if (k3 < cnt_8) f3 = src[j3];
      if (tid < cnt_m) fm = ring_row(h0, src[jm], cap);
      int4 b0, b1, b2, b3, c0, c1, c2, c3;
      float fa = 0.f;
      int32_t fp = 0;
      unsigned short fk = 0, fv = 0;
      if (k0 < cnt_8) { b0 = *(const int4 *)(pk + (size_t)ring_row(h0, f0, cap8) * D + c * 16); c0 = *(const int4 *)(pv + (size_t)ring_row(h0, f0, cap8) * D + c * 16); }
      if (k1 < cnt_8) { b1 = *(const int4 *)(pk + (size_t)ring_row(h0, f1, cap8) * D + c * 16); c1 = *(const int4 *)(pv + (size_t)ring_row(h0, f1, cap8) * D + c * 16); }
      if (k2 < cnt_8) { b2 = *(const int4 *)(pk + (size_t)ring_row(h0, f2, cap8) * D + c * 16); c2 = *(const int4 *)(pv + (size_t)ring_row(h0, f2, cap8) * D + c * 16); }
      if (k3 < cnt_8) { b3 = *(const int4 *)(pk + (size_t)ring_row(h0, f3, cap8) * D + c * 16); c3 = *(const int4 *)(pv + (size_t)ring_row(h0, f3, cap8) * D + c * 16); }
      if (tid < cnt_m) {
        fa = ema[fm];
        fp = pos[fm];
        if (!cv.chan && jm < n8_new) { fk = ks[fm]; fv = vs[fm]; }
      }
      __syncthreads();
      if (k0 < cnt_8) { *(int4 *)(pk + (size_t)ring_row(h0_new, j0, cap8) * D + c * 16) = b0; *(int4 *)(pv + (size_t)ring_row(h0_new, j0, cap8) * D + c * 16) = c0; }
      if (k1 < cnt_8) { *(int4 *)(pk + (size_t)ring_row(h0_new, j1, cap8) * D + c * 16) = b1; *(int4 *)(pv + (size_t)ring_row(h0_new, j1, cap8) * D + c * 16) = c1; }
      if (k2 < cnt_8) { *(int4 *)(pk + (size_t)ring_row(h0_new, j2, cap8) * D + c * 16) = b2; *(int4 *)(pv + (size_t)ring_row(h0_new, j2, cap8) * D + c * 16) = c2; }
      if (k3 < cnt_8) { *(int4 *)(pk + (size_t)ring_row(h0_new, j3, cap8) * D + c * 16) = b3; *(int4 *)(pv + (size_t)ring_row(h0_new, j3, cap8) * D + c * 16) = c3; }
      if (tid < cnt_m) {
        const int d = ring_row(h0_new, jm, cap);
        ema[d] = fa;
        pos[d] = fp;
        if (!cv.chan && jm < n8_new) { ks[d] = fk; vs[d] = fv; }
      }
      return;
    }
  }

  // FP16 ring rows.  Mixed cache: they only move (left) when an FP16 slot was evicted.
  // FP16-only cache: either side.
  auto move_fp16_rows = [&](bool k, bool v) {
    const int h16_new = (fp16_only && right) ? ring_row(h16, evicted, cap16) : h16;
    uint8_t *pk = (uint8_t *)(cv.k16 + (size_t)u * cap16 * D), *pv = (uint8_t *)(cv.v16 + (size_t)u * cap16 * D);
    move_rows<2 * D>(k ? pk : pv, (k && v) ? pv : nullptr, src,
                     right ? 0 : max(hole, n8_new), right ? jr : n_new, right,
                     [&](int s) { return ring_row(h16, s - n8_old, cap16); },
                     [&](int j) { return ring_row(h16_new, j - n8_new, cap16); });
  };
  if (fp16_only) {
    // the FP16 ring is the ring the holes lie in: its rows are the main rows (planes 3 and 4
    // of the unpaired form)
    if (paired ? y == 0 : y >= 3) move_fp16_rows(paired || y == 3, paired || y == 4);
  } else if (main_rows) {
    uint8_t *pk = (uint8_t *)(cv.k8 + (size_t)u * cap8 * D), *pv = (uint8_t *)(cv.v8 + (size_t)u * cap8 * D);
    move_rows<D>(do_k ? pk : pv, (do_k && do_v) ? pv : nullptr, src,
                 right ? 0 : hole, right ? jr : n8_new, right,
                 [&](int s) { return ring_row(h0, s, cap8); },
                 [&](int j) { return ring_row(h0_new, j, cap8); });
  }
  if (do_meta) {
    // per-slot planes: EMA and position for every moving slot, scales for the INT8 ones
    // (same ring offsets: cap8 = cap in a mixed cache)
    float *ema = cv.ema + (size_t)u * cap;
    int32_t *pos = cv.pos + (size_t)u * cap;
    __half *ks = cv.ks + (size_t)u * cap8, *vs = cv.vs + (size_t)u * cap8;
    const int lo = right ? 0 : hole, hi = right ? jr : n_new;
    constexpr int PASSES = 4;
    const int cnt = hi - lo;
    for (int done = 0; done < cnt; done += kEvThreads * PASSES) {
      int from[PASSES];
      float fa[PASSES];
      int32_t fp[PASSES];
      unsigned short fk[PASSES], fv[PASSES];
      // grouped loads (see move_rows)
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int k = done + p * kEvThreads + tid;
        if (k < cnt) from[p] = ring_row(h0, src[right ? hi - 1 - k : lo + k], cap);
      }
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int k = done + p * kEvThreads + tid;
        if (k < cnt) {
          fa[p] = ema[from[p]];
          fp[p] = pos[from[p]];
          if (!cv.chan && (right ? hi - 1 - k : lo + k) < n8_new) {
            fk[p] = ((const unsigned short *)ks)[from[p]];
            fv[p] = ((const unsigned short *)vs)[from[p]];
          }
        }
      }
      __syncthreads();
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int k = done + p * kEvThreads + tid;
        const int j = right ? hi - 1 - k : lo + k;
        if (k < cnt) {
          const int d = ring_row(h0_new, j, cap);
          ema[d] = fa[p];
          pos[d] = fp[p];
          if (!cv.chan && j < n8_new) {
            ((unsigned short *)ks)[d] = fk[p];
            ((unsigned short *)vs)[d] = fv[p];
          }
        }
      }
    }
  }
  if (!fp16_only && late16 && evicted != e8) move_fp16_rows(paired || y == 3, paired || y == 4);
}

// ---------------------------------------------------------------------------------------
// Paged layout: the compaction is an edit of the unit's block table ("Compatibility with
// serving systems": evicting whole blocks frees them without a gather).  Grid (U / 4), one
// wavefront per unit, 2 * npages ints of LDS per wavefront.  Under the layout's rules only
// whole INT8 pages leave, so new page q is the old page that held the source slot of new slot
// q * page; the pages that left follow the live ones (in their old order), the free ones
// keep their places behind them.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kEvThreads) void compact_paged_kernel(CacheView cv, const int32_t *__restrict__ src_all,
                                                                   const int32_t *__restrict__ sel_all, int U) {
  extern __shared__ int32_t pg_lds[];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int u = blockIdx.x * (kEvThreads / kWave) + w;
  clear_tagged_if_asked(cv);
  if (u >= U) return;
  const int32_t *sel = sel_all + (size_t)u * kSelInts;
  if (sel[3] == 0) return;                                   // nothing left the unit
  const int lg = cv.page_lg, g = 1 << lg;
  const int live_old = (cv.n8[u] + g - 1) >> lg, live_new = (sel[1] + g - 1) >> lg;
  if (live_old == live_new) return;
  int32_t *tab = cv.pt + (size_t)u * cv.npages;
  const int32_t *src = src_all + (size_t)u * cv.cap;
  int32_t *old = pg_lds + (size_t)w * 2 * cv.npages, *used = old + cv.npages;
  for (int p = lane; p < live_old; p += kWave) { old[p] = tab[p]; used[p] = 0; }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  for (int q = lane; q < live_new; q += kWave) {
    const int op = src[q << lg] >> lg;                       // old page of the new page's first slot
    tab[q] = old[op];
    used[op] = 1;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  int carry = live_new;
  for (int base = 0; base < live_old; base += kWave) {
    const int p = base + lane;
    const int gone = p < live_old && !used[p];
    const int rank = wave_scan_incl(gone) - gone;
    if (gone) tab[carry + rank] = old[p];
    carry += wave_sum(gone);
  }
}

// ---------------------------------------------------------------------------------------
// demote: grid (U / 4), one wavefront per unit.  Quantises the oldest FP16 slots until at most W stay
// FP16, appends them at the INT8 ring tail, and commits (len, n8, head16, head8).  The first
// wavefront also commits the step state in cv.ctl: the layers' next positions move past the
// appended tokens and the tag bases past the launches since the last commit; a base near the
// end of its range asks the next call's compaction kernel to clear the tagged words, after
// which both bases start over at 0.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kEvThreads) void demote_kernel(CacheView cv,
                                                            const int32_t *__restrict__ sel_all, int U,
                                                            LayerMask appended, unsigned attend_launches,
                                                            unsigned conf_launches) {
  if (blockIdx.x == 0 && threadIdx.x < kWave) {
    for (int l = threadIdx.x; l < cv.L; l += kWave)
      if (const int c = appended.get(l)) cv.ctl[kCtlPos + l] += (unsigned)c;
    if (threadIdx.x == 0) {
      if (cv.ctl[kCtlClear]) {
        cv.ctl[kCtlTag] = cv.ctl[kCtlConfTag] = cv.ctl[kCtlClear] = 0u;
      } else {
        const unsigned t = cv.ctl[kCtlTag] + attend_launches, c = cv.ctl[kCtlConfTag] + conf_launches;
        cv.ctl[kCtlTag] = t;
        cv.ctl[kCtlConfTag] = c;
        if (t > kTagRestart || c > kTagRestart) cv.ctl[kCtlClear] = 1u;
      }
    }
  }
  const int u = blockIdx.x * (kEvThreads / kWave) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (u >= U) return;
  const int32_t *sel = sel_all + (size_t)u * kSelInts;
  const int n_new = sel[0], n8_new = sel[1], h8 = sel[6];   // slot-anchored ring head after the compaction
  // an FP16-only cache that closed its holes from the front has advanced its FP16 ring too
  const int h16 = (cv.cap8 == 0 && sel[5]) ? ring_row(cv.head16[u], sel[3], cv.cap16) : cv.head16[u];
  const int n16 = n_new - n8_new;
  const int cnt = (cv.W < 0) ? 0 : max(0, n16 - cv.W);
  const int32_t *tab = cv.pt + (size_t)u * cv.npages;          // paged layout (already edited by the compaction)
  for (int t = 0; t < cnt; ++t) {
    const int row = ring_row(h16, t, cv.cap16);
    const int drow = cv.page_lg ? slot_row(cv, tab, 0, n8_new + t + 1, 0, n8_new + t) : ring_row(h8, n8_new + t, cv.cap8);
    const size_t dst = (size_t)u * cv.cap8 + drow;
    if (cv.page_lg && lane == 0) {
      // the slot's EMA and position move from the FP16 slots' metadata rows to its INT8 row
      const size_t from = (size_t)u * cv.cap + cv.cap - cv.cap16 + row;
      cv.ema[(size_t)u * cv.cap + drow] = cv.ema[from];
      cv.pos[(size_t)u * cv.cap + drow] = cv.pos[from];
    }
    if constexpr (D == 128) {
      if (cv.chan) {
        quantize_row_channels<D>(cv.k16 + ((size_t)u * cv.cap16 + row) * D, cv.k8 + dst * D, cv.ks + (size_t)u * D, lane);
        quantize_row_channels<D>(cv.v16 + ((size_t)u * cv.cap16 + row) * D, cv.v8 + dst * D, cv.vs + (size_t)u * D, lane);
        continue;
      }
    }
    quantize_row_wave<D>(cv.k16 + ((size_t)u * cv.cap16 + row) * D, cv.k8 + dst * D, cv.ks + dst, lane);
    quantize_row_wave<D>(cv.v16 + ((size_t)u * cv.cap16 + row) * D, cv.v8 + dst * D, cv.vs + dst, lane);
  }
  if (lane == 0) {
    cv.len[u] = n_new;
    cv.n8[u] = n8_new + cnt;
    cv.head16[u] = ring_row(h16, cnt % cv.cap16, cv.cap16);
    cv.head8[u] = h8;
    if (cnt) cv.unit_demoted[u] += (unsigned)cnt;
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------

hipError_t launch_load_prefill(const CacheView &cv, int layer, const __half *k16, const __half *v16,
                               int T0, const float *ema0, hipStream_t stream) {
  const int rw = kEvThreads / (cv.D / 8);            // tokens per workgroup of the loader
  dim3 grid(T0 > 0 ? (T0 + rw - 1) / rw : 1, cv.B * cv.Hkv);
  if (cv.chan)      // D = 128 by construction of the handle
    hipLaunchKernelGGL(channel_scales_kernel, dim3(cv.B * cv.Hkv, 2), dim3(1024), 0, stream, cv, layer, k16, v16, T0);
  if (cv.D == 64)
    hipLaunchKernelGGL(load_prefill_kernel<64>, grid, dim3(kEvThreads), 0, stream, cv, layer, k16, v16, T0, ema0);
  else
    hipLaunchKernelGGL(load_prefill_kernel<128>, grid, dim3(kEvThreads), 0, stream, cv, layer, k16, v16, T0, ema0);
  return hipGetLastError();
}

hipError_t launch_evict_compact(const CacheView &cv, const LayerMask &appended, double alpha,
                                const RankOptions &opt, double *score, int32_t *src, int32_t *sel,
                                int n_max, unsigned attend_launches, unsigned conf_launches, int after_prompt,
                                hipStream_t stream) {
  const int U = cv.L * cv.B * cv.Hkv;
  // The random ranker runs on the same kernels as the composite one (a different key per slot);
  // with the layer scope it needs no shared importance, only a key common to the kv-heads.
  RandomRank rr{};
  rr.on = opt.random;
  rr.layer_scope = opt.shared != nullptr;
  rr.seed = opt.seed;
  const bool shared_imp = opt.shared && !opt.random;          // the ranking reads the summed importance
  if (opt.page > 1) {
    // whole pages: the general kernel, behind the one-wavefront kernel that settles the units
    // that evict nothing (with pages of g slots a unit evicts once in g steps)
    if (shared_imp)
      hipLaunchKernelGGL(shared_mass_kernel, dim3(cv.L * cv.B, (cv.cap + kEvThreads - 1) / kEvThreads),
                         dim3(kEvThreads), 0, stream, cv, appended, opt.shared);
    hipLaunchKernelGGL((rank_small_kernel<false, 8>), dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, appended, alpha,
                       (const double *)nullptr, src, sel, U, 1, rr);
    if (n_max <= 256 * 20)    // (a short unit does not fill 1024 threads, and most units return at once)
      hipLaunchKernelGGL(rank_select_kernel<256>, dim3(U), dim3(256), 0, stream, cv, appended, alpha, opt,
                         1, score, src, sel);
    else
      hipLaunchKernelGGL(rank_select_kernel<1024>, dim3(U), dim3(1024), 0, stream, cv, appended, alpha, opt,
                         1, score, src, sel);
  } else if (shared_imp) {
    // layer-shared importance: the summed mass first, then the same three kernel shapes reading it
    hipLaunchKernelGGL(shared_mass_kernel, dim3(cv.L * cv.B, (cv.cap + kEvThreads - 1) / kEvThreads),
                       dim3(kEvThreads), 0, stream, cv, appended, opt.shared);
    hipLaunchKernelGGL((rank_small_kernel<true, 8>), dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, appended, alpha,
                       (const double *)opt.shared, src, sel, U, 0, rr);
    if (n_max <= 256 * 20)
      hipLaunchKernelGGL((rank_select_reg_kernel<256, 20, true>), dim3(U), dim3(256), 0, stream, cv, appended,
                         alpha, src, sel, (const double *)opt.shared, rr);
    else if (n_max <= 1024 * 33)
      hipLaunchKernelGGL((rank_select_reg_kernel<1024, 33, true>), dim3(U), dim3(1024), 0, stream, cv, appended,
                         alpha, src, sel, (const double *)opt.shared, rr);
    else
      hipLaunchKernelGGL(rank_select_kernel<1024>, dim3(U), dim3(1024), 0, stream, cv, appended, alpha, opt,
                         1, score, src, sel);
  } else if (opt.random) {
    // the random ranker: the same kernel shapes with the drawn key in place of the composite score
    if (U <= 4096)
      hipLaunchKernelGGL((rank_small_kernel<false, 32, true>), dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv,
                         appended, alpha, (const double *)nullptr, src, sel, U, 0, rr);
    else
      hipLaunchKernelGGL((rank_small_kernel<false, 8, true>), dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv,
                         appended, alpha, (const double *)nullptr, src, sel, U, 0, rr);
    if (n_max <= 64 * 33 && U >= 2048)
      hipLaunchKernelGGL((rank_select_reg_kernel<64, 33, false, true>), dim3(U), dim3(64), 0, stream, cv, appended,
                         alpha, src, sel, (const double *)nullptr, rr);
    else if (n_max <= 256 * 20)
      hipLaunchKernelGGL((rank_select_reg_kernel<256, 20, false, true>), dim3(U), dim3(256), 0, stream, cv, appended,
                         alpha, src, sel, (const double *)nullptr, rr);
    else if (n_max <= 1024 * 33)
      hipLaunchKernelGGL((rank_select_reg_kernel<1024, 33, false, true>), dim3(U), dim3(1024), 0, stream, cv, appended,
                         alpha, src, sel, (const double *)nullptr, rr);
    else
      hipLaunchKernelGGL(rank_select_kernel<1024>, dim3(U), dim3(1024), 0, stream, cv, appended, alpha, opt,
                         1, score, src, sel);
  } else {
  if (U <= 4096)    // few wavefronts per SIMD: registers to spare for deeper batches
    hipLaunchKernelGGL((rank_small_kernel<false, 32>), dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, appended,
                       alpha, (const double *)nullptr, src, sel, U, 0, rr);
  else
    hipLaunchKernelGGL((rank_small_kernel<false, 8>), dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, appended,
                       alpha, (const double *)nullptr, src, sel, U, 0, rr);
  // With thousands of short units one wavefront per unit is faster (its workgroup barriers cost
  // nothing); with few units the chip is filled by giving each unit four wavefronts.
  if (n_max <= 64 * 33 && U >= 2048)
    hipLaunchKernelGGL((rank_select_reg_kernel<64, 33>), dim3(U), dim3(64), 0, stream, cv, appended,
                       alpha, src, sel, (const double *)nullptr, rr);
  else if (n_max <= 256 * 20)
    hipLaunchKernelGGL((rank_select_reg_kernel<256, 20>), dim3(U), dim3(256), 0, stream, cv, appended,
                       alpha, src, sel, (const double *)nullptr, rr);
  else if (n_max <= 1024 * 33)
    hipLaunchKernelGGL((rank_select_reg_kernel<1024, 33>), dim3(U), dim3(1024), 0, stream, cv, appended,
                       alpha, src, sel, (const double *)nullptr, rr);
  else
    hipLaunchKernelGGL(rank_select_kernel<1024>, dim3(U), dim3(1024), 0, stream, cv, appended, alpha, opt,
                       1, score, src, sel);
  }
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  // measured: with 8192 units the paired form saves 6 us per step, with 2048 and fewer the
  // workgroup per plane is 3 to 4 us faster
  int paired = U >= 4096;
  if (const char *e = getenv("CONF_KV_COMPACT_PAIRED")) paired = atoi(e) != 0;   // test hook: force a form
  if (cv.page_lg) {
    // paged layout: a table edit instead of row moves (the ranking above was the general kernel)
    const size_t lds = (size_t)(kEvThreads / kWave) * 2 * cv.npages * sizeof(int32_t);
    hipLaunchKernelGGL(compact_paged_kernel, dim3((U + 3) / 4), dim3(kEvThreads), lds, stream, cv, src, sel, U);
    if (cv.D == 64)
      hipLaunchKernelGGL(demote_kernel<64>, dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, sel, U, appended,
                         attend_launches, conf_launches);
    else
      hipLaunchKernelGGL(demote_kernel<128>, dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, sel, U, appended,
                         attend_launches, conf_launches);
    return hipGetLastError();
  }
  const dim3 cgrid(U, paired ? 2 : 5);
  if (cv.D == 64) {
    if (after_prompt)
      hipLaunchKernelGGL((compact_kernel<64, false>), cgrid, dim3(kEvThreads), 0, stream, cv, src, sel, paired);
    else
      hipLaunchKernelGGL((compact_kernel<64, true>), cgrid, dim3(kEvThreads), 0, stream, cv, src, sel, paired);
    hipLaunchKernelGGL(demote_kernel<64>, dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, sel, U, appended,
                       attend_launches, conf_launches);
  } else {
    if (after_prompt)
      hipLaunchKernelGGL((compact_kernel<128, false>), cgrid, dim3(kEvThreads), 0, stream, cv, src, sel, paired);
    else
      hipLaunchKernelGGL((compact_kernel<128, true>), cgrid, dim3(kEvThreads), 0, stream, cv, src, sel, paired);
    hipLaunchKernelGGL(demote_kernel<128>, dim3((U + 3) / 4), dim3(kEvThreads), 0, stream, cv, sel, U, appended,
                       attend_launches, conf_launches);
  }
  return hipGetLastError();
}

}  // namespace confkv

// Decode attention over the mixed INT8 / FP16 cache with the attention-mass EMA fused in
// (paper: "Tiled attention and mixed precision" -- blockwise read, running max and
// normaliser, dequantisation fused into the read; "Budget and ranker" -- EMA of attention
// mass; Algorithm 1 -- append in FP16, update EMA metadata).
//
// One launch per layer, grid (splits, B * Hkv), 256 threads.  The `splits` workgroups of a
// unit (b, kv-head) each stream a contiguous, byte-balanced slice of the unit's slots once
// and serve all G query heads of the group from that single read:
//
//   stream   every slot lane-group keeps a running (max, normaliser, output) per head
//            (online softmax); raw scores s[h][i] of the slice stay in LDS
//   publish  lane-groups -> wavefront -> workgroup merge; (m, l, o) -> global, arrive; the
//            last workgroup to arrive merges the splits' partials into out
//   mass     the others wait until every split of the unit has arrived (they all publish
//            at about the same time), form the exact global (M, L), then per slot
//            A_i = sum_h e^{s[h][i]-M[h]} / L[h] and ema_i <- lambda ema_i + (1-lambda) A_i.
//
// Every K/V byte is read once; the scores never leave the chip.  The wait is between
// workgroups of one launch, so the host only launches grids that are co-resident
// (splits * units <= occupancy * CUs) and the wait itself is bounded.
//
// Lane mapping: a slot's row is D channels; lane c of a group of D/16 lanes owns channels
// [16c, 16c+16) -- one 128-bit load of an INT8 row, two of an FP16 row -- so a wavefront
// load instruction covers 64/(D/16) whole rows, contiguous in memory.
#include <algorithm>
#include <map>
#include <tuple>

#include "confkv_dev.h"
#include "launch.h"

namespace confkv {

constexpr int kAttThreads = 256;
constexpr int kAttWaves = 4;
constexpr int kSpinLimit = 4000000;

__device__ __forceinline__ void unpack_i8x16(const int4 &r, float (&f)[16]) {
  const int wds[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int e = 0; e < 4; ++e) f[4 * k + e] = (float)((wds[k] << (24 - 8 * e)) >> 24);
  }
}

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

// Partials travel between workgroups (possibly on different XCDs, whose L2s are not
// coherent for ordinary accesses) through agent-scope relaxed atomics: such loads and
// stores are coherent across the device by themselves, so no cache-wide release/acquire
// fence (an L2 write-back plus invalidate on this hardware) is ever issued.  Ordering is
// by completion: a publisher waits for its stores to complete before the workgroup
// barrier that precedes the arrival increment; a consumer only issues its loads after it
// has observed the arrival count.
__device__ __forceinline__ void st_agent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores_done() { __builtin_amdgcn_s_waitcnt(0); }

__device__ __forceinline__ void unpack_h16x16(const int4 &r0, const int4 &r1, float (&f)[16]) {
  half8_t a = __builtin_bit_cast(half8_t, r0), b = __builtin_bit_cast(half8_t, r1);
#pragma unroll
  for (int e = 0; e < 8; ++e) { f[e] = (float)a[e]; f[8 + e] = (float)b[e]; }
}

// Running softmax state of one slot lane-group: per head the maximum so far, the
// normaliser and this lane's 16 channels of the un-normalised output.
template <int G>
struct Stream {
  float m[G], l[G], acc[G][16];
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
__global__ __launch_bounds__(kAttThreads) void attend_kernel(CacheView cv, AttendLaunch a, int ns,
                                                             int S) {
  constexpr int LPT = D / 16;            // lanes per slot row
  constexpr int TW = kWave / LPT;        // slots per wavefront pass
  constexpr int TB = kAttWaves * TW;     // slots per workgroup pass
  constexpr int R8 = 4, R16 = 2;         // slots per lane-group per loop trip (INT8 / FP16)
  extern __shared__ float smem[];
  float *stash = smem;                          // [G][S] raw scores of the slice
  float *wo = stash + (size_t)G * S;            // [4][G][D] per-wave un-normalised output
  float *wm = wo + kAttWaves * G * D;           // [4][G] per-wave maximum
  float *wl = wm + kAttWaves * G;               // [4][G] per-wave normaliser
  float *gm = wl + kAttWaves * G;               // [G] global maximum (mass phase)
  double *ginv = (double *)(gm + G + (G & 1));  // [G] 1 / global normaliser
  __shared__ int s_ok;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane % LPT, ts = lane / LPT;
  const int ul = blockIdx.y, j = blockIdx.x;
  const int UPL = cv.B * cv.Hkv;
  const int u = a.layer * UPL + ul;
  const int b = ul / cv.Hkv, g = ul % cv.Hkv;
  const int cap = cv.cap, cap8 = cv.cap8, cap16 = cv.cap16;
  const int n8 = cv.n8[u];
  const int n = cv.len[u] + 1;           // the appended token included
  const int h16 = cv.head16[u];
  const int n16 = n - n8;
  const float NEG = -INFINITY;

  // byte-balanced split: an FP16 slot weighs two INT8 slots
  const long long nv = (long long)n8 + 2ll * n16;
  const long long vlo = nv * j / ns, vhi = nv * (j + 1) / ns;
  // (rounding down keeps the tail slice non-empty, so its owner always holds slot n-1)
  int lo = vlo <= n8 ? (int)vlo : n8 + (int)((vlo - n8) >> 1);
  int hi = vhi <= n8 ? (int)vhi : n8 + (int)((vhi - n8) >> 1);
  if (hi - lo > S) {                     // cannot happen when the host plan is right
    if (tid == 0) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
    hi = lo + S;
  }
  const int ntok = hi - lo;

  const int8_t *K8 = cv.k8 + (size_t)u * cap8 * D;
  const int8_t *V8 = cv.v8 + (size_t)u * cap8 * D;
  const __half *KS = cv.ks + (size_t)u * cap8;
  const __half *VS = cv.vs + (size_t)u * cap8;
  __half *K16 = cv.k16 + (size_t)u * cap16 * D;
  __half *V16 = cv.v16 + (size_t)u * cap16 * D;
  float *EMA = cv.ema + (size_t)u * cap;

  // ---- append: the workgroup that owns the tail writes the new token into the ring ----
  if (j == ns - 1) {
    const int row = ring_row(h16, n16 - 1, cap16);
    if (tid < D / 8) {
      const int4 *src = (const int4 *)(a.knew + (size_t)ul * D);
      ((int4 *)(K16 + (size_t)row * D))[tid] = src[tid];
    } else if (tid < D / 4) {
      const int t = tid - D / 8;
      const int4 *src = (const int4 *)(a.vnew + (size_t)ul * D);
      ((int4 *)(V16 + (size_t)row * D))[t] = src[t];
    }
    if (tid == 0) cv.pos[(size_t)u * cap + n - 1] = a.pos_new;
    __syncthreads();
  }

  const int hi8 = min(hi, n8), lo16 = max(lo, n8);
  const float sm = a.sm_scale;

  // ================= one streaming pass over the slice =================
  Stream<G> st;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    st.m[h] = NEG;
    st.l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) st.acc[h][e] = 0.f;
  }
  float qf[G][16];
  {
    const int Hq = cv.Hkv * G;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const int4 *qp = (const int4 *)(a.q + ((size_t)(b * Hq + g * G + h)) * D + c * 16);
      unpack_h16x16(qp[0], qp[1], qf[h]);
    }
  }
  // INT8 slots
  for (int base = lo; base < hi8; base += TB * R8) {
    int4 kr[R8], vr[R8];
    float ksc[R8], vsc[R8];
    bool ok[R8];
#pragma unroll
    for (int r = 0; r < R8; ++r) {
      const int i = base + r * TB + w * TW + ts;
      ok[r] = i < hi8;
      kr[r] = vr[r] = make_int4(0, 0, 0, 0);
      ksc[r] = vsc[r] = 0.f;
      if (ok[r]) {
        kr[r] = *(const int4 *)(K8 + (size_t)i * D + c * 16);
        vr[r] = *(const int4 *)(V8 + (size_t)i * D + c * 16);
        ksc[r] = __half2float(KS[i]);
        vsc[r] = __half2float(VS[i]);
      }
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
      const float f = ksc[r] * sm;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        s[r][h] *= f;
        if (ok[r] && c == 0) stash[h * S + (i - lo)] = s[r][h];
      }
      unpack_i8x16(vr[r], vf[r]);
    }
    fold_batch<G, R8>(st, s, vf, vsc, ok);
  }
  // FP16 slots (ring)
  for (int base = lo16; base < hi; base += TB * R16) {
    int4 kr[R16][2], vr[R16][2];
    float vsc[R16];
    bool ok[R16];
#pragma unroll
    for (int r = 0; r < R16; ++r) {
      const int i = base + r * TB + w * TW + ts;
      ok[r] = i < hi;
      vsc[r] = 1.f;
      kr[r][0] = kr[r][1] = vr[r][0] = vr[r][1] = make_int4(0, 0, 0, 0);
      if (ok[r]) {
        const size_t off = (size_t)ring_row(h16, i - n8, cap16) * D + c * 16;
        const int4 *pk = (const int4 *)(K16 + off), *pv = (const int4 *)(V16 + off);
        kr[r][0] = pk[0]; kr[r][1] = pk[1];
        vr[r][0] = pv[0]; vr[r][1] = pv[1];
      }
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
        if (ok[r] && c == 0) stash[h * S + (i - lo)] = s[r][h];
      }
      unpack_h16x16(vr[r][0], vr[r][1], vf[r]);
    }
    fold_batch<G, R16>(st, s, vf, vsc, ok);
  }

  // ---- merge the slot lane-groups of the wavefront, then the four wavefronts ----
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
    if (lane == 0) { wm[w * G + h] = mw; wl[w * G + h] = l; }
    if (ts == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) wo[(w * G + h) * D + c * 16 + e] = st.acc[h][e];
    }
  }
  __syncthreads();
  float *ml = a.part_ml + ((size_t)ul * a.max_splits + j) * G * 2;
  float *po = a.part_o + ((size_t)ul * a.max_splits + j) * G * D;
  for (int idx = tid; idx < G * D; idx += kAttThreads) {
    const int h = idx / D;
    const float M = fmaxf(fmaxf(wm[h], wm[G + h]), fmaxf(wm[2 * G + h], wm[3 * G + h]));
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int k = 0; k < kAttWaves; ++k) {
      const float mk = wm[k * G + h];
      const float f = (mk == NEG) ? 0.f : __expf(mk - M);
      o = fmaf(wo[k * G * D + idx], f, o);
      l = fmaf(wl[k * G + h], f, l);
    }
    st_agent(&po[idx], o);
    if (idx % D == 0) {
      st_agent(&ml[h * 2 + 0], M);
      st_agent(&ml[h * 2 + 1], l);
    }
  }
  wait_stores_done();
  __syncthreads();
  if (tid == 0) {
    __hip_atomic_fetch_add(&a.arrive[ul], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int ok = 1;
    if (ns > 1) {
      // bounded wait until all splits of the unit have published
      const unsigned want = a.arrive_base + (unsigned)ns;
      int spins = 0;
      while ((int)(__hip_atomic_load(&a.arrive[ul], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) -
                   want) < 0) {
        __builtin_amdgcn_s_sleep(2);
        if (++spins > kSpinLimit) { ok = 0; break; }
      }
      if (!ok) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
    }
    s_ok = ok;
  }
  __syncthreads();
  if (!s_ok) return;

  // ---- all (m, l) partials of the unit -> LDS in one round trip; global (M, 1/L) ----
  const float *mlu = a.part_ml + (size_t)ul * a.max_splits * G * 2;
  float *pml = wo;                                   // [ns][G][2], reuses the merge buffer
  for (int idx = tid; idx < ns * G * 2; idx += kAttThreads) pml[idx] = ld_agent(&mlu[idx]);
  __syncthreads();
  if (tid < G) {
    float M = NEG;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, pml[(s * G + tid) * 2]);
    double L = 0.0;
    for (int s = 0; s < ns; ++s) {
      const float ms = pml[(s * G + tid) * 2];
      if (ms > NEG) L += exp((double)ms - (double)M) * (double)pml[(s * G + tid) * 2 + 1];
    }
    gm[tid] = M;
    ginv[tid] = 1.0 / L;
  }
  __syncthreads();

  // ---- mass + EMA of the slice (EMA reads go out first, the output merge overlaps them) ----
  const double lam = (double)a.ema_decay, oml = 1.0 - lam;
  for (int t = tid; t < ntok; t += kAttThreads) {
    const int slot = lo + t;
    const double old = (slot == n - 1) ? 0.0 : (double)EMA[slot];
    double A = 0.0;
#pragma unroll
    for (int h = 0; h < G; ++h) A += (double)expf(stash[h * S + t] - gm[h]) * ginv[h];
    EMA[slot] = (float)(lam * old + oml * A);
  }

  // ---- this split normalises its share of the unit's output (online-softmax merge) ----
  {
    const float *pou = a.part_o + (size_t)ul * a.max_splits * G * D;
    const int Hq = cv.Hkv * G;
    const int per = (G * D + ns - 1) / ns;
    const int i1 = min(G * D, (j + 1) * per);
    for (int idx = j * per + tid; idx < i1; idx += kAttThreads) {
      const int h = idx / D;
      const float M = gm[h];
      float o = 0.f;
      for (int s0 = 0; s0 < ns; s0 += 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
          v[k] = (s0 + k < ns) ? ld_agent(&pou[(size_t)(s0 + k) * G * D + idx]) : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          if (s0 + k < ns) {
            const float ms = pml[((s0 + k) * G + h) * 2];
            if (ms > NEG) o = fmaf(v[k], expf(ms - M), o);
          }
        }
      }
      a.out[((size_t)(b * Hq + g * G)) * D + idx] = __float2half_rn((float)((double)o * ginv[h]));
    }
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------

typedef void (*AttendFn)(CacheView, AttendLaunch, int, int);

static AttendFn attend_fn(int D, int G) {
#define CONFKV_CASE(d, g) \
  if (D == d && G == g) return attend_kernel<d, g>;
  CONFKV_CASE(64, 1) CONFKV_CASE(64, 2) CONFKV_CASE(64, 4) CONFKV_CASE(64, 5) CONFKV_CASE(64, 8)
  CONFKV_CASE(128, 1) CONFKV_CASE(128, 2) CONFKV_CASE(128, 4) CONFKV_CASE(128, 5) CONFKV_CASE(128, 8)
#undef CONFKV_CASE
  return nullptr;
}

bool attend_supported(int D, int G) { return attend_fn(D, G) != nullptr; }

static size_t attend_lds_bytes(int D, int G, int S) {
  size_t floats = (size_t)G * S + (size_t)kAttWaves * G * D + 2 * kAttWaves * G + G + 2;
  return floats * sizeof(float) + (size_t)G * sizeof(double) + 16;
}

struct DeviceLimits {
  int cus = 0;
  size_t max_lds = 0;
  bool ok = false;
};

static const DeviceLimits &device_limits() {
  static DeviceLimits lim;
  if (!lim.ok) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
      lim.cus = prop.multiProcessorCount;
      lim.max_lds = prop.sharedMemPerBlockOptin ? prop.sharedMemPerBlockOptin
                                                : prop.sharedMemPerBlock;
      if (lim.max_lds > 160 * 1024) lim.max_lds = 160 * 1024;
      lim.ok = lim.cus > 0;
    }
  }
  return lim;
}

// Resident workgroups per CU of attend_kernel<D,G> with `lds` bytes of dynamic LDS.
static int attend_occupancy(int D, int G, size_t lds) {
  static std::map<std::tuple<int, int, size_t>, int> cache;
  auto key = std::make_tuple(D, G, lds);
  auto it = cache.find(key);
  if (it != cache.end()) return it->second;
  AttendFn fn = attend_fn(D, G);
  int nb = 0;
  if (lds > 64 * 1024)
    (void)hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void *)fn, kAttThreads, lds) !=
      hipSuccess)
    nb = 0;
  cache[key] = nb;
  return nb;
}

bool attend_plan(int D, int G, int units_per_layer, int n_ub, int n16_ub, int forced_splits,
                 AttendPlan *plan) {
  const DeviceLimits &lim = device_limits();
  if (!lim.ok || !attend_fn(D, G)) return false;
  const long long nv = (long long)n_ub + n16_ub;
  // aim for about three workgroups per CU, but keep at least 128 virtual slots per split
  int want = forced_splits > 0 ? forced_splits : (3 * lim.cus + units_per_layer - 1) / units_per_layer;
  want = std::min<long long>(want, std::max<long long>(1, nv / 128));
  want = std::max(1, std::min(want, kAttendMaxSplits));
  // preference order: want, want-1, .., 1 (fewer, always co-resident), then want+1, .. (more
  // splits shrink the LDS stash when a long unit does not fit otherwise)
  for (int k = 0; k < kAttendMaxSplits; ++k) {
    const int ns = k < want ? want - k : k + 1;
    // LDS is sized in steps of 256 slots so the occupancy query is cached across calls
    int S = (int)((nv + ns - 1) / ns) + 2;
    S = (S + 255) / 256 * 256;
    size_t lds = attend_lds_bytes(D, G, S);
    if (lds > lim.max_lds) continue;
    if (ns > 1) {
      int occ = attend_occupancy(D, G, lds);
      if ((long long)occ * lim.cus < (long long)ns * units_per_layer) continue;
    } else if (lds > 64 * 1024) {
      (void)attend_occupancy(D, G, lds);        // raises the dynamic-LDS limit
    }
    plan->splits = ns;
    plan->stash_tokens = S;
    plan->lds_bytes = lds;
    return true;
  }
  return false;
}

hipError_t launch_attend(const CacheView &cv, const AttendLaunch &a, const AttendPlan &plan,
                         hipStream_t stream) {
  AttendFn fn = attend_fn(cv.D, cv.G);
  if (!fn) return hipErrorInvalidValue;
  dim3 grid(plan.splits, cv.B * cv.Hkv);
  hipLaunchKernelGGL(fn, grid, dim3(kAttThreads), plan.lds_bytes, stream, cv, a, plan.splits,
                     plan.stash_tokens);
  return hipGetLastError();
}

}  // namespace confkv

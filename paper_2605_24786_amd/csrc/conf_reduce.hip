// Confidence estimator and budget selector (paper: Method, Eq. 1 and the budget rule of
// "Budget and ranker"; Algorithm 1, lines softmax / c / N).
//
// One launch: grid (chunks, B).  A workgroup reduces one 4096-logit chunk of one sequence
// to (max, sum e^{x-max}, sum (x-max) e^{x-max}, top-1, top-2) with the chunk held in
// registers and publishes it as words tagged with the call's epoch; the workgroup of the
// sequence's last chunk waits (bounded) until every chunk's words carry that tag, merges the
// chunk partials in float64, evaluates Eq. 1 and writes c, the tight/loose flag and the
// per-layer budgets.  Nobody does a read-modify-write: a ticket counter per sequence made the
// 32 arrivals of a row queue up at one address.  HBM traffic is one read of the logits
// (4 B per logit).
#include <mutex>

#include "confkv_dev.h"
#include "launch.h"

namespace confkv {

constexpr int kConfThreads = 256;
constexpr int kConfPerThread = 16;
constexpr int kConfChunk = kConfThreads * kConfPerThread;   // 4096 logits per workgroup
constexpr int kPartialStride = 8;                           // 8-byte words per chunk partial (5 in use)

// A float with the epoch of the call that wrote it in one 8-byte word: value and tag are seen
// together or not at all.  Agent-scope relaxed atomics are coherent across the XCDs by
// themselves, so no cache-wide fence is needed.
__device__ __forceinline__ void st_tagged(unsigned long long *p, unsigned epoch, float v) {
  __hip_atomic_store(p, ((unsigned long long)epoch << 32) | (unsigned long long)__float_as_uint(v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_word(const unsigned long long *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_coherent(const unsigned long long *p) {   // the value half
  return __uint_as_float((unsigned)ld_word(p));
}

__device__ __forceinline__ void top2_merge(float &a1, float &a2, float b1, float b2) {
  // two largest of the multiset {a1, a2, b1, b2} given a1 >= a2 and b1 >= b2
  float lo = fminf(a1, b1);
  a1 = fmaxf(a1, b1);
  a2 = fmaxf(lo, fmaxf(a2, b2));
}

__global__ __launch_bounds__(kConfThreads) void conf_reduce_kernel(
    const float *__restrict__ logits, int V, int nchunk, unsigned long long *__restrict__ partial,
    unsigned launch_no, int device_base, int spin_limit, int withhold, float *__restrict__ conf,
    uint8_t *__restrict__ sel, CacheView cv, double tau, double wH, double wm, double wp) {
  // the words' tag: the launch's number plus, for the handle's own words, the base the commit
  // at the end of conf_kv_evict_compact advances (so that a recorded launch can be replayed)
  // (requested now, added where the partial is published: the logits loads go out first)
  const unsigned tag_base = device_base ? cv.ctl[kCtlConfTag] : 0u;
  __shared__ float s_f[4 * 4];
  __shared__ double s_d[4 * 2];
  __shared__ int s_ok;
  const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const float *row = logits + (size_t)b * V;
  const float NEG = -INFINITY;

  float x[kConfPerThread];
  if ((V & 3) == 0) {
    // rows start on 16-byte boundaries: four 128-bit loads per thread, all in flight together
    // (a quad past the row re-reads its last quad and is masked afterwards)
    const int q0 = c * (kConfChunk / 4) + tid, nq = V / 4;
    float4 v[kConfPerThread / 4];
#pragma unroll
    for (int r = 0; r < kConfPerThread / 4; ++r) v[r] = ((const float4 *)row)[min(q0 + r * kConfThreads, nq - 1)];
#pragma unroll
    for (int r = 0; r < kConfPerThread / 4; ++r) {
      const bool in = q0 + r * kConfThreads < nq;
      x[4 * r] = in ? v[r].x : NEG;
      x[4 * r + 1] = in ? v[r].y : NEG;
      x[4 * r + 2] = in ? v[r].z : NEG;
      x[4 * r + 3] = in ? v[r].w : NEG;
    }
  } else {
    const int base = c * kConfChunk + tid;
    // branch-free loads (an index past the row re-reads its last logit and is masked afterwards),
    // so that all sixteen are in flight before the first one is waited for
#pragma unroll
    for (int r = 0; r < kConfPerThread; ++r) x[r] = row[min(base + r * kConfThreads, V - 1)];
#pragma unroll
    for (int r = 0; r < kConfPerThread; ++r) x[r] = base + r * kConfThreads < V ? x[r] : NEG;
  }
  float v1 = NEG, v2 = NEG;
#pragma unroll
  for (int r = 0; r < kConfPerThread; ++r) {
    float t = x[r];
    if (t > v1) { v2 = v1; v1 = t; } else if (t > v2) { v2 = t; }
  }
  // workgroup top-2 (v1 is also the chunk maximum)
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    float o1 = __shfl_xor(v1, m, kWave), o2 = __shfl_xor(v2, m, kWave);
    top2_merge(v1, v2, o1, o2);
  }
  if (lane == 0) { s_f[w] = v1; s_f[4 + w] = v2; }
  __syncthreads();
  v1 = s_f[0]; v2 = s_f[4];
#pragma unroll
  for (int k = 1; k < 4; ++k) top2_merge(v1, v2, s_f[k], s_f[4 + k]);
  const float mx = v1;

  float S = 0.f, T = 0.f;
  if (mx > NEG) {
#pragma unroll
    for (int r = 0; r < kConfPerThread; ++r) {
      float d = x[r] - mx;
      float e = expf(d);
      S += e;
      T += (e > 0.f) ? d * e : 0.f;     // 0 * log 0 = 0, also for -inf logits
    }
  }
  S = wave_sum(S);
  T = wave_sum(T);
  if (lane == 0) { s_f[8 + w] = S; s_f[12 + w] = T; }
  __syncthreads();
  const unsigned epoch = launch_no + tag_base;
  if (tid == 0 && withhold && c == 0) s_ok = 1;       // (test hook: chunk 0 keeps its words to itself)
  if (tid == 0 && !(withhold && c == 0)) {
    unsigned long long *p = partial + ((size_t)b * nchunk + c) * kPartialStride;
    st_tagged(&p[0], epoch, mx);
    st_tagged(&p[1], epoch, (s_f[8] + s_f[9]) + (s_f[10] + s_f[11]));
    st_tagged(&p[2], epoch, (s_f[12] + s_f[13]) + (s_f[14] + s_f[15]));
    st_tagged(&p[3], epoch, v1);
    st_tagged(&p[4], epoch, v2);
    s_ok = 1;
  }
  if (c != nchunk - 1) return;

  // ---- workgroup of the sequence's last chunk (every other chunk was dispatched before it):
  // wait for the words of all chunks, then merge the chunk partials in float64 ----
  const unsigned long long *pb = partial + (size_t)b * nchunk * kPartialStride;
  __syncthreads();                                  // s_ok is set
  for (int base = 0; base < nchunk * 5; base += kConfThreads) {
    const int i = base + tid;
    const bool mine = i < nchunk * 5;
    const unsigned long long *wp_ = pb + (size_t)(mine ? i / 5 : 0) * kPartialStride + (mine ? i % 5 : 0);
    bool here = !mine;
    int spins = 0;
    for (;;) {
      if (!here) here = (unsigned)(ld_word(wp_) >> 32) == epoch;
      if (__builtin_amdgcn_ballot_w64(!here) == 0ull) break;
      __builtin_amdgcn_s_sleep(1);
      if (++spins > spin_limit) {
        if (!here) s_ok = 0;
        break;
      }
    }
  }
  __syncthreads();
  if (!s_ok) {                                      // a chunk never arrived: no budgets are written
    if (tid == 0) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
    return;
  }
  float M = NEG, t1 = NEG, t2 = NEG;
  for (int k = tid; k < nchunk; k += kConfThreads) {
    const unsigned long long *p = pb + (size_t)k * kPartialStride;
    M = fmaxf(M, ld_coherent(&p[0]));
    top2_merge(t1, t2, ld_coherent(&p[3]), ld_coherent(&p[4]));
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    float o1 = __shfl_xor(t1, m, kWave), o2 = __shfl_xor(t2, m, kWave);
    top2_merge(t1, t2, o1, o2);
  }
  M = wave_max(M);
  __syncthreads();
  if (lane == 0) { s_f[w] = M; s_f[4 + w] = t1; s_f[8 + w] = t2; }
  __syncthreads();
  M = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
  t1 = s_f[4]; t2 = s_f[8];
#pragma unroll
  for (int k = 1; k < 4; ++k) top2_merge(t1, t2, s_f[4 + k], s_f[8 + k]);

  double Sd = 0.0, Td = 0.0;
  for (int k = tid; k < nchunk; k += kConfThreads) {
    const unsigned long long *p = pb + (size_t)k * kPartialStride;
    const float mk = ld_coherent(&p[0]), sk = ld_coherent(&p[1]), tk = ld_coherent(&p[2]);
    if (mk > NEG) {
      double shift = (double)mk - (double)M;       // <= 0
      double wgt = exp(shift);
      Sd += wgt * (double)sk;
      Td += wgt * ((double)tk + shift * (double)sk);
    }
  }
  Sd = wave_sum(Sd);
  Td = wave_sum(Td);
  if (lane == 0) { s_d[w] = Sd; s_d[4 + w] = Td; }
  __syncthreads();
  __shared__ int s_tight;
  if (tid == 0) {
    Sd = (s_d[0] + s_d[1]) + (s_d[2] + s_d[3]);
    Td = (s_d[4] + s_d[5]) + (s_d[6] + s_d[7]);
    // H = log S - T / S  with T = sum (x - M) e^{x - M};  p_(1) = 1 / S;  m = l_(1) - l_(2)
    double H = log(Sd) - Td / Sd;
    double Hhat = H / log((double)V);
    double margin = (double)t1 - (double)t2;        // +inf when the runner-up is -inf
    double sig = 1.0 / (1.0 + exp(-margin));
    double p1 = 1.0 / Sd;
    double cval = wH * (1.0 - Hhat) + wm * sig + wp * p1;
    int tight = cval >= tau;
    if (conf) conf[b] = (float)cval;
    if (sel) sel[b] = (uint8_t)tight;
    s_tight = tight;
    atomicAdd(&cv.stats[tight ? kStatTight : kStatLoose], 1ull);
  }
  __syncthreads();
  const int tight = s_tight;
  for (int l = tid; l < cv.L; l += kConfThreads)
    cv.budget[l * cv.B + b] = tight ? cv.n_tight[l] : cv.n_loose[l];
}

// ---------------------------------------------------------------------------------------
// The same reduction with the chunk partials in memory the library owns: for callers that
// cannot provide (or allocate) a workspace.  `scratch` is a host-side stand-in for the
// array: host code only ever uses the device address hipGetSymbolAddress returns for the
// current device (every device holds its own copy).  The array starts zeroed when the code
// object is loaded, and tag 0 is never used by a launch.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned long long scratch[kConfStaticBytes / 8];

namespace {
constexpr int kMaxDevices = 64;
struct StaticScratch {
  unsigned long long *ptr = nullptr;   // device address of `scratch` on this device
  unsigned epoch = 0;                  // tag of the last launch that used it
};
StaticScratch g_static[kMaxDevices];
std::mutex g_static_mutex;

// words [0, n) <- 0 (a kernel, not a memset node: the call may sit in a captured stream)
__global__ void conf_static_clear_kernel(unsigned long long *p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}
}  // namespace

hipError_t conf_reduce_static_setup() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static[dev].ptr) return hipSuccess;
  unsigned long long *ptr = nullptr;
  e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  g_static[dev].ptr = ptr;
  return hipSuccess;
}

hipError_t launch_conf_reduce_static(const CacheView &cv, const float *logits, int V, int spin_limit, int withhold,
                                     float *conf, uint8_t *sel, double tau, double wH, double wm, double wp,
                                     hipStream_t stream) {
  if (conf_reduce_scratch_bytes(cv.B, V) > kConfStaticBytes) return hipErrorInvalidValue;   // the caller checks first
  hipError_t e = conf_reduce_static_setup();
  if (e != hipSuccess) return e;
  int dev = -1;
  e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  unsigned long long *ptr;
  unsigned epoch;
  bool wrapped = false;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    ptr = g_static[dev].ptr;
    if (++g_static[dev].epoch == 0u) { g_static[dev].epoch = 1u; wrapped = true; }
    epoch = g_static[dev].epoch;
  }
  // after 2^32 launches the tags start over: no word may still carry one of the new round
  if (wrapped) (void)launch_zero_words(ptr, kConfStaticBytes, stream);
  return launch_conf_reduce(cv, logits, V, ptr, epoch, 0, spin_limit, withhold, conf, sel, tau, wH, wm, wp, stream);
}

hipError_t launch_zero_words(void *p, size_t bytes, hipStream_t stream) {
  hipLaunchKernelGGL(conf_static_clear_kernel, dim3(256), dim3(256), 0, stream, (unsigned long long *)p, bytes / 8);
  return hipGetLastError();
}

size_t conf_reduce_scratch_bytes(int B, int V) {
  int nchunk = (V + kConfChunk - 1) / kConfChunk;
  return (size_t)B * nchunk * kPartialStride * 8;
}

hipError_t launch_conf_reduce(const CacheView &cv, const float *logits, int V, unsigned long long *partial,
                              unsigned launch_no, int device_base, int spin_limit, int withhold, float *conf,
                              uint8_t *sel, double tau, double wH, double wm, double wp, hipStream_t stream) {
  int nchunk = (V + kConfChunk - 1) / kConfChunk;
  dim3 grid(nchunk, cv.B);
  hipLaunchKernelGGL(conf_reduce_kernel, grid, dim3(kConfThreads), 0, stream, logits, V, nchunk,
                     partial, launch_no, device_base, spin_limit, withhold, conf, sel, cv, tau, wH, wm, wp);
  return hipGetLastError();
}

}  // namespace confkv

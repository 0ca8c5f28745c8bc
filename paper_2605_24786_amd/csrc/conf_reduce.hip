// Confidence estimator and budget selector (paper: Method, Eq. 1 and the budget rule of
// "Budget and ranker"; Algorithm 1, lines softmax / c / N).
//
// One launch: grid (chunks, B).  A workgroup reduces one 4096-logit chunk of one sequence
// to (max, sum e^{x-max}, sum (x-max) e^{x-max}, top-1, top-2) with the chunk held in
// registers, publishes it, and the last workgroup to arrive for a sequence merges the
// chunk partials in float64, evaluates Eq. 1 and writes c, the tight/loose flag and the
// per-layer budgets.  HBM traffic is one read of the logits (4 B per logit).
#include "confkv_dev.h"
#include "launch.h"

namespace confkv {

constexpr int kConfThreads = 256;
constexpr int kConfPerThread = 16;
constexpr int kConfChunk = kConfThreads * kConfPerThread;   // 4096 logits per workgroup
constexpr int kPartialStride = 8;                           // floats per chunk partial

__device__ __forceinline__ void st_coherent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_coherent(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void top2_merge(float &a1, float &a2, float b1, float b2) {
  // two largest of the multiset {a1, a2, b1, b2} given a1 >= a2 and b1 >= b2
  float lo = fminf(a1, b1);
  a1 = fmaxf(a1, b1);
  a2 = fmaxf(lo, fmaxf(a2, b2));
}

__global__ __launch_bounds__(kConfThreads) void conf_reduce_kernel(
    const float *__restrict__ logits, int V, int nchunk, float *__restrict__ partial,
    unsigned *__restrict__ arrive, float *__restrict__ conf, uint8_t *__restrict__ sel,
    CacheView cv, double tau, double wH, double wm, double wp) {
  __shared__ float s_f[4 * 4];
  __shared__ double s_d[4 * 2];
  __shared__ int s_last;
  const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const float *row = logits + (size_t)b * V;
  const float NEG = -INFINITY;

  float x[kConfPerThread];
  const int base = c * kConfChunk + tid;
  // branch-free loads (an index past the row re-reads its last logit and is masked afterwards),
  // so that all sixteen are in flight before the first one is waited for
#pragma unroll
  for (int r = 0; r < kConfPerThread; ++r) x[r] = row[min(base + r * kConfThreads, V - 1)];
#pragma unroll
  for (int r = 0; r < kConfPerThread; ++r) x[r] = base + r * kConfThreads < V ? x[r] : NEG;
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
  if (tid == 0) {
    float *p = partial + ((size_t)b * nchunk + c) * kPartialStride;
    // agent-scope relaxed atomics are coherent across the XCDs by themselves; the stores
    // are complete before the ticket is taken, and the last arrival loads them the same
    // way, so no cache-wide fence is needed
    st_coherent(&p[0], mx);
    st_coherent(&p[1], (s_f[8] + s_f[9]) + (s_f[10] + s_f[11]));
    st_coherent(&p[2], (s_f[12] + s_f[13]) + (s_f[14] + s_f[15]));
    st_coherent(&p[3], v1);
    st_coherent(&p[4], v2);
    __builtin_amdgcn_s_waitcnt(0);
    unsigned ticket = __hip_atomic_fetch_add(&arrive[b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (ticket == (unsigned)(nchunk - 1));
  }
  __syncthreads();
  if (!s_last) return;

  // ---- last workgroup of this sequence: merge the chunk partials in float64 ----
  const float *pb = partial + (size_t)b * nchunk * kPartialStride;
  float M = NEG, t1 = NEG, t2 = NEG;
  for (int k = tid; k < nchunk; k += kConfThreads) {
    const float *p = pb + (size_t)k * kPartialStride;
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
    const float *p = pb + (size_t)k * kPartialStride;
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
    __hip_atomic_store(&arrive[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
  }
  __syncthreads();
  const int tight = s_tight;
  for (int l = tid; l < cv.L; l += kConfThreads)
    cv.budget[l * cv.B + b] = tight ? cv.n_tight[l] : cv.n_loose[l];
}

size_t conf_reduce_scratch_floats(int B, int V) {
  int nchunk = (V + kConfChunk - 1) / kConfChunk;
  return (size_t)B * nchunk * kPartialStride;
}

hipError_t launch_conf_reduce(const CacheView &cv, const float *logits, int V, float *partial,
                              unsigned *arrive, float *conf, uint8_t *sel, double tau, double wH,
                              double wm, double wp, hipStream_t stream) {
  int nchunk = (V + kConfChunk - 1) / kConfChunk;
  dim3 grid(nchunk, cv.B);
  hipLaunchKernelGGL(conf_reduce_kernel, grid, dim3(kConfThreads), 0, stream, logits, V, nchunk,
                     partial, arrive, conf, sel, cv, tau, wH, wm, wp);
  return hipGetLastError();
}

}  // namespace confkv

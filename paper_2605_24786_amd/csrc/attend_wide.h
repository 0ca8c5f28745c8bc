// Decode attention for calls that carry more query rows per kv-head than one matrix-core tile
// holds (conf_kv_attend_chunk / conf_kv_observe with tq * G > 16: chunks of a prompt, draft
// tokens under verification; paper: "Compatibility with serving systems").  Included by
// attend.hip, inside namespace confkv, after the helpers of the single-tile kernels.
//
// The call is DEFINED as tq single-token steps (see conf_kv_attend_chunk).  Rows r = token * G +
// head are cut into RB blocks of 16; a workgroup of eight wavefronts is RB row blocks times
// NS = 8 / RB tile streams.  The slice's K/V tiles (32 INT8 slots or 16 FP16 slots each) are
// brought into LDS eight at a time, one per wavefront -- every K/V byte is read from memory
// once per pass whatever the number of rows, and INT8 keys become fp16 once, when the tile is
// stored -- and each wavefront then runs ITS row block
// against the tiles of its stream: scores by matrix core, online softmax per row, P V by matrix
// core.  No score is stashed (R x slots floats would not fit anywhere): after the splits have
// exchanged their (m, l, o) per row, a second pass streams the keys again, recomputes the same
// scores (same instructions, hence the same bits), turns them into exact probabilities with
// the global (M, L), sums each slot's column over the rows (weights lambda^(tq-1-token)) and
// updates the EMA.  Key bytes are therefore read twice, value bytes once.
#pragma once

// A tile in LDS: K as fp16 rows (the codes of an INT8 tile are converted once, by the wavefront
// that stores the tile, not once per row block that reads it), V transposed as stored (its
// conversion is three instructions per four codes and stays with the reader), the reading
// wavefront's probability tile, and per slot the score factor and the value scale.
constexpr int kWideKBytes = kTile * kKRow16;
constexpr int kWideCoreBytes = kWideKBytes + kVBytes + 16 * kPRow * 2;
constexpr int kWideScaleBytes = 2 * kTile * 4;
constexpr int kWideTileBytes = kWideCoreBytes + kWideScaleBytes;
constexpr int kWideMaxRows = 128;
constexpr int kWideMaxSplits = 8;

__host__ __device__ constexpr size_t attend_wide_lds_bytes(int R, int ns) {
  return (size_t)kAttWaves * kWideTileBytes + ((size_t)3 * R + (size_t)kAttWaves * (R / 16) * kTile + (size_t)ns * R * 2) * 4 + 16;
}

template <int RB>
__global__ __launch_bounds__(kAttThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attend_wide_kernel(const int32_t *, const int32_t *, const int32_t *, const int32_t *, int , int , int , CacheView cv, AttendLaunch a_in, int ns, int /*unused*/) {
  const AttendLaunch a = resolve_launch(cv, a_in);
  constexpr int D = 128, NS = kAttWaves / RB, R = RB * 16;
  constexpr int kPartFloats = 16 * D + 32;                   // a wavefront's (o, m, l) for the stream merge
  static_assert((NS - 1) * RB * kPartFloats * 4 <= kAttWaves * kWideTileBytes, "stream merge fits the tile buffers");
  extern __shared__ __align__(16) float smem[];
  uint8_t *tiles = (uint8_t *)smem;
  float *Mrow = (float *)(tiles + kAttWaves * kWideTileBytes);   // [R] global maximum of a row
  float *Irow = Mrow + R;                                        // [R] 1 / global normaliser
  float *Frow = Irow + R;                                        // [R] the same times the row's mass weight
  float *mass = Frow + R;                                        // [8 tiles][RB][32] column sums per tile and row block
  float *pml = mass + kAttWaves * RB * kTile;                    // [ns][R][2] gathered statistics
  __shared__ int s_ok;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int rb = w % RB, st = w / RB;
  const int tq = a.tq, gq = a.gq;
  const float NEG = -INFINITY;
  const float sm = a.sm_scale;
  const int t16 = lane & 15, g4 = lane >> 4;
  const int c8 = lane & 7, r8 = lane >> 3;
  const int c16 = lane & 15, r4 = lane >> 4;
  const Slice sl = make_slice(cv, a, ns, 0x7fffffff);

  // rows of this wavefront in the accumulator layout: element i of a lane is row 4 * g4 + i of the block
  int rowc[4], seen[4];
  bool okc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    rowc[i] = rb * 16 + 4 * g4 + i;
    const int tok = rowc[i] / gq;
    okc[i] = tok < tq;
    seen[i] = sl.n - tq + tok + 1;               // the row of token t sees slots below n - tq + t + 1
  }

  const int8_t *K8 = cv.k8 + (size_t)sl.u * cv.cap8 * D;
  const int8_t *V8 = cv.v8 + (size_t)sl.u * cv.cap8 * D;
  const __half *KS = cv.ks + (size_t)sl.u * cv.cap8;
  const __half *VS = cv.vs + (size_t)sl.u * cv.cap8;
  const __half *K16 = cv.k16 + (size_t)sl.u * cv.cap16 * D;
  const __half *V16 = cv.v16 + (size_t)sl.u * cv.cap16 * D;
  const int ntiles = (sl.cnt8 + kTile - 1) / kTile;
  const int ntiles16 = (sl.hi16 - sl.lo16 + 15) / 16;
  const int nitems = ntiles + ntiles16;
  const int nsup = (nitems + kAttWaves - 1) / kAttWaves;

  struct TileRegs {
    int4 k0, k1, k2, k3, v0, v1, v2, v3;
    unsigned short ks0, ks1, vs0, vs1;
  };
  // branch-free loads (rows past the slice re-read its last row and are masked where they are used)
  auto load_item = [&](int it, bool with_v) -> TileRegs {
    TileRegs t = {};
    if (it < ntiles) {
      const int base = sl.lo8 + it * kTile, last = sl.hi8 - 1;
      const unsigned col = (unsigned)c8 * 16u;
      const int h8 = sl.h8, cap8 = cv.cap8;
      const unsigned o0 = (unsigned)ring_row_u(h8, min(base + r8, last), cap8) * D + col;
      const unsigned o1 = (unsigned)ring_row_u(h8, min(base + 8 + r8, last), cap8) * D + col;
      const unsigned o2 = (unsigned)ring_row_u(h8, min(base + 16 + r8, last), cap8) * D + col;
      const unsigned o3 = (unsigned)ring_row_u(h8, min(base + 24 + r8, last), cap8) * D + col;
      t.k0 = ld_stream16(K8 + o0);
      t.k1 = ld_stream16(K8 + o1);
      t.k2 = ld_stream16(K8 + o2);
      t.k3 = ld_stream16(K8 + o3);
      if (with_v) {
        t.v0 = ld_stream16(V8 + o0);
        t.v1 = ld_stream16(V8 + o1);
        t.v2 = ld_stream16(V8 + o2);
        t.v3 = ld_stream16(V8 + o3);
      }
      const unsigned j0 = (unsigned)ring_row_u(h8, min(base + t16, last), cap8);
      const unsigned j1 = (unsigned)ring_row_u(h8, min(base + 16 + t16, last), cap8);
      t.ks0 = ((const unsigned short *)KS)[j0];
      t.ks1 = ((const unsigned short *)KS)[j1];
      if (with_v) {
        t.vs0 = ((const unsigned short *)VS)[j0];
        t.vs1 = ((const unsigned short *)VS)[j1];
      }
    } else {
      const int base = sl.lo16 + 16 * (it - ntiles), last = sl.hi16 - 1;
      const int h16 = sl.h16, cap16 = cv.cap16, n8 = sl.n8;
      const unsigned col = (unsigned)c16 * 8u;
      // the call's own tokens come from the call's arguments, not from the ring
      const int first_new = a.observe_first >= 0 ? 0x3fffffff : sl.n - tq;
      const size_t tok = (size_t)cv.Hkv * D;
      const __half *kn = a.knew + ((size_t)sl.b * tq * cv.Hkv + sl.g) * D + col;
      const __half *vn = a.vnew + ((size_t)sl.b * tq * cv.Hkv + sl.g) * D + col;
      const int s0 = min(base + r4, last), s1 = min(base + 4 + r4, last);
      const int s2 = min(base + 8 + r4, last), s3 = min(base + 12 + r4, last);
      const unsigned o0 = (unsigned)ring_row(h16, s0 - n8, cap16) * D + col, o1 = (unsigned)ring_row(h16, s1 - n8, cap16) * D + col;
      const unsigned o2 = (unsigned)ring_row(h16, s2 - n8, cap16) * D + col, o3 = (unsigned)ring_row(h16, s3 - n8, cap16) * D + col;
      const int n0 = s0 - first_new, n1 = s1 - first_new, n2 = s2 - first_new, n3 = s3 - first_new;
      t.k0 = ld_stream16(n0 >= 0 ? kn + n0 * tok : K16 + o0);
      t.k1 = ld_stream16(n1 >= 0 ? kn + n1 * tok : K16 + o1);
      t.k2 = ld_stream16(n2 >= 0 ? kn + n2 * tok : K16 + o2);
      t.k3 = ld_stream16(n3 >= 0 ? kn + n3 * tok : K16 + o3);
      if (with_v) {
        t.v0 = ld_stream16(n0 >= 0 ? vn + n0 * tok : V16 + o0);
        t.v1 = ld_stream16(n1 >= 0 ? vn + n1 * tok : V16 + o1);
        t.v2 = ld_stream16(n2 >= 0 ? vn + n2 * tok : V16 + o2);
        t.v3 = ld_stream16(n3 >= 0 ? vn + n3 * tok : V16 + o3);
      }
    }
    return t;
  };
  // registers -> this wavefront's LDS buffer: K rows as they are, V transposed to [channel][slot],
  // and per slot the factor of the raw score (key scale times softmax scale) and the value scale
  auto store_item = [&](int it, const TileRegs &tr, bool with_v) {
    uint8_t *Kt = tiles + (size_t)w * kWideTileBytes;
    uint8_t *Vt = Kt + kWideKBytes;
    float *sc = (float *)(Kt + kWideCoreBytes);
    if (it < ntiles) {
      // sixteen codes of a row per lane -> sixteen fp16 values (exact)
      auto put_k = [&](int row, const int4 &k) {
        half8_t *dst = (half8_t *)(Kt + row * kKRow16 + c8 * 32);
        dst[0] = cvt_i8x8_f16x8((unsigned)k.x, (unsigned)k.y);
        dst[1] = cvt_i8x8_f16x8((unsigned)k.z, (unsigned)k.w);
      };
      put_k(r8, tr.k0);
      put_k(8 + r8, tr.k1);
      put_k(16 + r8, tr.k2);
      put_k(24 + r8, tr.k3);
      if (with_v) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const unsigned x0 = dword_of(tr.v0, q4), x1 = dword_of(tr.v1, q4);
          const unsigned x2 = dword_of(tr.v2, q4), x3 = dword_of(tr.v3, q4);
          const unsigned t0 = __builtin_amdgcn_perm(x1, x0, 0x05010400u), t1 = __builtin_amdgcn_perm(x1, x0, 0x07030602u);
          const unsigned t2 = __builtin_amdgcn_perm(x3, x2, 0x05010400u), t3 = __builtin_amdgcn_perm(x3, x2, 0x07030602u);
          const unsigned o0 = __builtin_amdgcn_perm(t2, t0, 0x05040100u), o1 = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
          const unsigned o2 = __builtin_amdgcn_perm(t3, t1, 0x05040100u), o3 = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
          uint8_t *dst = Vt + (16 * c8 + 4 * q4) * kVRow + kVSkew(c8) + 4 * r8;
          *(unsigned *)(dst) = o0;
          *(unsigned *)(dst + kVRow) = o1;
          *(unsigned *)(dst + 2 * kVRow) = o2;
          *(unsigned *)(dst + 3 * kVRow) = o3;
        }
      }
      if (g4 == 0) {
        sc[t16] = __half2float(__ushort_as_half(tr.ks0)) * sm;
        sc[16 + t16] = __half2float(__ushort_as_half(tr.ks1)) * sm;
        if (with_v) {
          sc[kTile + t16] = __half2float(__ushort_as_half(tr.vs0));
          sc[kTile + 16 + t16] = __half2float(__ushort_as_half(tr.vs1));
        }
      }
    } else {
      *(int4 *)(Kt + (r4)*kKRow16 + c16 * 16) = tr.k0;
      *(int4 *)(Kt + (4 + r4) * kKRow16 + c16 * 16) = tr.k1;
      *(int4 *)(Kt + (8 + r4) * kKRow16 + c16 * 16) = tr.k2;
      *(int4 *)(Kt + (12 + r4) * kKRow16 + c16 * 16) = tr.k3;
      if (with_v) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const unsigned x0 = dword_of(tr.v0, q4), x1 = dword_of(tr.v1, q4);
          const unsigned x2 = dword_of(tr.v2, q4), x3 = dword_of(tr.v3, q4);
          unsigned *dst = (unsigned *)(Vt + (8 * c16 + 2 * q4) * kVRow + kVSkew(c16 >> 1) + 8 * r4);
          dst[0] = __builtin_amdgcn_perm(x1, x0, 0x05040100u);
          dst[1] = __builtin_amdgcn_perm(x3, x2, 0x05040100u);
          dst[kVRow / 4] = __builtin_amdgcn_perm(x1, x0, 0x07060302u);
          dst[kVRow / 4 + 1] = __builtin_amdgcn_perm(x3, x2, 0x07060302u);
        }
      }
    }
  };

  // A operand of the score contraction: this wavefront's 16 query rows
  half8_t qa[4];
  {
    const int ra = rb * 16 + t16;
    const int q_tok = ra / gq, q_head = ra - q_tok * gq;
    const __half *qrow = a.q + ((((size_t)sl.b * a.q_tokens + q_tok) * cv.Hkv + sl.g) * gq + q_head) * D;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      int4 raw = make_int4(0, 0, 0, 0);
      if (q_tok < tq) raw = *(const int4 *)(qrow + g4 * 32 + 8 * s);
      qa[s] = __builtin_bit_cast(half8_t, raw);
    }
  }
  // raw scores of the 16 rows against the 16 slots [16 sb, 16 sb + 16) of INT8 tile buffer Kt,
  // or against the 16 slots of an FP16 tile; masked entries come back as -inf
  auto scores8 = [&](const uint8_t *Kt, const float *sc, int base, int sb, float (&sv)[4]) {
    const uint8_t *krow = Kt + (16 * sb + t16) * kKRow16 + g4 * 64;
    floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[s], *(const half8_t *)(krow + 16 * s), acc, 0, 0, 0);
    const int slot = base + 16 * sb + t16;
    const float f = sc[16 * sb + t16];
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = (slot < sl.hi8 && okc[i] && slot < seen[i]) ? acc[i] * f : NEG;
  };
  auto scores16 = [&](const uint8_t *Kt, int base, float (&sv)[4]) {
    const uint8_t *krow = Kt + t16 * kKRow16 + g4 * 64;
    floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[s], *(const half8_t *)(krow + 16 * s), acc, 0, 0, 0);
    const int slot = base + t16;
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = (slot < sl.hi16 && okc[i] && slot < seen[i]) ? acc[i] * sm : NEG;
  };

  // ---------------- pass 1: online softmax and output per row ----------------
  TileRegs tr = {};
  if (w < nitems) tr = load_item(w, true);
  append_new_token<D, false>(cv, a, sl, ns);
  _Float16 *Pb = (_Float16 *)(tiles + (size_t)w * kWideTileBytes + kWideKBytes + kVBytes);   // [16][kPRow], this wavefront's own
  for (int i = lane; i < 16 * kPRow / 2; i += kWave) ((unsigned *)Pb)[i] = 0u;
  floatx4_t O[8];
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) O[nt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  float mrun[4], lrun[4], pbias[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { mrun[i] = NEG; lrun[i] = 0.f; pbias[i] = 0.f; }

  for (int sup = 0; sup < nsup; ++sup) {
    const int mine = sup * kAttWaves + w;
    if (sup > 0) __syncthreads();                      // everybody has left the previous eight tiles
    if (mine < nitems) store_item(mine, tr, true);
    __syncthreads();
    if (mine + kAttWaves < nitems) tr = load_item(mine + kAttWaves, true);
    for (int j = st; j < kAttWaves; j += NS) {
      const int it = sup * kAttWaves + j;
      if (it >= nitems) break;
      const uint8_t *Kt = tiles + (size_t)j * kWideTileBytes;
      const uint8_t *Vt = Kt + kWideKBytes;
      const float *sc = (const float *)(Kt + kWideCoreBytes);
      if (it < ntiles) {
        const int base = sl.lo8 + it * kTile;
        float sv[2][4];
        scores8(Kt, sc, base, 0, sv[0]);
        scores8(Kt, sc, base, 1, sv[1]);
        // lazy reference: rescale only when a score of the tile exceeds it by more than kSlack
        constexpr float kSlack = 4.0f;
        bool grow = false;
        float lm[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          lm[i] = fmaxf(sv[0][i], sv[1][i]);
          grow |= lm[i] > mrun[i] + kSlack;
        }
        if (__builtin_amdgcn_ballot_w64(grow)) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float mn = fmaxf(mrun[i], row16_max(lm[i]));
            const float corr = (mn == NEG) ? 1.f : __expf(mrun[i] - mn);
            mrun[i] = mn;
            lrun[i] *= corr;
            pbias[i] *= corr;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) O[nt][i] *= corr;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
          for (int sb = 0; sb < 2; ++sb) {
            const float p = (sv[sb][i] == NEG) ? 0.f : __expf(sv[sb][i] - mrun[i]);
            lrun[i] += p;
            const _Float16 ph = (_Float16)(p * sc[kTile + 16 * sb + t16]);
            pbias[i] += (float)ph;                     // exactly what the matrix core will see
            const int tau = 16 * sb + t16;
            Pb[(4 * g4 + i) * kPRow + 4 * (tau & 7) + (tau >> 3)] = ph;
          }
        }
        wave_lds_sync();
        const half8_t pa = *(const half8_t *)(Pb + t16 * kPRow + 8 * g4);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
          const unsigned *vb = (const unsigned *)(Vt + (16 * nt + t16) * kVRow + kVSkew(nt) + 8 * g4);
          O[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, cvt_i8x8_f16x8_biased(vb[0], vb[1]), O[nt], 0, 0, 0);
        }
        wave_lds_sync();
      } else {
        const int base = sl.lo16 + 16 * (it - ntiles);
        float sv[4];
        scores16(Kt, base, sv);
        bool changed = false;
        float corr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float mn = fmaxf(mrun[i], row16_max(sv[i]));
          corr[i] = (mn == NEG) ? 1.f : __expf(mrun[i] - mn);
          changed |= (mn != mrun[i]);
          mrun[i] = mn;
          const float p = (sv[i] == NEG) ? 0.f : __expf(sv[i] - mn);
          Pb[(4 * g4 + i) * kPRow + 4 * (t16 & 3) + (t16 >> 2)] = (_Float16)p;
          lrun[i] = fmaf(lrun[i], corr[i], p);
          pbias[i] *= corr[i];
        }
        if (__builtin_amdgcn_ballot_w64(changed)) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) O[nt][i] *= corr[i];
        }
        wave_lds_sync();
        const half4_t pa = *(const half4_t *)(Pb + t16 * kPRow + 4 * g4);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
          const unsigned *vb = (const unsigned *)(Vt + (16 * nt + t16) * kVRow + kVSkew(nt) + 8 * g4);
          const uint2 v2 = make_uint2(vb[0], vb[1]);
          O[nt] = __builtin_amdgcn_mfma_f32_16x16x16f16(pa, __builtin_bit_cast(half4_t, v2), O[nt], 0, 0, 0);
        }
        wave_lds_sync();
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    lrun[i] = row16_sum(lrun[i]);
    const float bias = row16_sum(pbias[i]) * kCodeBias;   // what the biased INT8 values added per channel
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) O[nt][i] -= bias;
  }

  // ---------------- the tile streams of a row block merge in LDS ----------------
  if (tid == 0) s_ok = 1;
  __syncthreads();                                       // the tile buffers are free
  if (NS > 1) {
    if (st > 0) {
      float *part = (float *)tiles + (size_t)((st - 1) * RB + rb) * kPartFloats;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) part[(4 * g4 + i) * D + 16 * nt + t16] = O[nt][i];
        if (t16 == 0) { part[16 * D + 4 * g4 + i] = mrun[i]; part[16 * D + 16 + 4 * g4 + i] = lrun[i]; }
      }
    }
    __syncthreads();
    if (st == 0) {
      for (int s = 1; s < NS; ++s) {
        const float *ps = (const float *)tiles + (size_t)((s - 1) * RB + rb) * kPartFloats;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float m2 = ps[16 * D + 4 * g4 + i], l2 = ps[16 * D + 16 + 4 * g4 + i];
          const float M = fmaxf(mrun[i], m2);
          const float f1 = mrun[i] > NEG ? __expf(mrun[i] - M) : 0.f, f2 = m2 > NEG ? __expf(m2 - M) : 0.f;
          lrun[i] = fmaf(lrun[i], f1, m2 > NEG ? l2 * f2 : 0.f);
#pragma unroll
          for (int nt = 0; nt < 8; ++nt)
            O[nt][i] = fmaf(O[nt][i], f1, m2 > NEG ? ps[(4 * g4 + i) * D + 16 * nt + t16] * f2 : 0.f);
          mrun[i] = M;
        }
      }
    }
  }

  // ---------------- exchange between the splits of the unit ----------------
  const size_t row0 = ((size_t)sl.ul * a.max_splits + sl.j) * R;      // this split's first row in the exchange arrays
  if (ns > 1) {
    if (st == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (t16 == 0) {
          st_tagged(&a.part_ml[(row0 + rowc[i]) * 2], tag_of(a), mrun[i]);
          st_tagged(&a.part_ml[(row0 + rowc[i]) * 2 + 1], tag_of(a), lrun[i]);
        }
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) st_tagged(&a.part_o[(row0 + rowc[i]) * D + 16 * nt + t16], tag_of(a), O[nt][i]);
      }
    }
    // every thread gathers some of the ns * R * 2 statistics words of the unit (bounded poll)
    const unsigned long long *words = a.part_ml + (size_t)sl.ul * a.max_splits * R * 2;
    for (int base = 0; base < ns * R * 2; base += kAttThreads) {
      const int idx = base + tid;
      const bool minew = idx < ns * R * 2;
      bool here = !minew;
      for (int spins = 0;; ++spins) {
        if (!here) {
          const unsigned long long wv = ld_tagged(&words[idx]);
          if ((unsigned)(wv >> 32) == tag_of(a)) {
            pml[idx] = __uint_as_float((unsigned)wv);
            here = true;
          }
        }
        if (__builtin_amdgcn_ballot_w64(!here) == 0ull) break;
        __builtin_amdgcn_s_sleep(1);
        if (spins > a.spin_limit) {
          if (!here) s_ok = 0;
          break;
        }
      }
    }
    __syncthreads();
    if (s_ok == 0) {
      if (tid == 0) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
      return;
    }
    // global (M, L) of row r by thread r; the statistics of (split, row) become the weight of
    // that split's output partial
    if (tid < R) {
      float M = NEG;
      for (int s = 0; s < ns; ++s) M = fmaxf(M, pml[(s * R + tid) * 2]);
      double L = 0.0;
      for (int s = 0; s < ns; ++s) {
        const float ms = pml[(s * R + tid) * 2];
        const float es = ms > NEG ? exp_nonpos(ms - M) : 0.f;
        L += (double)es * (double)pml[(s * R + tid) * 2 + 1];
        pml[(s * R + tid) * 2] = es;
      }
      const double inv = recip_pos(L);
      Mrow[tid] = M;
      Irow[tid] = (float)inv;
      Frow[tid] = (float)(inv * row_weight(a, tq, gq, tid));
    }
    __syncthreads();
    if (st == 0) {
      // this split writes the channel groups nt with nt % ns == j of every row of the block
      for (int nt = sl.j; nt < 8; nt += ns) {
        float acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = O[nt][i] * pml[(sl.j * R + rowc[i]) * 2];
        for (int s = 0; s < ns; ++s) {
          if (s == sl.j) continue;
          const unsigned long long *src = a.part_o + (((size_t)sl.ul * a.max_splits + s) * R) * D + 16 * nt + t16;
          unsigned long long wv[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) wv[i] = ld_tagged(&src[(size_t)rowc[i] * D]);
          bool here = true;
#pragma unroll
          for (int i = 0; i < 4; ++i) here &= (unsigned)(wv[i] >> 32) == tag_of(a);
          for (int spins = 0; __builtin_amdgcn_ballot_w64(!here) != 0ull; ++spins) {
            if (spins > a.spin_limit) break;
            __builtin_amdgcn_s_sleep(1);
            if (!here) {
              here = true;
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                wv[i] = ld_tagged(&src[(size_t)rowc[i] * D]);
                here &= (unsigned)(wv[i] >> 32) == tag_of(a);
              }
            }
          }
          const unsigned long long missing = __builtin_amdgcn_ballot_w64(!here);
          if (missing && lane == __builtin_ctzll(missing)) atomicAdd(&cv.stats[kStatDeviceErr], 1ull);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float wgt = pml[(s * R + rowc[i]) * 2];
            acc[i] += wgt > 0.f ? __uint_as_float((unsigned)wv[i]) * wgt : 0.f;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (okc[i] && a.out)
            a.out[out_index(cv, sl, tq, gq, rowc[i] * D + 16 * nt + t16, D)] = __float2half_rn(acc[i] * Irow[rowc[i]]);
      }
    }
  } else {
    if (st == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const double inv = recip_pos((double)lrun[i]);
        if (t16 == 0) {
          Mrow[rowc[i]] = mrun[i];
          Irow[rowc[i]] = (float)inv;
          Frow[rowc[i]] = (float)(inv * row_weight(a, tq, gq, rowc[i]));
        }
        if (okc[i] && a.out) {
#pragma unroll
          for (int nt = 0; nt < 8; ++nt)
            a.out[out_index(cv, sl, tq, gq, rowc[i] * D + 16 * nt + t16, D)] = __float2half_rn(O[nt][i] * (float)inv);
        }
      }
    }
    __syncthreads();
  }

  // ---------------- pass 2: exact mass per slot, EMA ----------------
  float Mi[4], Fi[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { Mi[i] = Mrow[rowc[i]]; Fi[i] = okc[i] ? Frow[rowc[i]] : 0.f; }
  double lam = 1.0;
  for (int k = 0; k < tq; ++k) lam *= (double)a.ema_decay;
  const int first_new = sl.n - tq;
  float *EMA = cv.ema + (size_t)sl.u * cv.cap;
  if (w < nitems) tr = load_item(w, false);
  for (int sup = 0; sup < nsup; ++sup) {
    const int mine = sup * kAttWaves + w;
    __syncthreads();                                     // tiles and column sums of the previous round are done with
    if (mine < nitems) store_item(mine, tr, false);
    __syncthreads();
    if (mine + kAttWaves < nitems) tr = load_item(mine + kAttWaves, false);
    // thread (tile j, slot s) of the first 256 updates that slot's EMA after the column sums are in;
    // its old value is requested now
    const int ema_j = tid >> 5, ema_s = tid & 31;
    bool ema_valid = false;
    int ema_slot = 0, ema_row = 0;
    float ema_old = 0.f;
    if (tid < kAttWaves * kTile && sup * kAttWaves + ema_j < nitems) {
      const int it = sup * kAttWaves + ema_j;
      const bool is8 = it < ntiles;
      ema_slot = is8 ? sl.lo8 + it * kTile + ema_s : sl.lo16 + 16 * (it - ntiles) + ema_s;
      ema_valid = is8 ? ema_slot < sl.hi8 : (ema_s < 16 && ema_slot < sl.hi16);
      if (ema_valid) {
        ema_row = slot_row(cv, sl.tab, sl.h8, sl.n8, sl.h16, ema_slot);
        ema_old = EMA[ema_row];
      }
    }
    for (int j = st; j < kAttWaves; j += NS) {
      const int it = sup * kAttWaves + j;
      if (it >= nitems) break;
      const uint8_t *Kt = tiles + (size_t)j * kWideTileBytes;
      const float *sc = (const float *)(Kt + kWideCoreBytes);
      const int halves = it < ntiles ? 2 : 1;
      for (int sb = 0; sb < halves; ++sb) {
        float sv[4];
        if (it < ntiles) scores8(Kt, sc, sl.lo8 + it * kTile, sb, sv);
        else scores16(Kt, sl.lo16 + 16 * (it - ntiles), sv);
        float c = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) c += (sv[i] == NEG) ? 0.f : exp_nonpos(sv[i] - Mi[i]) * Fi[i];
        c += __shfl_xor(c, 16, kWave);
        c += __shfl_xor(c, 32, kWave);
        // column sums of row block rb over tile j: slot 16 sb + t16
        if (g4 == 0) mass[(size_t)(j * RB + rb) * kTile + 16 * sb + t16] = c;
      }
    }
    __syncthreads();
    if (ema_valid) {
      double A = 0.0;
      for (int r = 0; r < RB; ++r) A += (double)mass[(size_t)(ema_j * RB + r) * kTile + ema_s];   // fixed order: row blocks 0, 1, ..
      const double old = ema_slot >= first_new ? 0.0 : (double)ema_old;       // a token of the call starts at 0
      EMA[ema_row] = (float)(lam * old + a.mass_gain * A);
    }
  }
}

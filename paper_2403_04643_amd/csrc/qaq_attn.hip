// Decode-step attention over the quantized cache (Section 2.1 attention evaluated on
// the midpoint reconstruction of Section 4.1 with the outlier side store of Section 4.2).
//
// One workgroup handles one (sequence, query head, tile of 256 positions) and writes a
// partial (max, sum, unnormalised output); a second kernel merges the tiles, adds the
// unquantized new token and normalises the emitted scores.
//
// Arithmetic.  With per-token scale_t = range_t / 2^B and codes c_td,
//   q.K^_t  = min_t * sum(q) + scale_t * (sum_d q_d c_td + sum(q)/2) + outlier terms
//   X_d     = sum_t [p_t*min_t + w_t*(c_td + 1/2)] + outlier terms,   w_t = p_t*scale_t
// The sums over code fields are exact integer contractions: q (per head) and w (per
// tile) are written in fixed point with 24 resp. 32 bits, split into signed base-256
// digits, and each digit plane goes through the 16x16x64 int8 matrix instruction as one
// row of the A operand, the code bytes being the B operand.  Only one query row exists
// per KV head here, so the other rows of the 16-row tile carry the further digits (and,
// on the key side, three more groups of 16 tokens): the matrix unit is used as a wide
// integer dot engine because the plain vector ALU cannot unpack AND multiply 2-bit codes
// at HBM rate.  Code fields are spread to bytes with one shift and one mask per four
// codes.  All global loads of a tile are issued before the arithmetic starts.
#include "qaq_internal.h"

namespace {

constexpr int kThreads = 256;
typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float h2f(uint16_t b) { return __half2float(__ushort_as_half(b)); }
__device__ __forceinline__ v4i mma(v4i a, v4i b, v4i c) { return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }

template <int N>
__device__ __forceinline__ void load_dwords(const uint8_t* p, uint32_t (&w)[N]) {
  if constexpr (N == 1) {
    w[0] = *(const uint32_t*)p;
  } else if constexpr (N == 2) {
    const uint2 t = *(const uint2*)p;
    w[0] = t.x; w[1] = t.y;
  } else {
    static_assert(N % 4 == 0, "dword count");
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      const uint4 t = ((const uint4*)p)[i];
      w[4 * i] = t.x; w[4 * i + 1] = t.y; w[4 * i + 2] = t.z; w[4 * i + 3] = t.w;
    }
  }
}
template <int N>
__device__ __forceinline__ void zero_dwords(uint32_t (&w)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) w[i] = 0u;
}

template <int D>
struct AttnLds {
  float qf[D];
  alignas(16) int8_t ql[4][D];            // query digits (row 3 is zero)
  float logit[QAQ_TT];                    // raw logits by position, later p = exp(logit - max)
  alignas(16) int8_t wl2[4][QAQ_TT];      // weight digits per slot of the 2-bit field region
  alignas(16) int8_t wl1[4][QAQ_TT];      // ... of the 1-bit field region
  alignas(16) int8_t wl4[4][QAQ_TT];      // ... of the 4-bit region
  float w8[QAQ_TT];                       // fp32 weights of the 8-bit slots
  float xpart[4][D];                      // per-wavefront partial outputs (integer path)
  float x8part[4][D];                     // per-wavefront partials of the 8-bit class
  float xcorr[D];                         // outlier corrections of the output
  float red[12];
  int redi[4];
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Signed base-256 digits of an integer (each in [-128, 127]).
__device__ __forceinline__ void digits3(int x, int& d0, int& d1, int& d2) {
  d0 = ((x + 128) & 255) - 128;
  const int r = (x - d0) >> 8;
  d1 = ((r + 128) & 255) - 128;
  d2 = (r - d1) >> 8;
}
__device__ __forceinline__ uint32_t digits4_packed(int x) {
  const int d0 = ((x + 128) & 255) - 128;
  const int r = (x - d0) >> 8;
  const int d1 = ((r + 128) & 255) - 128;
  const int r2 = (r - d1) >> 8;
  const int d2 = ((r2 + 128) & 255) - 128;
  const int d3 = (r2 - d2) >> 8;
  return (uint32_t)(d0 & 255) | ((uint32_t)(d1 & 255) << 8) | ((uint32_t)(d2 & 255) << 16) | ((uint32_t)(d3 & 255) << 24);
}

// B operand (16 byte-spread codes of one slice) from packed fields.
template <int BF>
__device__ __forceinline__ v4i spread(const uint32_t* w, int nib) {
  v4i b;
  if constexpr (BF == 2) {
    b[0] = (int)(w[0] & 0x03030303u); b[1] = (int)((w[0] >> 2) & 0x03030303u);
    b[2] = (int)((w[0] >> 4) & 0x03030303u); b[3] = (int)((w[0] >> 6) & 0x03030303u);
  } else if constexpr (BF == 1) {
    const uint32_t x = w[0] >> (4 * nib);
    b[0] = (int)(x & 0x01010101u); b[1] = (int)((x >> 1) & 0x01010101u);
    b[2] = (int)((x >> 2) & 0x01010101u); b[3] = (int)((x >> 3) & 0x01010101u);
  } else if constexpr (BF == 4) {
    b[0] = (int)(w[0] & 0x0f0f0f0fu); b[1] = (int)((w[0] >> 4) & 0x0f0f0f0fu);
    b[2] = (int)(w[1] & 0x0f0f0f0fu); b[3] = (int)((w[1] >> 4) & 0x0f0f0f0fu);
  } else {
    b[0] = (int)w[0]; b[1] = (int)w[1]; b[2] = (int)w[2]; b[3] = (int)w[3];
  }
  return b;
}

// Dwords lane (n, g) reads of one key record of field width BF.
template <int D, int BF>
struct KRec {
  static constexpr int KS = D / 64;
  static constexpr int REC = D * BF / 8;
  static constexpr int NDW = (KS * BF / 2) > 0 ? (KS * BF / 2) : 1;
  static __device__ __forceinline__ void load(const uint8_t* rbase, int ridx, int g, uint32_t (&w)[NDW]) {
    const uint8_t* rec = rbase + (size_t)ridx * REC;
    if constexpr (BF == 1 && KS == 1) load_dwords<1>(rec + 4 * (g >> 1), w);
    else load_dwords<NDW>(rec + 4 * NDW * g, w);
  }
  // B operand of k-step ks
  static __device__ __forceinline__ v4i operand(const uint32_t (&w)[NDW], int ks, int g) {
    if constexpr (BF == 1) return spread<1>(w, KS == 1 ? (g & 1) : ks);
    else return spread<BF>(w + ks * (BF / 2), 0);
  }
};

// One group of 64 key records through the matrix unit: lane l ends with the digit sums
// (c[0], c[1], c[2]) of record 64*grp + l.
template <int D, int BF>
__device__ __forceinline__ v4i k_group(const uint32_t (&w)[4][KRec<D, BF>::NDW], const v4i (&aq)[D / 64], int tgp, int g) {
  constexpr int KS = D / 64;
  const v4i zero = {0, 0, 0, 0};
  v4i c = zero;
#pragma unroll
  for (int tg = 0; tg < 4; ++tg)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const v4i a = (tgp == tg) ? aq[ks] : zero;
      c = mma(a, KRec<D, BF>::operand(w[tg], ks, g), c);
    }
  return c;
}

template <int D, int BF>
__device__ __forceinline__ void k_load_group(const uint8_t* rbase, int n_rec, int grp, int nn, int g,
                                             uint32_t (&w)[4][KRec<D, BF>::NDW]) {
#pragma unroll
  for (int tg = 0; tg < 4; ++tg) {
    const int ridx = grp * 64 + 16 * tg + nn;
    if (ridx < n_rec) KRec<D, BF>::load(rbase, ridx, g, w[tg]);
    else zero_dwords(w[tg]);
  }
}

template <int D>
__global__ __launch_bounds__(kThreads) void k_attn_partial(QaqAttnArgs a) {
  constexpr int KS = D / 64;
  constexpr int NCG = D / 16;
  __shared__ AttnLds<D> S;
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nn = lane & 15, g = lane >> 4;
  const int tile = blockIdx.x;
  const int bq = blockIdx.y, b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
  const int n_tok = min(a.len - tile * QAQ_TT, QAQ_TT);
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const int no2 = v.no2;
  const v4i zero4 = {0, 0, 0, 0};

  // ---- issue every load of the tile that does not depend on the arithmetic ------------
  const QaqCounts cK = qaq_load_counts(v, 0, b, h, tile);
  const QaqCounts cV = qaq_load_counts(v, 1, b, h, tile);
  const QaqKRegions rK = qaq_k_regions(cK, D);
  const QaqVRegions rV = qaq_v_regions(cV, D);
  const uint8_t* baseK = qaq_tile_codes(v, 0, b, h, tile);
  const uint8_t* baseV = qaq_tile_codes(v, 1, b, h, tile);
  const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
  const int n32K = cK.n32(), n32V = cV.n32();

  float qv = 0.0f;
  if (tid < D) qv = __half2float(a.q[(size_t)bq * D + tid]);
  // metadata of key slot tid and value slot tid
  uint32_t mmK = 0, mmV = 0;
  int posK = 0, posV = 0;
  uint8_t oiK[QAQ_MAX_NO2], oiV[QAQ_MAX_NO2];
  uint16_t ovK[QAQ_MAX_NO2], ovV[QAQ_MAX_NO2];
  if (tid < n_tok) {
    mmK = v.mm[0][gi0 + tid]; posK = v.perm[0][gi0 + tid];
    mmV = v.mm[1][gi0 + tid]; posV = v.perm[1][gi0 + tid];
#pragma unroll
    for (int j = 0; j < QAQ_MAX_NO2; ++j) {
      if (j < no2) {
        oiK[j] = v.oidx[0][(gi0 + tid) * no2 + j]; ovK[j] = v.oval[0][(gi0 + tid) * no2 + j];
        oiV[j] = v.oidx[1][(gi0 + tid) * no2 + j]; ovV[j] = v.oval[1][(gi0 + tid) * no2 + j];
      }
    }
  }
  // key codes of the low-width regions: this wavefront's 64 records
  uint32_t kw2[4][KRec<D, 2>::NDW], kw1[4][KRec<D, 1>::NDW];
  k_load_group<D, 2>(baseK + rK.r2, n32K, wave, nn, g, kw2);
  k_load_group<D, 1>(baseK + rK.r1, cK.n3, wave, nn, g, kw1);
  // value codes of the low-width regions: this lane group's unit of 16 slots
  const int uV = wave * 4 + g;
  uint32_t vw2[NCG], vw1[NCG / 2];
  if (uV * 16 < n32V) load_dwords<NCG>(baseV + rV.r2 + (size_t)uV * (4 * D) + (size_t)nn * (NCG * 4), vw2);
  else zero_dwords(vw2);
  if (uV * 16 < cV.n3) load_dwords<NCG / 2>(baseV + rV.r1 + (size_t)uV * (2 * D) + (size_t)nn * (NCG * 2), vw1);
  else zero_dwords(vw1);

  // ---- query: fp32 copy, fixed-point digits ---------------------------------------------
  if (tid < D) { S.qf[tid] = qv; S.xcorr[tid] = 0.0f; S.ql[3][tid] = 0; }
  {
    const float am = wave_max(fabsf(qv));
    const float sm = wave_sum(qv);
    if (lane == 0) { S.red[wave] = am; S.red[4 + wave] = sm; }
  }
  __syncthreads();
  const float qmax = fmaxf(fmaxf(S.red[0], S.red[1]), fmaxf(S.red[2], S.red[3]));
  const float sumq = (S.red[4] + S.red[5]) + (S.red[6] + S.red[7]);
  int qexp = 0;
  if (qmax > 0.0f) (void)frexpf(qmax, &qexp);
  const float qscale = qmax > 0.0f ? ldexpf(1.0f, qexp - 22) : 0.0f;
  int qi = 0;
  if (tid < D) {
    qi = qmax > 0.0f ? (int)rintf(ldexpf(qv, 22 - qexp)) : 0;
    int d0, d1, d2;
    digits3(qi, d0, d1, d2);
    S.ql[0][tid] = (int8_t)d0; S.ql[1][tid] = (int8_t)d1; S.ql[2][tid] = (int8_t)d2;
  }
  {
    int si = qi;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) si += __shfl_xor(si, o);
    if (lane == 0) S.redi[wave] = si;
  }
  __syncthreads();
  const int sumqi = S.redi[0] + S.redi[1] + S.redi[2] + S.redi[3];
  // A operand of the key contraction: row r of the 16-row tile carries digit r%4 of the
  // query, and only the rows of token group r/4 are switched on per instruction
  v4i aq[KS];
  const int tgp = nn >> 2;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) aq[ks] = *(const v4i*)&S.ql[nn & 3][64 * ks + 16 * g];

  // ---- keys: logits -----------------------------------------------------------------------
  auto finish = [&](uint32_t m, int pos, const uint8_t* oi, const uint16_t* ov, int bits, float mult, float real) {
    const float mn = h2f((uint16_t)(m & 0xffffu)), mx = h2f((uint16_t)(m >> 16));
    const float range = mx - mn;
    const float scale = ldexpf(range, -bits);
    float val = mn * sumq + scale * (mult * real + 0.5f * sumq);
    const float ctop = (float)((1 << bits) - 1) + 0.5f;
#pragma unroll
    for (int j = 0; j < QAQ_MAX_NO2; ++j) {
      if (j < no2) {
        const float o = h2f(ov[j]);
        const float deq = mn + ((o >= mx && range > 0.0f) ? ctop : 0.5f) * scale;
        val += S.qf[oi[j]] * (o - deq);
      }
    }
    S.logit[pos] = val * inv_sqrt_d;
  };
  auto real_of = [&](const v4i& c) { return (((float)c[2] * 65536.0f + (float)c[1] * 256.0f) + (float)c[0]) * qscale; };

  if (wave * 64 < n32K) {
    const v4i c = k_group<D, 2>(kw2, aq, tgp, g);
    if (tid < n32K) {
      const bool three = tid < cK.n3;
      finish(mmK, posK, oiK, ovK, three ? 3 : 2, three ? 2.0f : 1.0f, real_of(c));
    }
  }
  // wider classes: loaded when needed (few tokens at the operating points of interest)
  for (int grp = wave; grp * 64 < cK.n4; grp += 4) {
    uint32_t w[4][KRec<D, 4>::NDW];
    k_load_group<D, 4>(baseK + rK.r4, cK.n4, grp, nn, g, w);
    const v4i c = k_group<D, 4>(w, aq, tgp, g);
    const int idx = grp * 64 + lane;
    if (idx < cK.n4) {
      const size_t gi = gi0 + n32K + idx;
      uint8_t oi[QAQ_MAX_NO2]; uint16_t ov[QAQ_MAX_NO2];
      for (int j = 0; j < no2; ++j) { oi[j] = v.oidx[0][gi * no2 + j]; ov[j] = v.oval[0][gi * no2 + j]; }
      finish(v.mm[0][gi], v.perm[0][gi], oi, ov, 4, 1.0f, real_of(c));
    }
  }
  for (int grp = wave; grp * 64 < cK.n8; grp += 4) {
    uint32_t w[4][KRec<D, 8>::NDW];
    k_load_group<D, 8>(baseK + rK.r8, cK.n8, grp, nn, g, w);
    const v4i c = k_group<D, 8>(w, aq, tgp, g);
    const int idx = grp * 64 + lane;
    if (idx < cK.n8) {
      const size_t gi = gi0 + n32K + cK.n4 + idx;
      uint8_t oi[QAQ_MAX_NO2]; uint16_t ov[QAQ_MAX_NO2];
      for (int j = 0; j < no2; ++j) { oi[j] = v.oidx[0][gi * no2 + j]; ov[j] = v.oval[0][gi * no2 + j]; }
      // stored bytes are code - 128
      const float real = ((((float)c[2] * 65536.0f + (float)c[1] * 256.0f) + (float)c[0]) + 128.0f * (float)sumqi) * qscale;
      finish(v.mm[0][gi], v.perm[0][gi], oi, ov, 8, 1.0f, real);
    }
  }
  // low bit of the 3-bit tokens: same slot, added to the logit written just above
  if (wave * 64 < cK.n3) {
    const v4i c = k_group<D, 1>(kw1, aq, tgp, g);
    if (tid < cK.n3) {
      const float range = h2f((uint16_t)(mmK >> 16)) - h2f((uint16_t)(mmK & 0xffffu));
      S.logit[posK] += ldexpf(range, -3) * real_of(c) * inv_sqrt_d;
    }
  }
  __syncthreads();

  // ---- softmax inside the tile ----------------------------------------------------------
  const float lg = tid < n_tok ? S.logit[tid] : -INFINITY;
  if (a.scores && tid < n_tok) a.scores[(size_t)bq * a.score_stride + tile * QAQ_TT + tid] = lg;
  {
    const float wm = wave_max(lg);
    if (lane == 0) S.red[wave] = wm;
  }
  __syncthreads();
  const float tmax = fmaxf(fmaxf(S.red[0], S.red[1]), fmaxf(S.red[2], S.red[3]));
  const float p = tid < n_tok ? __expf(lg - tmax) : 0.0f;
  if (tid < n_tok) S.logit[tid] = p;
  {
    const float ws = wave_sum(p);
    if (lane == 0) S.red[4 + wave] = ws;
  }
  __syncthreads();
  const float lsum = (S.red[4] + S.red[5]) + (S.red[6] + S.red[7]);

  // ---- values: weights per slot ---------------------------------------------------------
  float w_eff = 0.0f, w1 = 0.0f, bias_l = 0.0f;
  const int first8V = n32V + cV.n4;
  if (tid < n_tok) {
    const int s = tid;
    const float pt = S.logit[posV];
    const float mn = h2f((uint16_t)(mmV & 0xffffu)), mx = h2f((uint16_t)(mmV >> 16));
    const float range = mx - mn;
    const int bits = cV.bits_of_slot(s);
    const float scale = ldexpf(range, -bits);
    const float w = pt * scale;
    bias_l = pt * mn + 0.5f * w;
    const float ctop = (float)((1 << bits) - 1) + 0.5f;
#pragma unroll
    for (int j = 0; j < QAQ_MAX_NO2; ++j) {
      if (j < no2) {
        const float o = h2f(ovV[j]);
        const float deq = mn + ((o >= mx && range > 0.0f) ? ctop : 0.5f) * scale;
        atomicAdd(&S.xcorr[oiV[j]], pt * (o - deq));
      }
    }
    if (s < cV.n3) { w_eff = 2.0f * w; w1 = w; }
    else if (s < first8V) w_eff = w;
    else S.w8[s - first8V] = w;
  }
  {
    const float wm = wave_max(w_eff);
    const float bs = wave_sum(bias_l);
    if (lane == 0) { S.red[8 + wave] = wm; S.red[wave] = bs; }
  }
  __syncthreads();
  const float wmax = fmaxf(fmaxf(S.red[8], S.red[9]), fmaxf(S.red[10], S.red[11]));
  const float bias = (S.red[0] + S.red[1]) + (S.red[2] + S.red[3]);
  int wexp = 0;
  if (wmax > 0.0f) (void)frexpf(wmax, &wexp);
  const float wscale = wmax > 0.0f ? ldexpf(1.0f, wexp - 30) : 0.0f;
  {
    // every entry of the three digit tables is written exactly once (zero where the slot
    // is not in that region), so partial units multiply padding by zero
    const int s = tid;
    const bool live = wmax > 0.0f && s < n_tok;
    const uint32_t dg = live && s < first8V ? digits4_packed((int)rintf(ldexpf(w_eff, 30 - wexp))) : 0u;
    const uint32_t d2 = s < n32V ? dg : 0u;
    S.wl2[0][s] = (int8_t)d2; S.wl2[1][s] = (int8_t)(d2 >> 8); S.wl2[2][s] = (int8_t)(d2 >> 16); S.wl2[3][s] = (int8_t)(d2 >> 24);
    const uint32_t d1 = live && s < cV.n3 ? digits4_packed((int)rintf(ldexpf(w1, 30 - wexp))) : 0u;
    S.wl1[0][s] = (int8_t)d1; S.wl1[1][s] = (int8_t)(d1 >> 8); S.wl1[2][s] = (int8_t)(d1 >> 16); S.wl1[3][s] = (int8_t)(d1 >> 24);
    const int i4 = (s - n32V) & (QAQ_TT - 1);
    const uint32_t d4 = (s >= n32V && s < first8V) ? dg : 0u;
    S.wl4[0][i4] = (int8_t)d4; S.wl4[1][i4] = (int8_t)(d4 >> 8); S.wl4[2][i4] = (int8_t)(d4 >> 16); S.wl4[3][i4] = (int8_t)(d4 >> 24);
  }
  __syncthreads();

  // ---- values: integer contractions, rows 0..3 of the tile = the four digits of w --------
  v4i cv[NCG];
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) cv[cg] = zero4;
  if (wave * 64 < n32V) {
    const v4i wa = nn < 4 ? *(const v4i*)&S.wl2[nn][16 * uV] : zero4;
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) cv[cg] = mma(wa, spread<2>(&vw2[cg], 0), cv[cg]);
  }
  if (wave * 64 < cV.n3) {
    const v4i wa = nn < 4 ? *(const v4i*)&S.wl1[nn][16 * uV] : zero4;
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) cv[cg] = mma(wa, spread<1>(&vw1[cg >> 1], cg & 1), cv[cg]);
  }
  for (int blk = wave; blk * 64 < cV.n4; blk += 4) {
    const int u = blk * 4 + g;                 // 16 slots = half-units 2u, 2u+1
    uint32_t w0[NCG], w1d[NCG];
    if ((2 * u) * 8 < cV.n4) load_dwords<NCG>(baseV + rV.r4 + (size_t)(2 * u) * (4 * D) + (size_t)nn * (NCG * 4), w0);
    else zero_dwords(w0);
    if ((2 * u + 1) * 8 < cV.n4) load_dwords<NCG>(baseV + rV.r4 + (size_t)(2 * u + 1) * (4 * D) + (size_t)nn * (NCG * 4), w1d);
    else zero_dwords(w1d);
    const v4i wa = nn < 4 ? *(const v4i*)&S.wl4[nn][16 * u] : zero4;
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
      const uint32_t pr[2] = {w0[cg], w1d[cg]};
      cv[cg] = mma(wa, spread<4>(pr, 0), cv[cg]);
    }
  }
  if (g == 0) {
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg) {
      const float hi = (float)cv[cg][3] * 16777216.0f + (float)cv[cg][2] * 65536.0f;
      const float lo = (float)cv[cg][1] * 256.0f + (float)cv[cg][0];
      S.xpart[wave][16 * cg + nn] = (hi + lo) * wscale;
    }
  }
  // 8-bit codes: token-major bytes, plain fp32 multiply-add
  {
    constexpr int LPT8 = D / 4;          // lanes per token
    constexpr int TPW = 64 / LPT8;       // tokens per wavefront pass
    float a8[4] = {0.f, 0.f, 0.f, 0.f};
    const int sub = lane / LPT8, ch4 = lane % LPT8;
    for (int i8 = wave * TPW + sub; i8 < cV.n8; i8 += 4 * TPW) {
      const float w = S.w8[i8];
      const uint32_t dw = *(const uint32_t*)(baseV + rV.r8 + (size_t)i8 * D + 4 * ch4);
#pragma unroll
      for (int j = 0; j < 4; ++j) a8[j] += w * (float)((dw >> (8 * j)) & 255u);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float t = a8[j];
      if constexpr (TPW == 4) t += __shfl_xor(t, 16);
      t += __shfl_xor(t, 32);
      if (sub == 0) S.x8part[wave][4 * ch4 + j] = t;
    }
  }
  __syncthreads();
  if (tid < D) {
    float x = (S.xpart[0][tid] + S.xpart[1][tid]) + (S.xpart[2][tid] + S.xpart[3][tid]);
    x += (S.x8part[0][tid] + S.x8part[1][tid]) + (S.x8part[2][tid] + S.x8part[3][tid]);
    x += S.xcorr[tid] + bias;
    float* part = v.partial + ((size_t)bq * v.NT + tile) * (D + 4);
    part[tid] = x;
    if (tid == 0) { part[D] = tmax; part[D + 1] = lsum; }
  }
}

// Merge the tiles of one (sequence, query head), add the unquantized new token and
// normalise.  Block x = 0 writes the output vector; every block normalises its share of
// the emitted scores (each recomputes the head's max and sum from the per-tile pairs).
template <int D>
__global__ __launch_bounds__(kThreads) void k_attn_combine(QaqAttnArgs a) {
  __shared__ float red[8];
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bq = blockIdx.y, b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  const float* part = v.partial + (size_t)bq * v.NT * (D + 4);
  float a_new = -INFINITY;
  if (a.k_new) {
    float t = 0.0f;
    if (tid < D) t = __half2float(a.q[(size_t)bq * D + tid]) * __half2float(a.k_new[((size_t)b * v.Hkv + h) * D + tid]);
    t = wave_sum(t);
    if (lane == 0) red[wave] = t;
    __syncthreads();
    a_new = ((red[0] + red[1]) + (red[2] + red[3])) / sqrtf((float)D);
  }
  // per-tile (max, sum): lanes take tiles round robin, then an all-reduce in the wavefront
  float M = a_new;
  for (int i = lane; i < ntile; i += 64) M = fmaxf(M, part[(size_t)i * (D + 4) + D]);
  M = wave_max(M);
  float lsum = 0.0f;
  for (int i = lane; i < ntile; i += 64)
    lsum += __expf(part[(size_t)i * (D + 4) + D] - M) * part[(size_t)i * (D + 4) + D + 1];
  lsum = wave_sum(lsum);
  float e_new = 0.0f;
  if (a.k_new) { e_new = __expf(a_new - M); lsum += e_new; }
  const float inv = 1.0f / lsum;
  if (blockIdx.x == 0) {
    if (tid < D) {
      float x = 0.0f;
      for (int i = 0; i < ntile; ++i) x += __expf(part[(size_t)i * (D + 4) + D] - M) * part[(size_t)i * (D + 4) + tid];
      if (a.k_new) x += e_new * __half2float(a.v_new[((size_t)b * v.Hkv + h) * D + tid]);
      if (a.out_is_fp32) ((float*)a.out)[(size_t)bq * D + tid] = x * inv;
      else ((__half*)a.out)[(size_t)bq * D + tid] = __float2half_rn(x * inv);
    }
    if (a.scores && a.k_new && tid == 0) a.scores[(size_t)bq * a.score_stride + a.len] = e_new * inv;
  }
  if (a.scores) {
    float* sc = a.scores + (size_t)bq * a.score_stride;
    const int t0 = blockIdx.x * (4 * kThreads);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int t = t0 + k * kThreads + tid;
      if (t < a.len) sc[t] = __expf(sc[t] - M) * inv;
    }
  }
}

}  // namespace

hipError_t qaq_launch_attention(const QaqAttnArgs& a, hipStream_t s, hipEvent_t* ev) {
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  const int BQ = a.v.B * a.v.Hq;
  if (ev) (void)hipEventRecord(ev[0], s);
  if (ntile > 0) {
    if (a.v.D == 128) hipLaunchKernelGGL(k_attn_partial<128>, dim3(ntile, BQ), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(k_attn_partial<64>, dim3(ntile, BQ), dim3(kThreads), 0, s, a);
  }
  if (ev) (void)hipEventRecord(ev[1], s);
  const int nblk = a.scores ? (a.len + 4 * kThreads - 1) / (4 * kThreads) : 1;
  dim3 grid(nblk < 1 ? 1 : nblk, BQ);
  if (a.v.D == 128) hipLaunchKernelGGL(k_attn_combine<128>, grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(k_attn_combine<64>, grid, dim3(kThreads), 0, s, a);
  if (ev) (void)hipEventRecord(ev[2], s);
  return hipGetLastError();
}

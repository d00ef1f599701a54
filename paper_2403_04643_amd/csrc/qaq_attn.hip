// Decode-step attention over the quantized cache (Section 2.1 attention evaluated on
// the midpoint reconstruction of Section 4.1 with the outlier side store of Section 4.2).
//
// One workgroup handles one (sequence, query head) and a chunk of up to four tiles of 256
// positions and writes a partial (max, sum, unnormalised output); a second kernel merges
// the chunks, adds the unquantized new token and normalises the emitted scores.
//
// Arithmetic.  With per-token scale_t = range_t / 2^B and codes c_td,
//   q.K^_t  = min_t * sum(q) + scale_t * (sum_d q_d c_td + sum(q)/2) + outlier terms
//   X_d     = sum_t [p_t*min_t + w_t*(c_td + 1/2)] + outlier terms,   w_t = p_t*scale_t
// The sums over code fields are exact integer contractions: q (per head) and w (per
// chunk) are written in fixed point with 24 resp. 32 bits, split into signed base-256
// digits, and each digit plane goes through the 16x16x64 int8 matrix instruction as one
// row of the A operand, the code bytes being the B operand.  Only one query row exists
// per KV head here, so the other rows of the 16-row tile carry the further digits (and,
// on the key side, three more groups of 16 tokens): the matrix unit is used as a wide
// integer dot engine because the plain vector ALU cannot unpack AND multiply 2-bit codes
// at HBM rate.  Code fields are spread to bytes with one shift and one mask per four
// codes.
//
// Schedule of a workgroup: all key-side loads of the chunk are issued first; the key
// contractions of the tiles run without barriers and leave logits in LDS; value-side
// loads are issued as key registers free up; after one barrier the chunk maximum is
// known, every thread turns its value slot of each tile into weight digits, and after a
// second barrier the value contractions of all tiles accumulate into one set of integer
// accumulators that is converted to fp32 once per chunk.
#include "qaq_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int NTC = 4;   // tiles per workgroup
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
  alignas(16) int8_t ql[4][D];                     // query digits, row 3 zero
  alignas(16) int8_t qa[4][D / 64][4][16][16];     // A operands [token group][k-step][lane group][row][16 B]
  float logit[NTC][QAQ_TT];                        // raw logits by position
  alignas(16) int8_t wl2[NTC][4][QAQ_TT];          // weight digits per slot of the 2-bit field region
  alignas(16) int8_t wl1[NTC][4][QAQ_TT];          // ... of the 1-bit field region
  alignas(16) int8_t wl4[NTC][4][QAQ_TT];          // ... of the 4-bit region
  float w8[NTC][QAQ_TT];                           // fp32 weights of the 8-bit slots
  float xpart[4][D];                               // per-wavefront partial outputs (integer path)
  float x8part[4][D];                              // per-wavefront partials of the 8-bit class
  float xcorr[D];                                  // outlier corrections of the output
  float red[16];
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
    const uint8_t* rec = rbase + (uint32_t)ridx * (uint32_t)REC;
    if constexpr (BF == 1 && KS == 1) load_dwords<1>(rec + 4 * (g >> 1), w);
    else load_dwords<NDW>(rec + 4 * NDW * g, w);
  }
  static __device__ __forceinline__ v4i operand(const uint32_t (&w)[NDW], int ks, int g) {
    if constexpr (BF == 1) return spread<1>(w, KS == 1 ? (g & 1) : ks);
    else return spread<BF>(w + ks * (BF / 2), 0);
  }
};

// 64 key records through the matrix unit: lane l ends with the digit sums (c[0..2]) of
// record 64*grp + l.  The A operand of token group tg has the query digits in rows
// 4*tg..4*tg+2 and zeros elsewhere, so the four groups land in the four row blocks.
template <int D, int BF>
__device__ __forceinline__ v4i k_group(const uint32_t (&w)[4][KRec<D, BF>::NDW], const AttnLds<D>& S, int nn, int g) {
  constexpr int KS = D / 64;
  v4i c = {0, 0, 0, 0};
#pragma unroll
  for (int tg = 0; tg < 4; ++tg)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const v4i a = *(const v4i*)&S.qa[tg][ks][g][nn][0];
      c = mma(a, KRec<D, BF>::operand(w[tg], ks, g), c);
    }
  return c;
}

// Records past the end of the region read the last record instead (never out of bounds);
// their results are not used.
template <int D, int BF>
__device__ __forceinline__ void k_load_group(const uint8_t* rbase, int n_rec, int grp, int nn, int g,
                                             uint32_t (&w)[4][KRec<D, BF>::NDW]) {
#pragma unroll
  for (int tg = 0; tg < 4; ++tg) {
    const int ridx = min(grp * 64 + 16 * tg + nn, n_rec - 1);
    KRec<D, BF>::load(rbase, ridx, g, w[tg]);
  }
}

// Outlier side store of one slot: NO2 entries known at compile time (0 or 2), or up to 8
// with a run-time count.
template <int NO2>
struct Outl {
  static constexpr int CAP = NO2 ? NO2 : 1;
  uint8_t idx[CAP];
  uint16_t val[CAP];
  __device__ __forceinline__ void load(const QaqView& v, int side, size_t gi, int no2) {
    if constexpr (NO2 == 2) {
      const uint16_t i2 = *(const uint16_t*)(v.oidx[side] + gi * 2);
      const uint32_t v2 = *(const uint32_t*)(v.oval[side] + gi * 2);
      idx[0] = (uint8_t)i2; idx[1] = (uint8_t)(i2 >> 8);
      val[0] = (uint16_t)v2; val[1] = (uint16_t)(v2 >> 16);
    } else if constexpr (NO2 > 2) {
#pragma unroll
      for (int j = 0; j < NO2; ++j)
        if (j < no2) { idx[j] = v.oidx[side][gi * no2 + j]; val[j] = v.oval[side][gi * no2 + j]; }
    }
  }
};

template <int D, int NO2>
__global__ __launch_bounds__(kThreads) void k_attn_partial(QaqAttnArgs a) {
  constexpr int KS = D / 64;
  constexpr int NCG = D / 16;
  __shared__ AttnLds<D> S;
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nn = lane & 15, g = lane >> 4;
  const int chunk = blockIdx.x;
  const int bq = blockIdx.y, b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  const int tile0 = chunk * NTC;
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const int no2 = v.no2;
  const v4i zero4 = {0, 0, 0, 0};

  // ---- per-tile bookkeeping (uniform) and the loads that do not wait for arithmetic ------
  QaqCounts cK[NTC], cV[NTC];
  int ntok[NTC];
#pragma unroll
  for (int t = 0; t < NTC; ++t) {
    const int tile = tile0 + t;
    ntok[t] = tile < ntile ? min(a.len - tile * QAQ_TT, QAQ_TT) : 0;
    if (ntok[t] > 0) { cK[t] = qaq_load_counts(v, 0, b, h, tile); cV[t] = qaq_load_counts(v, 1, b, h, tile); }
    else { cK[t].n3 = cK[t].n2 = cK[t].n4 = cK[t].n8 = 0; cV[t] = cK[t]; }
  }
  float qv = 0.0f;
  if (tid < D) qv = __half2float(a.q[(size_t)bq * D + tid]);

  uint32_t kw2[NTC][4][KRec<D, 2>::NDW], kw1[NTC][4][KRec<D, 1>::NDW];
  uint32_t mmK[NTC], mmV[NTC];
  int posK[NTC], posV[NTC];
  Outl<NO2> oK[NTC], oV[NTC];
#pragma unroll
  for (int t = 0; t < NTC; ++t) {
    if (ntok[t] > 0) {
      const int tile = tile0 + t;
      const uint8_t* baseK = qaq_tile_codes(v, 0, b, h, tile);
      const QaqKRegions rK = qaq_k_regions(cK[t], D);
      if (cK[t].n32() > wave * 64) k_load_group<D, 2>(baseK + rK.r2, cK[t].n32(), wave, nn, g, kw2[t]);
      if (cK[t].n3 > wave * 64) k_load_group<D, 1>(baseK + rK.r1, cK[t].n3, wave, nn, g, kw1[t]);
      const size_t gi = qaq_slot_index(v, b, h, tile, min(tid, ntok[t] - 1));
      mmK[t] = v.mm[0][gi]; posK[t] = v.perm[0][gi]; oK[t].load(v, 0, gi, no2);
      mmV[t] = v.mm[1][gi]; posV[t] = v.perm[1][gi]; oV[t].load(v, 1, gi, no2);
    }
  }

  // ---- query: fp32 copy, fixed-point digits, A operands ------------------------------------
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
  for (int e = tid; e < 4 * KS * 4 * 16; e += kThreads) {
    const int row = e & 15, gg = (e >> 4) & 3, ks = (e >> 6) % KS, tg = (e >> 6) / KS;
    v4i val = zero4;
    if ((row >> 2) == tg) val = *(const v4i*)&S.ql[row & 3][64 * ks + 16 * gg];
    *(v4i*)&S.qa[tg][ks][gg][row][0] = val;
  }
  __syncthreads();

  // ---- keys: logits of every tile of the chunk --------------------------------------------
  auto real_of = [&](const v4i& c) { return (((float)c[2] * 65536.0f + (float)c[1] * 256.0f) + (float)c[0]) * qscale; };
  auto key_logit = [&](uint32_t m, const Outl<NO2>& o, int bits, float dotq) {
    // dotq = sum_d q_d c_d in real units
    const float mn = h2f((uint16_t)(m & 0xffffu)), mx = h2f((uint16_t)(m >> 16));
    const float range = mx - mn;
    const float scale = ldexpf(range, -bits);
    float val = mn * sumq + scale * (dotq + 0.5f * sumq);
    const float ctop = (float)((1 << bits) - 1) + 0.5f;
#pragma unroll
    for (int j = 0; j < Outl<NO2>::CAP; ++j) {
      if (j < NO2 && j < no2) {
        const float ov = h2f(o.val[j]);
        const float deq = mn + ((ov >= mx && range > 0.0f) ? ctop : 0.5f) * scale;
        val += S.qf[o.idx[j]] * (ov - deq);
      }
    }
    return val * inv_sqrt_d;
  };

  uint32_t vw2[NTC][NCG], vw1[NTC][NCG / 2];
  float vmax = -INFINITY;
#pragma unroll
  for (int t = 0; t < NTC; ++t) {
    if (ntok[t] <= 0) continue;
    const int tile = tile0 + t;
    const QaqCounts& c = cK[t];
    const int n32 = c.n32();
    const uint8_t* baseK = qaq_tile_codes(v, 0, b, h, tile);
    const QaqKRegions rK = qaq_k_regions(c, D);
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    if (wave * 64 < n32) {
      v4i c2 = k_group<D, 2>(kw2[t], S, nn, g);
      float dotq = real_of(c2);
      const bool three = tid < c.n3;
      if (wave * 64 < c.n3) {
        const v4i c1 = k_group<D, 1>(kw1[t], S, nn, g);
        dotq = three ? 2.0f * dotq + real_of(c1) : dotq;
      }
      if (tid < n32) {
        const float lg = key_logit(mmK[t], oK[t], three ? 3 : 2, dotq);
        S.logit[t][posK[t]] = lg;
        vmax = fmaxf(vmax, lg);
      }
    }
    // value codes of the low-width regions: issued now so they fly during the next tiles
    {
      const uint8_t* baseV = qaq_tile_codes(v, 1, b, h, tile);
      const QaqVRegions rV = qaq_v_regions(cV[t], D);
      const int nu2 = (cV[t].n32() + 15) >> 4, nu1 = (cV[t].n3 + 15) >> 4;
      if (wave * 4 < nu2) load_dwords<NCG>(baseV + rV.r2 + (uint32_t)min(wave * 4 + g, nu2 - 1) * (4u * D) + (uint32_t)nn * (NCG * 4), vw2[t]);
      if (wave * 4 < nu1) load_dwords<NCG / 2>(baseV + rV.r1 + (uint32_t)min(wave * 4 + g, nu1 - 1) * (2u * D) + (uint32_t)nn * (NCG * 2), vw1[t]);
    }
    // wider classes: loaded when needed (few tokens at the operating points of interest)
    for (int grp = wave; grp * 64 < c.n4; grp += 4) {
      uint32_t w[4][KRec<D, 4>::NDW];
      k_load_group<D, 4>(baseK + rK.r4, c.n4, grp, nn, g, w);
      const v4i cc = k_group<D, 4>(w, S, nn, g);
      const int idx = grp * 64 + lane;
      if (idx < c.n4) {
        const size_t gi = gi0 + n32 + idx;
        Outl<NO2> o; o.load(v, 0, gi, no2);
        const float lg = key_logit(v.mm[0][gi], o, 4, real_of(cc));
        S.logit[t][v.perm[0][gi]] = lg;
        vmax = fmaxf(vmax, lg);
      }
    }
    for (int grp = wave; grp * 64 < c.n8; grp += 4) {
      uint32_t w[4][KRec<D, 8>::NDW];
      k_load_group<D, 8>(baseK + rK.r8, c.n8, grp, nn, g, w);
      const v4i cc = k_group<D, 8>(w, S, nn, g);
      const int idx = grp * 64 + lane;
      if (idx < c.n8) {
        const size_t gi = gi0 + n32 + c.n4 + idx;
        Outl<NO2> o; o.load(v, 0, gi, no2);
        // stored bytes are code - 128
        const float dotq = ((((float)cc[2] * 65536.0f + (float)cc[1] * 256.0f) + (float)cc[0]) + 128.0f * (float)sumqi) * qscale;
        const float lg = key_logit(v.mm[0][gi], o, 8, dotq);
        S.logit[t][v.perm[0][gi]] = lg;
        vmax = fmaxf(vmax, lg);
      }
    }
  }
  // bound on w/p over the chunk: the largest effective value scale
  float smax_l = 0.0f;
#pragma unroll
  for (int t = 0; t < NTC; ++t) {
    if (tid < ntok[t]) {
      const int bits = cV[t].bits_of_slot(tid);
      const float range = h2f((uint16_t)(mmV[t] >> 16)) - h2f((uint16_t)(mmV[t] & 0xffffu));
      smax_l = fmaxf(smax_l, ldexpf(range, bits == 3 ? -2 : -bits));
    }
  }
  {
    const float wm = wave_max(vmax);
    const float sm = wave_max(smax_l);
    if (lane == 0) { S.red[8 + wave] = wm; S.red[12 + wave] = sm; }
  }
  __syncthreads();
  const float M = fmaxf(fmaxf(S.red[8], S.red[9]), fmaxf(S.red[10], S.red[11]));
  const float smax = fmaxf(fmaxf(S.red[12], S.red[13]), fmaxf(S.red[14], S.red[15]));
  int wexp = 0;
  if (smax > 0.0f) (void)frexpf(smax, &wexp);
  const float wscale = smax > 0.0f ? ldexpf(1.0f, wexp - 30) : 0.0f;

  // ---- values: weights of every slot, as digits --------------------------------------------
  float lsum_l = 0.0f, bias_l = 0.0f;
#pragma unroll
  for (int t = 0; t < NTC; ++t) {
    if (ntok[t] <= 0) continue;
    const QaqCounts& c = cV[t];
    const int n32 = c.n32(), first8 = n32 + c.n4;
    const int s = tid;
    const bool live = s < ntok[t];
    float w = 0.0f;
    int bits = 2;
    if (a.scores && live) a.scores[(size_t)bq * a.score_stride + (tile0 + t) * QAQ_TT + tid] = S.logit[t][tid];
    if (live) {
      const float pt = __expf(S.logit[t][posV[t]] - M);
      lsum_l += pt;
      const uint32_t m = mmV[t];
      const float mn = h2f((uint16_t)(m & 0xffffu)), mx = h2f((uint16_t)(m >> 16));
      const float range = mx - mn;
      bits = c.bits_of_slot(s);
      const float scale = ldexpf(range, -bits);
      w = pt * scale;
      bias_l += pt * mn + 0.5f * w;
      const float ctop = (float)((1 << bits) - 1) + 0.5f;
#pragma unroll
      for (int j = 0; j < Outl<NO2>::CAP; ++j) {
        if (j < NO2 && j < no2) {
          const float ov = h2f(oV[t].val[j]);
          const float deq = mn + ((ov >= mx && range > 0.0f) ? ctop : 0.5f) * scale;
          atomicAdd(&S.xcorr[oV[t].idx[j]], pt * (ov - deq));
        }
      }
      if (s >= first8) S.w8[t][s - first8] = w;
    }
    // fixed point in units of 2^(e-30): W = round(w * 2^(30-e)).  A 3-bit code is
    // 2*top + low, so its top plane weighs 2W (at most smax by construction) and its
    // low plane W.  Every entry of the three digit tables is written exactly once (zero
    // where the slot is not in that region), so partial units multiply padding by zero.
    const int W = (live && smax > 0.0f && s < first8) ? (int)rintf(ldexpf(w, 30 - wexp)) : 0;
    const uint32_t dgt = digits4_packed(s < c.n3 ? 2 * W : W);
    const uint32_t d2 = s < n32 ? dgt : 0u;
    S.wl2[t][0][s] = (int8_t)d2; S.wl2[t][1][s] = (int8_t)(d2 >> 8); S.wl2[t][2][s] = (int8_t)(d2 >> 16); S.wl2[t][3][s] = (int8_t)(d2 >> 24);
    const uint32_t d1 = s < c.n3 ? digits4_packed(W) : 0u;
    S.wl1[t][0][s] = (int8_t)d1; S.wl1[t][1][s] = (int8_t)(d1 >> 8); S.wl1[t][2][s] = (int8_t)(d1 >> 16); S.wl1[t][3][s] = (int8_t)(d1 >> 24);
    const int i4 = (s - n32) & (QAQ_TT - 1);
    const uint32_t d4 = (s >= n32 && s < first8) ? dgt : 0u;
    S.wl4[t][0][i4] = (int8_t)d4; S.wl4[t][1][i4] = (int8_t)(d4 >> 8); S.wl4[t][2][i4] = (int8_t)(d4 >> 16); S.wl4[t][3][i4] = (int8_t)(d4 >> 24);
  }
  {
    const float ls = wave_sum(lsum_l);
    const float bs = wave_sum(bias_l);
    if (lane == 0) { S.red[wave] = ls; S.red[4 + wave] = bs; }
  }
  __syncthreads();

  // ---- values: integer contractions, rows 0..3 of the tile = the four digits of w ---------
  v4i cv[NCG];
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) cv[cg] = zero4;
  float a8[4] = {0.f, 0.f, 0.f, 0.f};
  const int uV = wave * 4 + g;
#pragma unroll
  for (int t = 0; t < NTC; ++t) {
    if (ntok[t] <= 0) continue;
    const QaqCounts& c = cV[t];
    const int n32 = c.n32();
    const uint8_t* baseV = qaq_tile_codes(v, 1, b, h, tile0 + t);
    const QaqVRegions rV = qaq_v_regions(c, D);
    if (wave * 64 < n32) {
      const v4i wa = nn < 4 ? *(const v4i*)&S.wl2[t][nn][16 * uV] : zero4;
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) cv[cg] = mma(wa, spread<2>(&vw2[t][cg], 0), cv[cg]);
    }
    if (wave * 64 < c.n3) {
      const v4i wa = nn < 4 ? *(const v4i*)&S.wl1[t][nn][16 * uV] : zero4;
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) cv[cg] = mma(wa, spread<1>(&vw1[t][cg >> 1], cg & 1), cv[cg]);
    }
    for (int blk = wave; blk * 64 < c.n4; blk += 4) {
      const int u = blk * 4 + g;                 // 16 slots = half-units 2u, 2u+1
      const int nhu = (c.n4 + 7) >> 3;
      uint32_t w0[NCG], w1d[NCG];
      load_dwords<NCG>(baseV + rV.r4 + (uint32_t)min(2 * u, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4), w0);
      load_dwords<NCG>(baseV + rV.r4 + (uint32_t)min(2 * u + 1, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4), w1d);
      // slots past the end carry zero digits; a clamped (repeated) half-unit is masked here
      const bool ok0 = 2 * u < nhu, ok1 = 2 * u + 1 < nhu;
      const v4i wa = nn < 4 ? *(const v4i*)&S.wl4[t][nn][16 * u] : zero4;
#pragma unroll
      for (int cg = 0; cg < NCG; ++cg) {
        const uint32_t pr[2] = {ok0 ? w0[cg] : 0u, ok1 ? w1d[cg] : 0u};
        cv[cg] = mma(wa, spread<4>(pr, 0), cv[cg]);
      }
    }
    // 8-bit codes: token-major bytes, plain fp32 multiply-add
    {
      constexpr int LPT8 = D / 4;          // lanes per token
      constexpr int TPW = 64 / LPT8;       // tokens per wavefront pass
      const int sub = lane / LPT8, ch4 = lane % LPT8;
      for (int i8 = wave * TPW + sub; i8 < c.n8; i8 += 4 * TPW) {
        const float w = S.w8[t][i8];
        const uint32_t dw = *(const uint32_t*)(baseV + rV.r8 + (uint32_t)i8 * D + 4 * ch4);
#pragma unroll
        for (int j = 0; j < 4; ++j) a8[j] += w * (float)((dw >> (8 * j)) & 255u);
      }
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
  {
    constexpr int LPT8 = D / 4;
    constexpr int TPW = 64 / LPT8;
    const int sub = lane / LPT8, ch4 = lane % LPT8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float tsum = a8[j];
      if constexpr (TPW == 4) tsum += __shfl_xor(tsum, 16);
      tsum += __shfl_xor(tsum, 32);
      if (sub == 0) S.x8part[wave][4 * ch4 + j] = tsum;
    }
  }
  __syncthreads();
  if (tid < D) {
    const float lsum = (S.red[0] + S.red[1]) + (S.red[2] + S.red[3]);
    const float bias = (S.red[4] + S.red[5]) + (S.red[6] + S.red[7]);
    float x = (S.xpart[0][tid] + S.xpart[1][tid]) + (S.xpart[2][tid] + S.xpart[3][tid]);
    x += (S.x8part[0][tid] + S.x8part[1][tid]) + (S.x8part[2][tid] + S.x8part[3][tid]);
    x += S.xcorr[tid] + bias;
    float* part = v.partial + ((size_t)bq * v.NT + chunk) * (D + 4);
    part[tid] = x;
    if (tid == 0) { part[D] = M; part[D + 1] = lsum; }
  }
}

// Merge the chunks of one (sequence, query head), add the unquantized new token and
// normalise.  Block x = 0 writes the output vector; every block normalises its share of
// the emitted scores (each recomputes the head's max and sum from the per-chunk pairs).
template <int D>
__global__ __launch_bounds__(kThreads) void k_attn_combine(QaqAttnArgs a) {
  __shared__ float red[8];
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bq = blockIdx.y, b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  const int nparts = (ntile + NTC - 1) / NTC;
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
  // per-chunk (max, sum): lanes take chunks round robin, then an all-reduce in the wavefront
  float M = a_new;
  for (int i = lane; i < nparts; i += 64) M = fmaxf(M, part[(size_t)i * (D + 4) + D]);
  M = wave_max(M);
  float lsum = 0.0f;
  for (int i = lane; i < nparts; i += 64)
    lsum += __expf(part[(size_t)i * (D + 4) + D] - M) * part[(size_t)i * (D + 4) + D + 1];
  lsum = wave_sum(lsum);
  float e_new = 0.0f;
  if (a.k_new) { e_new = __expf(a_new - M); lsum += e_new; }
  const float inv = 1.0f / lsum;
  if (blockIdx.x == 0) {
    if (tid < D) {
      float x = 0.0f;
      for (int i = 0; i < nparts; ++i) x += __expf(part[(size_t)i * (D + 4) + D] - M) * part[(size_t)i * (D + 4) + tid];
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

template <int D>
void launch_partial(const QaqAttnArgs& a, dim3 grid, hipStream_t s) {
  if (a.v.no2 == 2) hipLaunchKernelGGL((k_attn_partial<D, 2>), grid, dim3(kThreads), 0, s, a);
  else if (a.v.no2 == 0) hipLaunchKernelGGL((k_attn_partial<D, 0>), grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL((k_attn_partial<D, 8>), grid, dim3(kThreads), 0, s, a);
}

}  // namespace

hipError_t qaq_launch_attention(const QaqAttnArgs& a, hipStream_t s, hipEvent_t* ev) {
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  const int nparts = (ntile + NTC - 1) / NTC;
  const int BQ = a.v.B * a.v.Hq;
  if (ev) (void)hipEventRecord(ev[0], s);
  if (nparts > 0) {
    if (a.v.D == 128) launch_partial<128>(a, dim3(nparts, BQ), s);
    else launch_partial<64>(a, dim3(nparts, BQ), s);
  }
  if (ev) (void)hipEventRecord(ev[1], s);
  const int nblk = a.scores ? (a.len + 4 * kThreads - 1) / (4 * kThreads) : 1;
  dim3 grid(nblk < 1 ? 1 : nblk, BQ);
  if (a.v.D == 128) hipLaunchKernelGGL(k_attn_combine<128>, grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(k_attn_combine<64>, grid, dim3(kThreads), 0, s, a);
  if (ev) (void)hipEventRecord(ev[2], s);
  return hipGetLastError();
}

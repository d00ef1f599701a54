// Decode-step attention over the quantized cache (Section 2.1 attention evaluated on
// the midpoint reconstruction of Section 4.1 with the outlier side store of Section 4.2).
//
// One workgroup handles one (sequence, query head, tile of 256 positions) and writes a
// partial (max, sum, unnormalised output); a second kernel merges the tiles, adds the
// unquantized new token and normalises.
//
// Arithmetic.  The dot products over code fields are exact integer sums:
//   q.K^_t  = min_t * sum(q) + scale_t * (sum_d q_d c_td + sum(q)/2) + outlier terms
//   X_d     = sum_t p_t*min_t + w_t*(c_td + 1/2) + outlier terms,   w_t = p_t*scale_t
// q (per head) and w (per tile) are turned into fixed point with 24 resp. 32 bits,
// split into signed base-256 digits, and each digit plane is contracted with the code
// bytes by 4-way int8 dot instructions; digits are recombined in fp32.  The code
// fields are unpacked to bytes with one shift and one mask per four codes.
#include "qaq_internal.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float h2f(uint16_t b) { return __half2float(__ushort_as_half(b)); }
__device__ __forceinline__ int sdot4(int a, int b, int c) { return __builtin_amdgcn_sdot4(a, b, c, false); }

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

template <int D>
struct AttnLds {
  float qf[D];
  int8_t ql[3][D];
  float logit[QAQ_TT];            // raw logits by position, later p = exp(logit - max)
  int8_t wl2[4][QAQ_TT];          // weight digits per slot of the 2-bit field region
  int8_t wl1[4][QAQ_TT];          // ... of the 1-bit field region
  int8_t wl4[4][QAQ_TT];          // ... of the 4-bit region
  float w8[QAQ_TT];               // fp32 weights of the 8-bit slots
  float xpart[16][D];             // per (wave, lane group) partial outputs
  float x8part[4][4][D];          // per (wave, token lane-group) partials of the 8-bit class
  float xcorr[D];                 // outlier corrections of the output
  float red[8];
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
__device__ __forceinline__ void digits4(int x, int& d0, int& d1, int& d2, int& d3) {
  d0 = ((x + 128) & 255) - 128;
  const int r = (x - d0) >> 8;
  d1 = ((r + 128) & 255) - 128;
  const int r2 = (r - d1) >> 8;
  d2 = ((r2 + 128) & 255) - 128;
  d3 = (r2 - d2) >> 8;
}

// Four byte-spread codes of slice element group v (elements 4v..4v+3).
template <int BF>
__device__ __forceinline__ uint32_t unpack4(const uint32_t* w, int v, int nib) {
  if constexpr (BF == 2) return (w[0] >> (2 * v)) & 0x03030303u;
  else if constexpr (BF == 1) return (w[0] >> (4 * nib + v)) & 0x01010101u;
  else if constexpr (BF == 4) return (w[v >> 1] >> (4 * (v & 1))) & 0x0f0f0f0fu;
  else return w[v];
}

// K side: integer dot products of the query digits with the records of one region.
// Lane (n, g) of a wavefront reads slices g*KS..g*KS+KS-1 of record 16*tg + n; after the
// exchange lane l holds the three digit sums of record  group*64 + l.
template <int D, int BF, class Epilogue>
__device__ __forceinline__ void k_region(const uint8_t* rbase, int n_rec, int wave, int lane,
                                         const int (&qreg)[3][D / 64][4], Epilogue&& epi) {
  constexpr int KS = D / 64;
  constexpr int REC = D * BF / 8;
  constexpr int NDW = (KS * BF / 2) > 0 ? (KS * BF / 2) : 1;   // dwords per lane per record
  const int nn = lane & 15, g = lane >> 4;
  for (int grp = wave; grp * 64 < n_rec; grp += 4) {
    int acc[4][3];
#pragma unroll
    for (int tg = 0; tg < 4; ++tg) {
      acc[tg][0] = acc[tg][1] = acc[tg][2] = 0;
      const int ridx = grp * 64 + 16 * tg + nn;
      if (ridx < n_rec) {
        uint32_t w[NDW];
        const uint8_t* rec = rbase + (size_t)ridx * REC;
        if constexpr (BF == 1 && KS == 1) load_dwords<1>(rec + 4 * (g >> 1), w);
        else load_dwords<NDW>(rec + 4 * NDW * g, w);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            uint32_t u;
            if constexpr (BF == 1) u = unpack4<1>(w, v, KS == 1 ? (g & 1) : ks);
            else u = unpack4<BF>(w + ks * (BF / 2), v, 0);
#pragma unroll
            for (int L = 0; L < 3; ++L) acc[tg][L] = sdot4((int)u, qreg[L][ks][v], acc[tg][L]);
          }
        }
      }
    }
    // sum over the four lane groups, leaving record group*64 + 16*g + n in lane (n, g)
    int z[3];
#pragma unroll
    for (int L = 0; L < 3; ++L) {
      const bool g0 = g & 1, g1 = g & 2;
      const int keepA = g0 ? acc[1][L] : acc[0][L], sendA = g0 ? acc[0][L] : acc[1][L];
      const int keepB = g0 ? acc[3][L] : acc[2][L], sendB = g0 ? acc[2][L] : acc[3][L];
      const int yA = keepA + __shfl_xor(sendA, 16);
      const int yB = keepB + __shfl_xor(sendB, 16);
      const int keep = g1 ? yB : yA, send = g1 ? yA : yB;
      z[L] = keep + __shfl_xor(send, 32);
    }
    const int idx = grp * 64 + lane;
    if (idx < n_rec) epi(idx, z[0], z[1], z[2]);
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

  // ---- query: fp32 copy, fixed-point digits -------------------------------------
  float qv = 0.0f;
  if (tid < D) {
    qv = __half2float(a.q[(size_t)bq * D + tid]);
    S.qf[tid] = qv;
  }
  for (int i = tid; i < 4 * QAQ_TT; i += kThreads) {
    (&S.wl2[0][0])[i] = 0; (&S.wl1[0][0])[i] = 0; (&S.wl4[0][0])[i] = 0;
  }
  if (tid < D) S.xcorr[tid] = 0.0f;
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
  int qreg[3][KS][4];
#pragma unroll
  for (int L = 0; L < 3; ++L)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) qreg[L][ks][vv] = *(const int*)&S.ql[L][64 * ks + 16 * g + 4 * vv];

  // ---- keys: logits -----------------------------------------------------------------
  const int no2 = v.no2;
  {
    const QaqCounts c = qaq_load_counts(v, 0, b, h, tile);
    const QaqKRegions r = qaq_k_regions(c, D);
    const uint8_t* base = qaq_tile_codes(v, 0, b, h, tile);
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    const uint32_t* mmK = v.mm[0] + gi0;
    const uint8_t* permK = v.perm[0] + gi0;
    const uint8_t* oidxK = v.oidx[0] + gi0 * no2;
    const uint16_t* ovalK = v.oval[0] + gi0 * no2;
    const int n32 = c.n32();

    auto finish = [&](int s, int bits, float mult, float real) {
      const uint32_t m = mmK[s];
      const float mn = h2f((uint16_t)(m & 0xffffu)), mx = h2f((uint16_t)(m >> 16));
      const float range = mx - mn;
      const float scale = ldexpf(range, -bits);
      float val = mn * sumq + scale * (mult * real + 0.5f * sumq);
      const float ctop = (float)((1 << bits) - 1) + 0.5f;
      for (int j = 0; j < no2; ++j) {
        const int o = oidxK[s * no2 + j];
        const float ov = h2f(ovalK[s * no2 + j]);
        const float deq = mn + ((ov >= mx && range > 0.0f) ? ctop : 0.5f) * scale;
        val += S.qf[o] * (ov - deq);
      }
      S.logit[permK[s]] = val * inv_sqrt_d;
    };
    auto real_of = [&](int z0, int z1, int z2) {
      return (((float)z2 * 65536.0f + (float)z1 * 256.0f) + (float)z0) * qscale;
    };
    k_region<D, 2>(base + r.r2, n32, wave, lane, qreg, [&](int idx, int z0, int z1, int z2) {
      const bool three = idx < c.n3;
      finish(idx, three ? 3 : 2, three ? 2.0f : 1.0f, real_of(z0, z1, z2));
    });
    k_region<D, 4>(base + r.r4, c.n4, wave, lane, qreg, [&](int idx, int z0, int z1, int z2) {
      finish(n32 + idx, 4, 1.0f, real_of(z0, z1, z2));
    });
    k_region<D, 8>(base + r.r8, c.n8, wave, lane, qreg, [&](int idx, int z0, int z1, int z2) {
      // stored bytes are code - 128
      const float real = ((((float)z2 * 65536.0f + (float)z1 * 256.0f) + (float)z0) + 128.0f * (float)sumqi) * qscale;
      finish(n32 + c.n4 + idx, 8, 1.0f, real);
    });
    __syncthreads();
    k_region<D, 1>(base + r.r1, c.n3, wave, lane, qreg, [&](int idx, int z0, int z1, int z2) {
      const uint32_t m = mmK[idx];
      const float range = h2f((uint16_t)(m >> 16)) - h2f((uint16_t)(m & 0xffffu));
      S.logit[permK[idx]] += ldexpf(range, -3) * real_of(z0, z1, z2) * inv_sqrt_d;
    });
    __syncthreads();
  }

  // ---- softmax inside the tile --------------------------------------------------------
  float lg = tid < n_tok ? S.logit[tid] : -INFINITY;
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
  __syncthreads();

  // ---- values -----------------------------------------------------------------------
  const QaqCounts c = qaq_load_counts(v, 1, b, h, tile);
  const QaqVRegions r = qaq_v_regions(c, D);
  const uint8_t* base = qaq_tile_codes(v, 1, b, h, tile);
  const int n32 = c.n32();
  float w_eff = 0.0f, w1 = 0.0f, bias_l = 0.0f;
  {
    if (tid < n_tok) {
      const int s = tid;
      const size_t gi = qaq_slot_index(v, b, h, tile, s);
      const float pt = S.logit[v.perm[1][gi]];
      const uint32_t m = v.mm[1][gi];
      const float mn = h2f((uint16_t)(m & 0xffffu)), mx = h2f((uint16_t)(m >> 16));
      const float range = mx - mn;
      const int bits = c.bits_of_slot(s);
      const float scale = ldexpf(range, -bits);
      const float w = pt * scale;
      bias_l = pt * mn + 0.5f * w;
      const float ctop = (float)((1 << bits) - 1) + 0.5f;
      for (int j = 0; j < no2; ++j) {
        const int o = v.oidx[1][gi * no2 + j];
        const float ov = h2f(v.oval[1][gi * no2 + j]);
        const float deq = mn + ((ov >= mx && range > 0.0f) ? ctop : 0.5f) * scale;
        atomicAdd(&S.xcorr[o], pt * (ov - deq));
      }
      if (s < c.n3) { w_eff = 2.0f * w; w1 = w; }
      else if (s < n32 + c.n4) w_eff = w;
      else S.w8[s - n32 - c.n4] = w;
    }
    const float wm = wave_max(w_eff);
    const float bs = wave_sum(bias_l);
    if (lane == 0) { S.red[wave] = wm; S.red[4 + wave] = bs; }
  }
  __syncthreads();
  const float wmax = fmaxf(fmaxf(S.red[0], S.red[1]), fmaxf(S.red[2], S.red[3]));
  const float bias = (S.red[4] + S.red[5]) + (S.red[6] + S.red[7]);
  int wexp = 0;
  if (wmax > 0.0f) (void)frexpf(wmax, &wexp);
  const float wscale = wmax > 0.0f ? ldexpf(1.0f, wexp - 30) : 0.0f;
  if (tid < n_tok && wmax > 0.0f) {
    const int s = tid;
    int d0, d1, d2, d3;
    if (s < n32 + c.n4) {
      digits4((int)rintf(ldexpf(w_eff, 30 - wexp)), d0, d1, d2, d3);
      if (s < n32) { S.wl2[0][s] = (int8_t)d0; S.wl2[1][s] = (int8_t)d1; S.wl2[2][s] = (int8_t)d2; S.wl2[3][s] = (int8_t)d3; }
      else { const int i4 = s - n32; S.wl4[0][i4] = (int8_t)d0; S.wl4[1][i4] = (int8_t)d1; S.wl4[2][i4] = (int8_t)d2; S.wl4[3][i4] = (int8_t)d3; }
    }
    if (s < c.n3) {
      digits4((int)rintf(ldexpf(w1, 30 - wexp)), d0, d1, d2, d3);
      S.wl1[0][s] = (int8_t)d0; S.wl1[1][s] = (int8_t)d1; S.wl1[2][s] = (int8_t)d2; S.wl1[3][s] = (int8_t)d3;
    }
  }
  __syncthreads();

  int acc[NCG][4];
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) acc[cg][0] = acc[cg][1] = acc[cg][2] = acc[cg][3] = 0;

  // 2-bit fields: units of 16 slots, lane (n, g) holds channels 16*cg + n of its unit
  for (int u = wave * 4 + g; u * 16 < n32; u += 16) {
    uint32_t w[NCG];
    load_dwords<NCG>(base + r.r2 + (size_t)u * (4 * D) + (size_t)nn * (NCG * 4), w);
    int wr[4][4];
#pragma unroll
    for (int L = 0; L < 4; ++L)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) wr[L][vv] = *(const int*)&S.wl2[L][16 * u + 4 * vv];
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const int uu = (int)unpack4<2>(&w[cg], vv, 0);
#pragma unroll
        for (int L = 0; L < 4; ++L) acc[cg][L] = sdot4(uu, wr[L][vv], acc[cg][L]);
      }
  }
  // 1-bit fields of the 3-bit slots
  for (int u = wave * 4 + g; u * 16 < c.n3; u += 16) {
    uint32_t w[NCG / 2];
    load_dwords<NCG / 2>(base + r.r1 + (size_t)u * (2 * D) + (size_t)nn * (NCG * 2), w);
    int wr[4][4];
#pragma unroll
    for (int L = 0; L < 4; ++L)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) wr[L][vv] = *(const int*)&S.wl1[L][16 * u + 4 * vv];
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const int uu = (int)unpack4<1>(&w[cg >> 1], vv, cg & 1);
#pragma unroll
        for (int L = 0; L < 4; ++L) acc[cg][L] = sdot4(uu, wr[L][vv], acc[cg][L]);
      }
  }
  // 4-bit codes: a 16-token slice is two half-units of 8 tokens
  for (int u = wave * 4 + g; u * 16 < c.n4; u += 16) {
    uint32_t w0[NCG], w1d[NCG];
    load_dwords<NCG>(base + r.r4 + (size_t)(2 * u) * (4 * D) + (size_t)nn * (NCG * 4), w0);
    if ((2 * u + 1) * 8 < c.n4) load_dwords<NCG>(base + r.r4 + (size_t)(2 * u + 1) * (4 * D) + (size_t)nn * (NCG * 4), w1d);
    else {
#pragma unroll
      for (int i = 0; i < NCG; ++i) w1d[i] = 0u;
    }
    int wr[4][4];
#pragma unroll
    for (int L = 0; L < 4; ++L)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) wr[L][vv] = *(const int*)&S.wl4[L][16 * u + 4 * vv];
#pragma unroll
    for (int cg = 0; cg < NCG; ++cg)
#pragma unroll
      for (int vv = 0; vv < 4; ++vv) {
        const uint32_t src = vv < 2 ? w0[cg] : w1d[cg];
        const int uu = (int)((src >> (4 * (vv & 1))) & 0x0f0f0f0fu);
#pragma unroll
        for (int L = 0; L < 4; ++L) acc[cg][L] = sdot4(uu, wr[L][vv], acc[cg][L]);
      }
  }
#pragma unroll
  for (int cg = 0; cg < NCG; ++cg) {
    const float hi = (float)acc[cg][3] * 16777216.0f + (float)acc[cg][2] * 65536.0f;
    const float lo = (float)acc[cg][1] * 256.0f + (float)acc[cg][0];
    S.xpart[wave * 4 + g][16 * cg + nn] = (hi + lo) * wscale;
  }
  // 8-bit codes: token-major bytes, plain fp32 multiply-add
  {
    constexpr int LPT8 = D / 4;          // lanes per token
    constexpr int TPW = 64 / LPT8;       // tokens per wavefront pass
    float a8[4] = {0.f, 0.f, 0.f, 0.f};
    const int sub = lane / LPT8, ch4 = lane % LPT8;
    for (int i8 = wave * TPW + sub; i8 < c.n8; i8 += 4 * TPW) {
      const float w = S.w8[i8];
      const uint32_t dw = *(const uint32_t*)(base + r.r8 + (size_t)i8 * D + 4 * ch4);
#pragma unroll
      for (int j = 0; j < 4; ++j) a8[j] += w * (float)((dw >> (8 * j)) & 255u);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) S.x8part[wave][sub][4 * ch4 + j] = a8[j];
  }
  __syncthreads();
  if (tid < D) {
    float x = 0.0f;
#pragma unroll
    for (int k = 0; k < 16; ++k) x += S.xpart[k][tid];
    constexpr int TPW = 64 / (D / 4);
#pragma unroll
    for (int wv = 0; wv < 4; ++wv)
#pragma unroll
      for (int sb = 0; sb < TPW; ++sb) x += S.x8part[wv][sb][tid];
    x += S.xcorr[tid] + bias;
    float* part = v.partial + ((size_t)bq * v.NT + tile) * (D + 4);
    part[tid] = x;
    if (tid == 0) { part[D] = tmax; part[D + 1] = lsum; }
  }
}

// Merge the tiles of one (sequence, query head), add the unquantized new token, normalise.
template <int D>
__global__ __launch_bounds__(kThreads) void k_attn_combine(QaqAttnArgs a) {
  __shared__ float red[8];
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bq = blockIdx.x, b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
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
  float M = a_new;
  for (int i = 0; i < ntile; ++i) M = fmaxf(M, part[(size_t)i * (D + 4) + D]);
  float lsum = 0.0f, x = 0.0f;
  for (int i = 0; i < ntile; ++i) {
    const float e = __expf(part[(size_t)i * (D + 4) + D] - M);
    lsum += e * part[(size_t)i * (D + 4) + D + 1];
    if (tid < D) x += e * part[(size_t)i * (D + 4) + tid];
  }
  float e_new = 0.0f;
  if (a.k_new) {
    e_new = __expf(a_new - M);
    lsum += e_new;
    if (tid < D) x += e_new * __half2float(a.v_new[((size_t)b * v.Hkv + h) * D + tid]);
  }
  const float inv = 1.0f / lsum;
  if (tid < D) {
    if (a.out_is_fp32) ((float*)a.out)[(size_t)bq * D + tid] = x * inv;
    else ((__half*)a.out)[(size_t)bq * D + tid] = __float2half_rn(x * inv);
  }
  if (a.scores) {
    float* sc = a.scores + (size_t)bq * a.score_stride;
    for (int t = tid; t < a.len; t += kThreads) sc[t] = __expf(sc[t] - M) * inv;
    if (a.k_new && tid == 0) sc[a.len] = e_new * inv;
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
  if (a.v.D == 128) hipLaunchKernelGGL(k_attn_combine<128>, dim3(BQ), dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(k_attn_combine<64>, dim3(BQ), dim3(kThreads), 0, s, a);
  if (ev) (void)hipEventRecord(ev[2], s);
  return hipGetLastError();
}

// Quantization side of libqaq: tile build (append / requantize), width selection,
// canonical export, dequantization, accounting.  Compiled with FP contraction off:
// the fp32 operation order of the encoder and decoder is part of the contract
// (one rounding per operation, round to nearest even).
#include "qaq_internal.h"

namespace {

constexpr int kThreads = 256;

template <int D>
struct TileLds {
  uint8_t stage[QAQ_TT][D];            // one code per (position, channel), at the token's width
  uint32_t mm[QAQ_TT];                 // fp16 min | fp16 max << 16, by position
  uint8_t oidx[QAQ_TT][QAQ_MAX_NO2];   // outlier channels, by position
  uint16_t oval[QAQ_TT][QAQ_MAX_NO2];  // outlier fp16 values
  uint8_t bits_old[QAQ_TT];
  uint8_t bits_new[QAQ_TT];
  uint16_t slot_of_pos[QAQ_TT];
  uint16_t pos_of_slot[QAQ_TT];
  int wave_cnt[4][4];
  int flag;
};

__device__ __forceinline__ float h2f(uint16_t b) { return __half2float(__ushort_as_half(b)); }
__device__ __forceinline__ uint16_t f2h(float f) { return __half_as_ushort(__float2half_rn(f)); }

__device__ __forceinline__ uint32_t rd_field(const uint8_t* base, QaqFieldPos p, uint32_t mask) {
  return (*(const uint32_t*)(base + p.byte_off) >> p.shift) & mask;
}

// Code of (slot, channel d) as stored for this tile side.
template <int D, bool HAS1 = true>
__device__ __forceinline__ uint32_t load_code(int side, const uint8_t* base, const QaqCounts& c, uint32_t r2,
                                              uint32_t r1, uint32_t r4, uint32_t r8, uint32_t r1b, int slot, int d) {
  const int n32 = c.n32();
  if (HAS1 && slot >= c.first1()) {
    const int i1 = slot - c.first1();
    return side == 0 ? rd_field(base, qaq_k_field(r1b, 1, i1, d, D), 1u) : rd_field(base, qaq_v_field(r1b, 1, i1, d, D), 1u);
  }
  if (slot < n32) {
    uint32_t f = side == 0 ? rd_field(base, qaq_k_field(r2, 2, slot, d, D), 3u)
                           : rd_field(base, qaq_v_field(r2, 2, slot, d, D), 3u);
    if (slot < c.n3) {
      uint32_t lo = side == 0 ? rd_field(base, qaq_k_field(r1, 1, slot, d, D), 1u)
                              : rd_field(base, qaq_v_field(r1, 1, slot, d, D), 1u);
      return f * 2u + lo;
    }
    return f;
  }
  if (slot < n32 + c.n4) {
    int i4 = slot - n32;
    return side == 0 ? rd_field(base, qaq_k_field(r4, 4, i4, d, D), 15u)
                     : rd_field(base, qaq_v_field(r4, 4, i4, d, D), 15u);
  }
  int i8 = slot - n32 - c.n4;
  if (side == 0) return rd_field(base, qaq_k_field(r8, 8, i8, d, D), 255u) ^ 0x80u;
  return base[r8 + (uint32_t)i8 * D + d];
}

// Bring a stored tile side into LDS, indexed by position.
template <int D>
__device__ void tile_load(const QaqView& v, int side, int b, int h, int tile, int n_tok, TileLds<D>& L) {
  const int tid = threadIdx.x;
  const QaqCounts c = qaq_load_counts(v, side, b, h, tile, n_tok);
  uint32_t r2, r1, r4, r8, r1b;
  if (side == 0) { QaqKRegions r = qaq_k_regions(c, D); r2 = r.r2; r1 = r.r1; r4 = r.r4; r8 = r.r8; r1b = r.r1b; }
  else { QaqVRegions r = qaq_v_regions(c, D); r2 = r.r2; r1 = r.r1; r4 = r.r4; r8 = r.r8; r1b = r.r1b; }
  if (tid < n_tok) {
    const int s = tid;
    const size_t gi = qaq_slot_index(v, b, h, tile, s);
    const int pos = v.perm[side][gi];
    L.mm[pos] = v.mm[side][gi];
    L.slot_of_pos[pos] = (uint16_t)s;
    L.bits_old[pos] = (uint8_t)c.bits_of_slot(s);
    for (int k = 0; k < v.no2 && !v.csr; ++k) {
      L.oidx[pos][k] = v.oidx[side][gi * v.no2 + k];
      L.oval[pos][k] = v.oval[side][gi * v.no2 + k];
    }
  }
  if (v.csr && tid < n_tok) {       // variable-length side store: by position; unused places of the row = channel 255
    const size_t pi = qaq_slot_index(v, b, h, tile, tid);
    const size_t pool0 = qaq_slot_index(v, b, h, tile, 0) * (size_t)v.no2;
    const int cnt = v.ocnt[side][pi], st = v.ostart[side][pi];
    for (int k = 0; k < v.no2; ++k) {
      L.oidx[tid][k] = k < cnt ? v.oidx[side][pool0 + st + k] : (uint8_t)0xffu;
      L.oval[tid][k] = k < cnt ? v.oval[side][pool0 + st + k] : (uint16_t)0;
    }
  }
  __syncthreads();
  const uint8_t* base = qaq_tile_codes(v, side, b, h, tile);
  for (int e = tid; e < n_tok * D; e += kThreads) {
    const int pos = e / D, d = e % D;
    L.stage[pos][d] = (uint8_t)load_code<D>(side, base, c, r2, r1, r4, r8, r1b, L.slot_of_pos[pos], d);
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------
// Tile build (append / requantize).  Codes travel through LDS as one byte per
// (position, channel); both directions between that staging form and the stored code
// planes work on whole 32-bit words: one AND and one shift move four codes, and the
// token-transposed value planes go through 4x4 byte transposes in registers.
// ---------------------------------------------------------------------------------
template <int D, int MAXO = QAQ_MAX_NO2>   // MAXO: outlier entries held per token (2 in the common one-per-end build)
struct BuildLds {
  static constexpr int SROW = D / 4 + 1;   // dwords per staged row; the odd stride spreads rows over the banks
  uint32_t stage[QAQ_TT * SROW];           // byte d of row pos = code of channel d
  uint32_t mm[QAQ_TT];                     // fp16 min | fp16 max << 16, by position
  uint8_t oidx[QAQ_TT][MAXO];              // outlier channels, by position
  uint16_t oval[QAQ_TT][MAXO];             // outlier fp16 values
  uint8_t bits_old[QAQ_TT];
  uint8_t bits_new[QAQ_TT];
  uint8_t shf[QAQ_TT];                     // by position: low bits a staged code still has to drop (narrowing);
                                           // bit 7: the token keeps its slot and its width (what is stored for it stays valid)
  uint8_t kept[QAQ_TT];                    // by slot: a token stays here
  uint16_t pos_of_slot[QAQ_TT];
  uint16_t slot_of_pos[QAQ_TT];
  uint16_t freeslot[QAQ_TT];               // per class, in slot order: the slots nobody keeps
  uint16_t pos_old[QAQ_TT];                // position of the token that held a slot before
  uint8_t need[QAQ_TT];                    // by position: 1 = the stored code of this cached token is read again
                                           // (it moves), 2 = it is re-encoded from the unquantized copy, 0 = neither
  uint32_t mask2[16];                      // value side, per unit of 16 slots of the 2-bit field region: slots whose
                                           // fields are written (bit i = slot 16u+i)
  uint32_t mask4[32];                      // ... per half-unit of 8 slots of the 4-bit region
  uint32_t mask1b[16];                     // ... per unit of 16 slots of the 1-bit tokens' region
  int wave_cnt[QAQ_NCLASS][4];
  int wave_need[QAQ_NCLASS][4];
  int wave_free[QAQ_NCLASS][4];
  float wave_bound[4];
  float wave_bound2[4];
  int wave_ocnt[4];                        // variable-length side store: entries of the new tokens per wavefront
  int wave_wide[4];                        // widenings asked for, per wavefront
};
constexpr int kKeptFlag = 0x80;

// rows of four bytes <-> columns of four bytes: t[k] byte j = w[j] byte k
__device__ __forceinline__ void transpose4(const uint32_t (&w)[4], uint32_t (&t)[4]) {
  const uint32_t a = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);   // w0.b0 w1.b0 w0.b1 w1.b1
  const uint32_t b = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);   // w0.b2 w1.b2 w0.b3 w1.b3
  const uint32_t c = __builtin_amdgcn_perm(w[3], w[2], 0x05010400u);
  const uint32_t d = __builtin_amdgcn_perm(w[3], w[2], 0x07030602u);
  t[0] = __builtin_amdgcn_perm(c, a, 0x05040100u);
  t[1] = __builtin_amdgcn_perm(c, a, 0x07060302u);
  t[2] = __builtin_amdgcn_perm(d, b, 0x05040100u);
  t[3] = __builtin_amdgcn_perm(d, b, 0x07060302u);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, 0xf, 0xf, false);
}
// Reductions over the four consecutive lanes (one quad) that share a token; every lane
// of the quad ends up with the result.
__device__ __forceinline__ uint32_t quad_umax(uint32_t x) {
  uint32_t y = dpp_u<0xB1>(x); x = x > y ? x : y;      // quad_perm [1,0,3,2]
  y = dpp_u<0x4E>(x); return x > y ? x : y;            // quad_perm [2,3,0,1]
}
__device__ __forceinline__ uint32_t quad_umin(uint32_t x) {
  uint32_t y = dpp_u<0xB1>(x); x = x < y ? x : y;
  y = dpp_u<0x4E>(x); return x < y ? x : y;
}
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Integer image of a float that orders like the float (unsigned compare), maps +0 and -0
// to the same number, and has its low 13 bits clear when the float is an fp16 value: the
// channel number can ride in the low 7 bits, so that "largest value, lowest channel" is a
// single unsigned maximum of key + (127 - channel), and "smallest value, lowest channel"
// a single unsigned minimum of key + channel.
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t b = __float_as_uint(x);
  const uint32_t mag = b & 0x7fffffffu;
  return (int32_t)b < 0 ? 0x80000000u - mag : 0x80000000u + mag;
}
__device__ __forceinline__ float key_value(uint32_t key) {
  key &= ~0x7fu;
  return key >= 0x80000000u ? __uint_as_float(key - 0x80000000u) : __uint_as_float((0x80000000u - key) | 0x80000000u);
}
// The same order on the fp16 bit patterns themselves, two at a time: per 16-bit half,
// 0x8000 + magnitude for a positive number, 0x8000 - magnitude for a negative one (both zeros
// give 0x8000).  Shifted into the upper half of a word such a key leaves 16 low bits for the
// channel number.
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef short ss2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t order_keys_pair(uint32_t two_halves) {
  const us2 b = __builtin_bit_cast(us2, two_halves);
  const us2 sg = __builtin_bit_cast(us2, __builtin_bit_cast(ss2, b) >> (ss2)15);    // 0xffff where negative
  const us2 mag = b & (us2)0x7fffu;
  const us2 t = (mag ^ sg) - sg;                                                      // +-magnitude, two's complement
  return __builtin_bit_cast(uint32_t, (us2)(t + (us2)0x8000u));
}
// value of a key made from order_keys_pair (upper 16 bits; the low bits carry a channel number)
__device__ __forceinline__ float key16_value(uint32_t key) {
  const uint32_t k = key >> 16;
  const uint32_t hb = k >= 0x8000u ? k - 0x8000u : ((0x8000u - k) | 0x8000u);
  return h2f((uint16_t)hb);
}

// ---------------------------------------------------------------------------------
// Encoder for one token vector, run by the four lanes of a quad; lane c holds the 8-channel
// chunks c, c+4, c+8, ... (a quad reads 64 contiguous bytes per load).  Outliers
// (Section 4.2): the n_o largest, then the n_o smallest of the rest, ties to the lower
// channel; [min,max] over what remains; then the midpoint quantizer of Section 4.1:
// code = clamp(floor((x-min)*2^B/range)).
// ---------------------------------------------------------------------------------
template <int D, bool ONE>   // ONE: exactly one outlier per end (the common case) has its own, shorter search
struct TokenEncoder {
  static constexpr int NCH = D / 32;          // 16-byte chunks per lane
  static constexpr int EPL = 8 * NCH;         // elements per lane

  __device__ static __forceinline__ uint32_t half_bits(const uint4 (&raw)[NCH], int i, int e) {
    const uint32_t w = e < 2 ? raw[i].x : e < 4 ? raw[i].y : e < 6 ? raw[i].z : raw[i].w;
    return (w >> (16 * (e & 1))) & 0xffffu;
  }
  __device__ static __forceinline__ int channel(int c, int i, int e) { return 32 * i + 8 * c + e; }

  // fp16 bits of the outlier on channel ch (held by this lane), whose value is `val`
  __device__ static __forceinline__ uint16_t outlier_bits(const uint4 (&raw)[NCH], int c, int ch, float val) {
    uint32_t hv = f2h(val);
    if (val == 0.0f) {   // the key does not keep the sign of a zero: take the stored bits
#pragma unroll
      for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (channel(c, i, e) == ch) hv = half_bits(raw, i, e);
    }
    return (uint16_t)hv;
  }

  // thr_lo, thr_hi: an outlier must lie below thr_lo resp. above thr_hi (+inf, -inf: the count
  // rule, every candidate passes); a side stops at its first candidate that does not, and the
  // rows of the side store are filled from the front, the rest marked unused (channel 255)
  __device__ static __forceinline__ void run(const uint4 (&raw)[NCH], int c, bool fresh, int bits, int n_o, uint32_t* mm_pos,
                                             uint8_t* oidx_row, uint16_t* oval_row, uint32_t* stage_row,
                                             float thr_lo = INFINITY, float thr_hi = -INFINITY) {
    float mn, mx;
    if (fresh) {
      uint32_t key_mx, key_mn;
      if constexpr (ONE) {
        // largest and second largest key, smallest and second smallest key, in one sweep
        uint32_t a1 = 0u, a2 = 0u, b1 = 0xffffffffu, b2 = 0xffffffffu;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t w = e2 == 0 ? raw[i].x : e2 == 1 ? raw[i].y : e2 == 2 ? raw[i].z : raw[i].w;
            const uint32_t kk = order_keys_pair(w);     // keys of elements 2*e2 (low half) and 2*e2+1 (high half)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
              const uint32_t k = hf ? (kk & 0xffff0000u) : (kk << 16);
              const int ch = channel(c, i, 2 * e2 + hf);
              const uint32_t kx = k | (uint32_t)(127 - ch), kn = k | (uint32_t)ch;
              a2 = umed3(a1, a2, kx); a1 = a1 > kx ? a1 : kx;
              b2 = umed3(b1, b2, kn); b1 = b1 < kn ? b1 : kn;
            }
          }
        const uint32_t A1 = quad_umax(a1), A2 = quad_umax(a1 == A1 ? a2 : a1);
        const uint32_t B1 = quad_umin(b1), B2 = quad_umin(b1 == B1 ? b2 : b1);
        const int ch_top = 127 - (int)(A1 & 127u);
        // the smallest of the rest is the overall smallest unless that is the top element
        // itself (all values equal): then it is the runner-up
        const uint32_t Bb = (int)(B1 & 127u) == ch_top ? B2 : B1;
        const int ch_bot = (int)(Bb & 127u);
        if (((ch_top >> 3) & 3) == c) { oidx_row[0] = (uint8_t)ch_top; oval_row[0] = outlier_bits(raw, c, ch_top, key16_value(A1)); }
        if (((ch_bot >> 3) & 3) == c) { oidx_row[1] = (uint8_t)ch_bot; oval_row[1] = outlier_bits(raw, c, ch_bot, key16_value(Bb)); }
        // what remains: its largest value is the runner-up of the maximum search, its smallest
        // the runner-up of the minimum search (equal values make the choice of element moot)
        mx = key16_value(A2); mn = key16_value(B2);
      } else {
        uint32_t kx[EPL], kn[EPL];
#pragma unroll
        for (int i = 0; i < NCH; ++i)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t k = order_key(h2f((uint16_t)half_bits(raw, i, e)));
            kx[8 * i + e] = k + (uint32_t)(127 - channel(c, i, e));
            kn[8 * i + e] = k + (uint32_t)channel(c, i, e);
          }
        int n_rec = 0;
        bool alive = true;
        for (int k = 0; k < 2 * n_o; ++k) {
          const bool top = k < n_o;
          if (k == n_o) alive = true;
          uint32_t m = top ? 0u : 0xffffffffu;
#pragma unroll
          for (int j = 0; j < EPL; ++j) m = top ? (m > kx[j] ? m : kx[j]) : (m < kn[j] ? m : kn[j]);
          const uint32_t M = top ? quad_umax(m) : quad_umin(m);
          const int ch = top ? 127 - (int)(M & 127u) : (int)(M & 127u);
          const float val = key_value(M);
          alive = alive && (top ? val > thr_hi : val < thr_lo);      // the same for the four lanes of the quad
          if (alive) {
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
              const bool dead = top ? kx[j] == M : kn[j] == M;
              if (dead) { kx[j] = 0u; kn[j] = 0xffffffffu; }
            }
            if (((ch >> 3) & 3) == c) { oidx_row[n_rec] = (uint8_t)ch; oval_row[n_rec] = outlier_bits(raw, c, ch, val); }
            ++n_rec;
          }
        }
        if (c == 0)
          for (int k = n_rec; k < 2 * n_o; ++k) { oidx_row[k] = 0xffu; oval_row[k] = 0; }
        uint32_t m1 = 0u, m0 = 0xffffffffu;
#pragma unroll
        for (int j = 0; j < EPL; ++j) { m1 = m1 > kx[j] ? m1 : kx[j]; m0 = m0 < kn[j] ? m0 : kn[j]; }
        key_mx = quad_umax(m1); key_mn = quad_umin(m0);
        mx = key_value(key_mx); mn = key_value(key_mn);
      }
      if (c == 0) *mm_pos = (uint32_t)f2h(mn) | ((uint32_t)f2h(mx) << 16);
    } else {
      const uint32_t m = *mm_pos;
      mn = h2f((uint16_t)(m & 0xffffu));
      mx = h2f((uint16_t)(m >> 16));
    }
    const float range = mx - mn;
    const float levels = (float)(1 << bits);
    const float inv = range > 0.0f ? levels / range : 0.0f;   // an empty range gives code 0 everywhere
    const float top_code = levels - 1.0f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      uint32_t w[2] = {0u, 0u};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float diff = h2f((uint16_t)half_bits(raw, i, e)) - mn;
        const float prod = diff * inv;
        // the byte conversion saturates: a negative product (an outlier below min) gives 0
        w[e >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(fminf(floorf(prod), top_code), e & 3, w[e >> 2]);
      }
      stage_row[2 * (4 * i + c)] = w[0];
      stage_row[2 * (4 * i + c) + 1] = w[1];
    }
  }
};

// Stored code planes of one tile side -> staged bytes (old widths, nothing dropped yet), for
// the cached tokens whose codes are read again (L.need == 1); whole words / units that hold
// none of them are not touched.
template <int D, int MAXO, bool HAS1>
__device__ void unpack_tile(int side, const uint8_t* base, const QaqCounts& c, BuildLds<D, MAXO>& L) {
  constexpr int SROW = BuildLds<D, MAXO>::SROW, NQ = D / 16, KS = D / 64;
  const int tid = threadIdx.x;
  const int n32 = c.n32();
  if (side == 0) {
    const QaqKRegions r = qaq_k_regions(c, D);
    for (int it = tid; it < n32 * NQ; it += kThreads) {
      const int s = it / NQ, q = it % NQ;
      const int pos = L.pos_old[s];
      if (L.need[pos] != 1) continue;
      const bool three = s < c.n3;
      const uint32_t w2 = *(const uint32_t*)(base + r.r2 + 4u * (uint32_t)it);
      uint32_t w1 = 0;
      if (three) w1 = *(const uint32_t*)(base + r.r1 + (uint32_t)s * (D / 8) + 4u * (uint32_t)(q >> 1)) >> (4 * (q & 1));
      uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS)];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        uint32_t code = (w2 >> (2 * v)) & 0x03030303u;
        if (three) code = (code << 1) | ((w1 >> v) & 0x01010101u);
        row[v] = code;
      }
    }
    for (int it = tid; it < c.n4 * (D / 8); it += kThreads) {
      const int i4 = it / (D / 8), jj = it % (D / 8), q = jj >> 1, dw = jj & 1;
      const int pos = L.pos_old[n32 + i4];
      if (L.need[pos] != 1) continue;
      const uint32_t w = *(const uint32_t*)(base + r.r4 + 4u * (uint32_t)it);
      uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS) + 2 * dw];
      row[0] = w & 0x0f0f0f0fu;
      row[1] = (w >> 4) & 0x0f0f0f0fu;
    }
    for (int it = tid; it < c.n8 * (D / 4); it += kThreads) {
      const int i8 = it / (D / 4), jj = it % (D / 4), q = jj >> 2, v = jj & 3;
      const int pos = L.pos_old[n32 + c.n4 + i8];
      if (L.need[pos] != 1) continue;
      const uint32_t w = *(const uint32_t*)(base + r.r8 + 4u * (uint32_t)it);
      L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS) + v] = w ^ 0x80808080u;
    }
    for (int it = tid; HAS1 && it < c.n1 * (D / 32); it += kThreads) {
      const int i1 = it / (D / 32), jj = it % (D / 32);
      const int pos = L.pos_old[c.first1() + i1];
      if (L.need[pos] != 1) continue;
      const uint32_t w = *(const uint32_t*)(base + r.r1b + 4u * (uint32_t)it);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int q = 2 * jj + hh;
        uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS)];
#pragma unroll
        for (int v = 0; v < 4; ++v) row[v] = (w >> (4 * hh + v)) & 0x01010101u;
      }
    }
  }
  // (value side: unpack_moved_v)
}

// Value side: codes of the cached tokens that move, token by token.  The list holds their
// positions (L.freeslot) and the slots they had (L.kept, reused); a work item is (token, four
// channels), and every code is read with the per-element accessor of the layout -- a tile in
// a decode step moves a handful of tokens, far fewer than its units hold.
template <int D, int MAXO, bool HAS1>
__device__ void unpack_moved_v(const uint8_t* base, const QaqCounts& c, int n_moved, BuildLds<D, MAXO>& L) {
  constexpr int SROW = BuildLds<D, MAXO>::SROW;
  const QaqVRegions r = qaq_v_regions(c, D);
  for (int e = threadIdx.x; e < n_moved * (D / 4); e += kThreads) {
    const int m = e / (D / 4), c4 = e % (D / 4);
    const int pos = L.freeslot[m], slot = L.kept[m];
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) w |= load_code<D, HAS1>(1, base, c, r.r2, r.r1, r.r4, r.r8, r.r1b, slot, 4 * c4 + k) << (8 * k);
    L.stage[pos * SROW + c4] = w;
  }
}

// Staged bytes -> stored code planes of one tile side, in the new slot order; codes that
// narrow drop their low bits here (the coarser grid's segments contain the finer one's).
// c0 = the class counts the tile had before (all zero for a tile that did not exist): a
// word whose tokens all keep slot and width, in a region that has not moved, is left alone.
template <int D, int MAXO, bool HAS1>
__device__ void pack_tile(int side, uint8_t* base, const QaqCounts& c, const QaqCounts& c0, const BuildLds<D, MAXO>& L) {
  constexpr int SROW = BuildLds<D, MAXO>::SROW, NQ = D / 16, KS = D / 64;
  const int tid = threadIdx.x;
  const int n32 = c.n32();
  const bool had = c0.total() > 0;
  const bool same32 = had && c0.n32() == n32;
  if (side == 0) {
    const QaqKRegions r = qaq_k_regions(c, D), r0 = qaq_k_regions(c0, D);
    const bool same1 = had && r.r1 == r0.r1;
    const bool same4 = same32 && r.r4 == r0.r4;
    const bool same8 = same4 && c0.n4 == c.n4 && r.r8 == r0.r8;
    for (int it = tid; it < n32 * NQ; it += kThreads) {
      const int s = it / NQ, q = it % NQ;
      const int pos = L.pos_of_slot[s];
      const int f = L.shf[pos];
      if (had && (f & kKeptFlag)) continue;
      const int sh = (f & 7) + (s < c.n3 ? 1 : 0);
      const uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS)];
      uint32_t w = 0;
#pragma unroll
      for (int v = 0; v < 4; ++v) w |= ((row[v] >> sh) & 0x03030303u) << (2 * v);
      *(uint32_t*)(base + r.r2 + 4u * (uint32_t)it) = w;
    }
    for (int it = tid; it < c.n3 * (D / 32); it += kThreads) {
      const int s = it / (D / 32), jj = it % (D / 32);
      const int pos = L.pos_of_slot[s];
      const int f = L.shf[pos];
      if (same1 && (f & kKeptFlag)) continue;
      const int sh = f & 7;
      uint32_t w = 0;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int q = 2 * jj + hh;
        const uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS)];
#pragma unroll
        for (int v = 0; v < 4; ++v) w |= ((row[v] >> sh) & 0x01010101u) << (4 * hh + v);
      }
      *(uint32_t*)(base + r.r1 + 4u * (uint32_t)it) = w;
    }
    for (int it = tid; it < c.n4 * (D / 8); it += kThreads) {
      const int i4 = it / (D / 8), jj = it % (D / 8), q = jj >> 1, dw = jj & 1;
      const int pos = L.pos_of_slot[n32 + i4];
      const int f = L.shf[pos];
      if (same4 && (f & kKeptFlag)) continue;
      const int sh = f & 7;
      const uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS) + 2 * dw];
      *(uint32_t*)(base + r.r4 + 4u * (uint32_t)it) = ((row[0] >> sh) & 0x0f0f0f0fu) | (((row[1] >> sh) & 0x0f0f0f0fu) << 4);
    }
    for (int it = tid; it < c.n8 * NQ; it += kThreads) {        // one slice (16 bytes) per item
      const int i8 = it / NQ, q = it % NQ;
      const int pos = L.pos_of_slot[n32 + c.n4 + i8];
      if (same8 && (L.shf[pos] & kKeptFlag)) continue;
      const uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS)];
      *(uint4*)(base + r.r8 + 16u * (uint32_t)it) =
          make_uint4(row[0] ^ 0x80808080u, row[1] ^ 0x80808080u, row[2] ^ 0x80808080u, row[3] ^ 0x80808080u);
    }
    const bool same1b = same8 && c0.n8 == c.n8;           // then r1b has not moved either
    for (int it = tid; HAS1 && it < c.n1 * (D / 32); it += kThreads) {
      const int i1 = it / (D / 32), jj = it % (D / 32);
      const int pos = L.pos_of_slot[c.first1() + i1];
      const int f = L.shf[pos];
      if (same1b && (f & kKeptFlag)) continue;
      const int sh = f & 7;
      uint32_t w = 0;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int q = 2 * jj + hh;
        const uint32_t* row = &L.stage[pos * SROW + 16 * (q % KS) + 4 * (q / KS)];
#pragma unroll
        for (int v = 0; v < 4; ++v) w |= ((row[v] >> sh) & 0x01010101u) << (4 * hh + v);
      }
      *(uint32_t*)(base + r.r1b + 4u * (uint32_t)it) = w;
    }
    return;
  }
  const QaqVRegions r = qaq_v_regions(c, D), r0 = qaq_v_regions(c0, D);
  const bool same8 = same32 && r.r4 == r0.r4 && c0.n4 == c.n4 && r.r8 == r0.r8;
  // every unit is written (a tile that held nothing; see pack_masked_v for a rebuild)
  for (int it = tid; it < ((n32 + 15) / 16) * (D / 4); it += kThreads) {
    const int u = it / (D / 4), c4 = it % (D / 4), cg = c4 >> 2;
    uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      uint32_t w[4], t[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int s = 16 * u + 4 * v + j;
        w[j] = 0;
        if (s < n32) {
          const int pos = L.pos_of_slot[s];
          w[j] = (L.stage[pos * SROW + c4] >> ((L.shf[pos] & 7) + (s < c.n3 ? 1 : 0))) & 0x03030303u;
        }
      }
      transpose4(w, t);
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] |= t[k] << (2 * v);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      *(uint32_t*)(base + r.r2 + (uint32_t)u * (4 * D) + 4u * (uint32_t)((4 * (c4 & 3) + k) * (D / 16) + cg)) = o[k];
  }
  for (int it = tid; it < ((c.n3 + 15) / 16) * (D / 8); it += kThreads) {
    const int u = it / (D / 8), rest = it % (D / 8), cgp = rest >> 2, n4 = rest & 3;
    uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int c4 = 4 * (2 * cgp + hh) + n4;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        uint32_t w[4], t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int s = 16 * u + 4 * v + j;
          w[j] = 0;
          if (s < c.n3) {
            const int pos = L.pos_of_slot[s];
            w[j] = (L.stage[pos * SROW + c4] >> (L.shf[pos] & 7)) & 0x01010101u;
          }
        }
        transpose4(w, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] |= t[k] << (4 * hh + v);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      *(uint32_t*)(base + r.r1 + (uint32_t)u * (2 * D) + 4u * (uint32_t)((4 * n4 + k) * (D / 32) + cgp)) = o[k];
  }
  for (int it = tid; it < ((c.n4 + 7) / 8) * (D / 4); it += kThreads) {
    const int hu = it / (D / 4), c4 = it % (D / 4), cg = c4 >> 2;
    uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2) {
      uint32_t w[4], t[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i4 = 8 * hu + 4 * g2 + j;
        w[j] = 0;
        if (i4 < c.n4) {
          const int pos = L.pos_of_slot[n32 + i4];
          w[j] = (L.stage[pos * SROW + c4] >> (L.shf[pos] & 7)) & 0x0f0f0f0fu;
        }
      }
      transpose4(w, t);
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] |= t[k] << (4 * g2);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      *(uint32_t*)(base + r.r4 + (uint32_t)hu * (4 * D) + 4u * (uint32_t)((4 * (c4 & 3) + k) * (D / 16) + cg)) = o[k];
  }
  for (int it = tid; it < c.n8 * (D / 16); it += kThreads) {    // 16 bytes per item
    const int i8 = it / (D / 16), dq = 4 * (it % (D / 16));
    const int pos = L.pos_of_slot[n32 + c.n4 + i8];
    if (same8 && (L.shf[pos] & kKeptFlag)) continue;
    const uint32_t* row = &L.stage[pos * SROW + dq];
    *(uint4*)(base + r.r8 + 16u * (uint32_t)it) = make_uint4(row[0], row[1], row[2], row[3]);
  }
  for (int it = tid; HAS1 && it < ((c.n1 + 15) / 16) * (D / 8); it += kThreads) {
    const int u = it / (D / 8), rest = it % (D / 8), cgp = rest >> 2, n4 = rest & 3;
    uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int c4 = 4 * (2 * cgp + hh) + n4;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        uint32_t w[4], t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int i1 = 16 * u + 4 * v + j;
          w[j] = 0;
          if (i1 < c.n1) {
            const int pos = L.pos_of_slot[c.first1() + i1];
            w[j] = (L.stage[pos * SROW + c4] >> (L.shf[pos] & 7)) & 0x01010101u;
          }
        }
        transpose4(w, t);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] |= t[k] << (4 * hh + v);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      *(uint32_t*)(base + r.r1b + (uint32_t)u * (2 * D) + 4u * (uint32_t)((4 * n4 + k) * (D / 32) + cgp)) = o[k];
  }
}

// ---------------------------------------------------------------------------------
// Tile build: append new tokens and / or move cached tokens to other widths, then
// write the tile side back in class order.
// Value side of a rebuild: only the fields of the slots in L.mask2 / L.mask4 are written,
// into the words as they are stored (read-modify-write; a word of a unit that did not exist,
// or whose region has moved, starts from zero -- then the masks hold all its slots).  Fields
// of slots past the end of a region are left as they are: no reader looks at them.
template <int D, int MAXO, bool HAS1>
__device__ void pack_masked_v(uint8_t* base, const QaqCounts& c, const QaqCounts& c0, const BuildLds<D, MAXO>& L) {
  constexpr int SROW = BuildLds<D, MAXO>::SROW;
  const int tid = threadIdx.x;
  const int n32 = c.n32(), n32o = c0.n32();
  const QaqVRegions r = qaq_v_regions(c, D), r0 = qaq_v_regions(c0, D);
  const bool same1 = r.r1 == r0.r1;
  const bool same4 = n32 == n32o && r.r4 == r0.r4;
  const bool same8 = same4 && c0.n4 == c.n4 && r.r8 == r0.r8;
  const int units2_old = (n32o + 15) / 16;
  const int units1_old = same1 ? (c0.n3 + 15) / 16 : 0;
  const int half4_old = same4 ? (c0.n4 + 7) / 8 : 0;
  for (int it = tid; it < ((n32 + 15) / 16) * (D / 4); it += kThreads) {
    const int u = it / (D / 4), c4 = it % (D / 4), cg = c4 >> 2;
    uint32_t m = L.mask2[u];
    if (!m) continue;
    uint32_t* wp = (uint32_t*)(base + r.r2 + (uint32_t)u * (4 * D)) + (4 * (c4 & 3)) * (D / 16) + cg;
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = u < units2_old ? wp[k * (D / 16)] : 0u;
    while (m) {
      const int i = __ffs(m) - 1;
      m &= m - 1;
      const int sl = 16 * u + i;
      const int pos = L.pos_of_slot[sl];
      const uint32_t w = (L.stage[pos * SROW + c4] >> ((L.shf[pos] & 7) + (sl < c.n3 ? 1 : 0))) & 0x03030303u;
      const int bp = 8 * (i & 3) + 2 * (i >> 2);
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(3u << bp)) | (((w >> (8 * k)) & 3u) << bp);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) wp[k * (D / 16)] = o[k];
  }
  for (int it = tid; it < ((c.n3 + 15) / 16) * (D / 8); it += kThreads) {
    const int u = it / (D / 8), rest = it % (D / 8), cgp = rest >> 2, n4 = rest & 3;
    const int in3 = c.n3 - 16 * u;                       // slots of this unit inside the 3-bit class
    uint32_t m = L.mask2[u] & (in3 >= 16 ? 0xffffu : (1u << in3) - 1u);
    if (!m) continue;
    uint32_t* wp = (uint32_t*)(base + r.r1 + (uint32_t)u * (2 * D)) + (4 * n4) * (D / 32) + cgp;
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = u < units1_old ? wp[k * (D / 32)] : 0u;
    while (m) {
      const int i = __ffs(m) - 1;
      m &= m - 1;
      const int pos = L.pos_of_slot[16 * u + i];
      const int sh = L.shf[pos] & 7;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const uint32_t w = (L.stage[pos * SROW + 4 * (2 * cgp + hh) + n4] >> sh) & 0x01010101u;
        const int bp = 8 * (i & 3) + 4 * hh + (i >> 2);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(1u << bp)) | (((w >> (8 * k)) & 1u) << bp);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) wp[k * (D / 32)] = o[k];
  }
  for (int it = tid; it < ((c.n4 + 7) / 8) * (D / 4); it += kThreads) {
    const int hu = it / (D / 4), c4 = it % (D / 4), cg = c4 >> 2;
    uint32_t m = L.mask4[hu];
    if (!m) continue;
    uint32_t* wp = (uint32_t*)(base + r.r4 + (uint32_t)hu * (4 * D)) + (4 * (c4 & 3)) * (D / 16) + cg;
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = hu < half4_old ? wp[k * (D / 16)] : 0u;
    while (m) {
      const int i = __ffs(m) - 1;
      m &= m - 1;
      const int pos = L.pos_of_slot[n32 + 8 * hu + i];
      const uint32_t w = (L.stage[pos * SROW + c4] >> (L.shf[pos] & 7)) & 0x0f0f0f0fu;
      const int bp = 8 * (i & 3) + 4 * (i >> 2);
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(15u << bp)) | (((w >> (8 * k)) & 15u) << bp);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) wp[k * (D / 16)] = o[k];
  }
  for (int it = tid; it < c.n8 * (D / 16); it += kThreads) {    // 16 bytes per item
    const int i8 = it / (D / 16), dq = 4 * (it % (D / 16));
    const int pos = L.pos_of_slot[n32 + c.n4 + i8];
    if (same8 && (L.shf[pos] & kKeptFlag)) continue;
    const uint32_t* row = &L.stage[pos * SROW + dq];
    *(uint4*)(base + r.r8 + 16u * (uint32_t)it) = make_uint4(row[0], row[1], row[2], row[3]);
  }
  const bool same1b = same8 && c0.n8 == c.n8;
  const int units1b_old = same1b ? (c0.n1 + 15) / 16 : 0;
  for (int it = tid; HAS1 && it < ((c.n1 + 15) / 16) * (D / 8); it += kThreads) {
    const int u = it / (D / 8), rest = it % (D / 8), cgp = rest >> 2, n4 = rest & 3;
    uint32_t m = L.mask1b[u];
    if (!m) continue;
    uint32_t* wp = (uint32_t*)(base + r.r1b + (uint32_t)u * (2 * D)) + (4 * n4) * (D / 32) + cgp;
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = u < units1b_old ? wp[k * (D / 32)] : 0u;
    while (m) {
      const int i = __ffs(m) - 1;
      m &= m - 1;
      const int pos = L.pos_of_slot[c.first1() + 16 * u + i];
      const int sh = L.shf[pos] & 7;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const uint32_t w = (L.stage[pos * SROW + 4 * (2 * cgp + hh) + n4] >> sh) & 0x01010101u;
        const int bp = 8 * (i & 3) + 4 * hh + (i >> 2);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(1u << bp)) | (((w >> (8 * k)) & 1u) << bp);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) wp[k * (D / 32)] = o[k];
  }
}

// ---------------------------------------------------------------------------------
// Widenings asked for in a tile side: every wavefront leaves its count in LDS (`per_wave`,
// four entries); after the next barrier add_widenings, called by one thread, adds them to the
// tile side's own counters (kind 0 = refused for want of the unquantized copy, 1 = served).
// A tile side is only ever written by the workgroup that owns it, so no atomics are needed;
// the accounting kernel sums the counters.
__device__ __forceinline__ void note_widenings(int* per_wave, bool wider) {
  const unsigned long long bal = __ballot(wider);
  if ((threadIdx.x & 63) == 0) per_wave[threadIdx.x >> 6] = __popcll(bal);
}
__device__ __forceinline__ void add_widenings(const QaqView& v, size_t tile_side, const int* per_wave, bool served) {
  const int n = per_wave[0] + per_wave[1] + per_wave[2] + per_wave[3];
  if (n) v.refused[tile_side * 2 + (served ? 1 : 0)] += (unsigned int)n;
}

// HAS1: the width set contains 1 (five classes); without it the fifth class costs nothing.
// One tile side (unit bh, tile, side) of a build.
template <int D, bool ONE, bool HAS1>
__device__ __forceinline__ void build_tile(const QaqBuildArgs& a, const int bh, const int tile, const int side) {
  constexpr int MAXO = ONE ? 2 : QAQ_MAX_NO2;
  __shared__ BuildLds<D, MAXO> L;
  constexpr int NC = HAS1 ? QAQ_NCLASS : 4;
  auto bits_at = [](const QaqCounts& c, int s) { return HAS1 ? c.bits_of_slot(s) : c.bits_of_slot4(s); };
  constexpr int SROW = BuildLds<D, MAXO>::SROW;

  const QaqView& v = a.v;
  const bool csr = !ONE && v.csr;     // (the one-per-end build never has the variable-length side store)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = bh / v.Hkv, h = bh % v.Hkv;
  const int t0 = tile * QAQ_TT;
  const int len_before = qaq_seq_len(v, b, a.len_before), len_after = qaq_seq_len(v, b, a.len_after);   // of this sequence
  const int n_before = min(max(len_before - t0, 0), QAQ_TT);
  const int n_after = min(max(len_after - t0, 0), QAQ_TT);
  if (n_after == 0) return;
  const int n_o = v.no2 / 2;

  if (a.mode == 1 && a.newbits[side] == nullptr) return;   // requantize: nothing to do for this side
  // an append, where sequences differ in length: the grid starts at the shortest sequence's open
  // tile, which a longer sequence may have filled already
  if ((a.mode == 0 || a.mode == 3) && n_before == n_after) return;

  // decode-step update, key side: the rule compares a token's range with one threshold per
  // (T, head); the tile keeps, from when it was built, the interval of thresholds for which
  // none of its tokens changes width, so a tile with nothing to do costs one 8-byte load
  if (a.mode == 2 && side == 0 && n_before == n_after && !a.rule.out_bits[0]) {
    const float2 keep = ((const float2*)v.kthr)[qaq_bh(v, b, h) * v.NT + tile];
    const float tau = qaq_tau_k(a.rule, v, b, h);
    if (tau >= keep.x && tau < keep.y) return;
  }

  // cached tokens: everything whose address is known up front is requested in one go (the
  // slot-order metadata, and for a requantize the widths that decide whether the tile is
  // touched at all), so that a rebuild costs two dependent round trips to memory, not three
  uint8_t* base = qaq_tile_codes(v, side, b, h, tile);
  QaqCounts c_old;
  c_old.n3 = c_old.n2 = c_old.n4 = c_old.n8 = c_old.n1 = 0;
  int pos_old = 0;
  uint32_t mm_old = 0;
  uint8_t oi_old[MAXO];
  uint16_t ov_old[MAXO];
  if (n_before > 0) {
    c_old = qaq_load_counts(v, side, b, h, tile, n_before);
    if (!HAS1) c_old.n1 = 0;
    if (tid < n_before) {
      const size_t gi = qaq_slot_index(v, b, h, tile, tid);
      pos_old = v.perm[side][gi];
      mm_old = v.mm[side][gi];
#pragma unroll
      for (int k = 0; k < MAXO; ++k)
        if (k < v.no2 && !csr) { oi_old[k] = v.oidx[side][gi * v.no2 + k]; ov_old[k] = v.oval[side][gi * v.no2 + k]; }
    }
  }
  // decode-step update: the inputs of the width rules that are indexed by position (this
  // step's scores, the window rows) are requested now as well; the value side keeps the window
  // (an append by the rules, mode 3, takes the window as it stands and writes no row)
  float pred = 0.0f;
  if ((a.mode == 2 || (a.mode == 3 && tid >= n_before)) && side == 1 && tid < n_after) {
    const QaqRuleArgs& ru = a.rule;
    const int t = t0 + tid;
    const size_t ring_row = (size_t)v.B * v.Hkv * v.Tmax;
    const size_t ri = qaq_bh(v, b, h) * v.Tmax + t;
    // (the scores row by row, the window's rows at once, in the compact form: the decode-step kernel's
    // form with its variants by row count makes this kernel call its helpers out of line)
    float s = 0.0f;
    if (a.mode == 2)
      for (int g = 0; g < ru.G; ++g) s = fmaxf(s, ru.scores[((size_t)b * v.Hq + (h * ru.G + g)) * ru.score_stride + t]);
    s = qaq_ring_value(v, s);
    pred = qaq_window_max_compact(v, qaq_rows_covering(v, ru.row_len, b, t), ru.new_row, ri, s);
    if (a.mode == 2) qaq_ring_store(v, (size_t)ru.new_row * ring_row + ri, s);
  }
  if (a.mode == 1) {
    // no token of the tile changes: leave it alone
    bool changed = false, wider = false;
    if (tid < n_before) {
      const int oldb = v.tags[side][qaq_slot_index(v, b, h, tile, tid)];
      const int req = a.newbits[side][(size_t)bh * a.len_before + t0 + tid];
      if (req < oldb) changed = true;
      else if (req > oldb) { wider = true; if (a.orig[side]) changed = true; }
    }
    note_widenings(L.wave_wide, wider);
    const bool any = __syncthreads_or(changed ? 1 : 0) != 0;
    if (tid == 0) add_widenings(v, (qaq_bh(v, b, h) * v.NT + tile) * 2 + side, L.wave_wide, a.orig[side] != nullptr);
    if (!any) return;
  }

  // metadata by position
  if (n_before > 0 && tid < n_before) {
    L.mm[pos_old] = mm_old;
    L.pos_of_slot[tid] = (uint16_t)pos_old;
    L.pos_old[tid] = (uint16_t)pos_old;
    L.slot_of_pos[pos_old] = (uint16_t)tid;
    L.bits_old[pos_old] = (uint8_t)bits_at(c_old, tid);
#pragma unroll
    for (int k = 0; k < MAXO; ++k)
      if (k < v.no2 && !csr) { L.oidx[pos_old][k] = oi_old[k]; L.oval[pos_old][k] = ov_old[k]; }
  }
  // variable-length side store: the tile's pool is in position order and a token's entries never
  // move; thread `tid` fetches those of position tid (unused places of its row: channel 255)
  const size_t pool0 = qaq_slot_index(v, b, h, tile, 0) * (size_t)v.no2;
  if (csr && tid < n_before) {
    const size_t pi = qaq_slot_index(v, b, h, tile, tid);
    const int cnt = v.ocnt[side][pi], st = v.ostart[side][pi];
#pragma unroll
    for (int k = 0; k < MAXO; ++k) {
      const bool have = k < cnt;
      L.oidx[tid][k] = have ? v.oidx[side][pool0 + st + k] : (uint8_t)0xffu;
      L.oval[tid][k] = have ? v.oval[side][pool0 + st + k] : (uint16_t)0;
    }
  }
  __syncthreads();

  // decode-step update: widths of the cached positions by the rules; the tile is left alone
  // if none of them moves and the new token is not in it
  auto rule_width = [&](uint32_t m) {
    const QaqRuleArgs& ru = a.rule;
    const float range = h2f((uint16_t)(m >> 16)) - h2f((uint16_t)(m & 0xffffu));
    const float lhs = side == 0 ? range : range * pred;
    const float thr = side == 0 ? qaq_tau_k(ru, v, b, h) : qaq_c_v(ru, v, b);
    int w = ru.bit_set[ru.nbits - 1];
    for (int i = ru.nbits - 1; i >= 0; --i)
      if (lhs <= ldexpf(thr, ru.bit_set[i])) w = ru.bit_set[i];
    return w;
  };
  int req_rule = 0;
  if (a.mode == 2) {
    bool changed = false, wider = false;
    if (tid < n_before) {
      const int oldb = L.bits_old[tid];
      req_rule = rule_width(L.mm[tid]);
      if (a.rule.out_bits[side]) a.rule.out_bits[side][(size_t)bh * a.len_after + t0 + tid] = (uint8_t)req_rule;
      if (req_rule < oldb) changed = true;
      else if (req_rule > oldb) { wider = true; if (a.orig[side]) changed = true; }
    }
    note_widenings(L.wave_wide, wider);
    const bool has_new = len_before >= t0 && len_before < t0 + QAQ_TT;
    const bool any = __syncthreads_or(changed ? 1 : 0) != 0;
    if (tid == 0) add_widenings(v, (qaq_bh(v, b, h) * v.NT + tile) * 2 + side, L.wave_wide, a.orig[side] != nullptr);
    if (!any && !has_new) return;
  }

  // final width of every position; whether it is encoded in this pass (new tokens, and
  // cached tokens that widen from the unquantized copy)
  bool enc = false;
  if (tid < n_after) {
    int nb, drop = 0;
    if (tid < n_before) {
      const int oldb = L.bits_old[tid];
      nb = oldb;
      if (a.mode == 1 || a.mode == 2) {       // appends leave the cached tokens at their widths
        const int req = a.mode == 1 ? (int)a.newbits[side][(size_t)bh * a.len_before + t0 + tid] : req_rule;
        if (req < oldb) { nb = req; drop = oldb - req; }
        else if (req > oldb && a.orig[side]) nb = req;
      }
      enc = nb > oldb;
    } else {
      const int r = t0 + tid - len_before;
      nb = a.newbits[side] ? a.newbits[side][(size_t)bh * a.n_new + r] : a.widest;
      L.bits_old[tid] = (uint8_t)nb;
      enc = true;
    }
    L.bits_new[tid] = (uint8_t)nb;
    L.shf[tid] = (uint8_t)drop;
  }
  // In a tile that has cached tokens the few positions to encode are gathered into a list,
  // so that they fill the encoder's passes densely; a tile with none (most value-side tiles
  // of a decode step without the unquantized copies) goes on after one barrier.
  const bool listed = n_before > 0;
  unsigned long long enc_bal = 0ull;
  if (listed) {
    enc_bal = __ballot(enc);
    if (lane == 0) L.wave_need[0][wave] = __popcll(enc_bal);    // (this array's other use comes two barriers later)
  }
  __syncthreads();

  // encode: a quad of lanes per token, 64 tokens per pass; the rows of the next pass are
  // requested before the current pass is computed
  int n_enc = n_after;
  if (listed) {
    int off = 0;
    for (int w = 0; w < wave; ++w) off += L.wave_need[0][w];
    if (enc) L.freeslot[off + __popcll(enc_bal & ((1ull << lane) - 1ull))] = (uint16_t)tid;
    n_enc = L.wave_need[0][0] + L.wave_need[0][1] + L.wave_need[0][2] + L.wave_need[0][3];
    if (n_enc > 0) __syncthreads();          // uniform: every thread has the same sum
  }
  if (n_enc > 0) {
    typedef TokenEncoder<D, ONE> Enc;
    const float thr_lo = csr ? v.othr[(side * v.Hkv + h) * 2] : INFINITY;
    const float thr_hi = csr ? v.othr[(side * v.Hkv + h) * 2 + 1] : -INFINITY;
    constexpr int TPP = kThreads / 4;     // tokens per pass
    const int NP = (n_enc + TPP - 1) / TPP;
    const int c = tid & 3, gt = tid >> 2;
    auto position = [&](int pass) { const int e = pass * TPP + gt; return listed ? (int)L.freeslot[min(e, QAQ_TT - 1)] : e; };
    auto fetch = [&](int pass, uint4 (&raw)[Enc::NCH]) -> int {   // 0 = nothing to do, 1 = fresh, 2 = widen
      if (pass >= NP || pass * TPP + gt >= n_enc) return 0;
      const int p = position(pass);
      const bool fresh = p >= n_before;
      const __half* src = fresh ? a.newx[side] + ((size_t)bh * a.n_new + (t0 + p - len_before)) * D
                                : a.orig[side] + ((size_t)bh * a.orig_tokens + (t0 + p)) * D;
#pragma unroll
      for (int i = 0; i < Enc::NCH; ++i) {      // read once: streaming loads
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 t = __builtin_nontemporal_load((const u32x4*)src + (4 * i + c));
        raw[i] = make_uint4(t.x, t.y, t.z, t.w);
      }
      if (fresh && a.orig_put[side]) {     // keep the unquantized token for later widening
        uint4* dst = (uint4*)(a.orig_put[side] + ((size_t)bh * a.orig_tokens + (t0 + p)) * D);
#pragma unroll
        for (int i = 0; i < Enc::NCH; ++i) dst[4 * i + c] = raw[i];
      }
      return fresh ? 1 : 2;
    };
    uint4 cur[Enc::NCH], nxt[Enc::NCH];
    int kind = fetch(0, cur);
#pragma unroll 1
    for (int pass = 0; pass < NP; ++pass) {
      const int kind_next = fetch(pass + 1, nxt);
      if (kind) {                          // whole quads drop out together
        const int p = position(pass);
        Enc::run(cur, c, kind == 1, L.bits_new[p], n_o, &L.mm[p], L.oidx[p], L.oval[p], &L.stage[p * SROW], thr_lo, thr_hi);
      }
#pragma unroll
      for (int i = 0; i < Enc::NCH; ++i) cur[i] = nxt[i];
      kind = kind_next;
    }
    __syncthreads();
  }

  // decode-step update, append by the rules: the width of a new token from the range the
  // encoder has just found (it was encoded at the widest width; narrowing drops low bits)
  if ((a.mode == 2 || a.mode == 3) && tid >= n_before && tid < n_after) {
    const int w = rule_width(L.mm[tid]);
    if (a.rule.out_bits[side]) {
      if (a.mode == 2) a.rule.out_bits[side][(size_t)bh * a.len_after + t0 + tid] = (uint8_t)w;
      else a.rule.out_bits[side][(size_t)bh * a.n_new + (t0 + tid - len_before)] = (uint8_t)w;
    }
    L.shf[tid] = (uint8_t)(a.widest - w);
    L.bits_new[tid] = (uint8_t)w;
  }

  // side store of fresh tokens: order by channel
  if (tid >= n_before && tid < n_after && v.no2 > 1) {
    for (int i = 1; i < v.no2; ++i) {
      const uint8_t ki = L.oidx[tid][i];
      const uint16_t vi = L.oval[tid][i];
      int j = i - 1;
      while (j >= 0 && L.oidx[tid][j] > ki) {
        L.oidx[tid][j + 1] = L.oidx[tid][j];
        L.oval[tid][j + 1] = L.oval[tid][j];
        --j;
      }
      L.oidx[tid][j + 1] = ki;
      L.oval[tid][j + 1] = vi;
    }
  }

  // values: what the attention kernel needs as the fixed-point range of a tile -- the largest
  // per-token step range/2^B (a 3-bit code is split into planes, the upper one weighs twice the
  // step) and the largest magnitude an outlier correction (stored value minus reconstruction) can have
  if (side == 1) {
    float bnd = 0.0f;
    if (tid < n_after) {
      const int bits = L.bits_new[tid];
      const float mn = h2f((uint16_t)(L.mm[tid] & 0xffffu)), mx = h2f((uint16_t)(L.mm[tid] >> 16));
      const float range = mx - mn;
      bnd = ldexpf(range, bits == 3 ? -2 : -bits);
      for (int k = 0; k < v.no2; ++k) {
        if (L.oidx[tid][k] == 0xffu) continue;        // (variable-length side store: an unused place)
        const float ov = h2f(L.oval[tid][k]);
        bnd = fmaxf(bnd, fmaxf(fabsf(ov - mx), fabsf(ov - mn)) + range);
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) bnd = fmaxf(bnd, __shfl_xor(bnd, o));
    if (lane == 0) L.wave_bound[wave] = bnd;
  } else {
    // keys: thresholds for which every token keeps its width (Section 4.1 key rule as the
    // comparison range <= threshold * 2^B): a token at width B widens below range / 2^B and
    // narrows from range / 2^B' on, B' the next narrower width; the power-of-two scalings are exact
    float lo = 0.0f, hi = INFINITY;
    if (tid < n_after) {
      const int bits = L.bits_new[tid];
      const float range = h2f((uint16_t)(L.mm[tid] >> 16)) - h2f((uint16_t)(L.mm[tid] & 0xffffu));
      int narrower = 0;
      for (int i = 0; i < a.rule.nbits; ++i)
        if (a.rule.bit_set[i] < bits) narrower = a.rule.bit_set[i];
      if (bits < a.rule.bit_set[a.rule.nbits - 1]) lo = ldexpf(range, -bits);
      if (narrower > 0) hi = ldexpf(range, -narrower);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { lo = fmaxf(lo, __shfl_xor(lo, o)); hi = fminf(hi, __shfl_xor(hi, o)); }
    if (lane == 0) { L.wave_bound[wave] = lo; L.wave_bound2[wave] = hi; }
  }

  // Slots: class by class (3, 2, 4, 8).  A cached token whose class is unchanged and whose
  // old slot still lies in its class's range stays where it is; the others (new tokens, tokens
  // that change class, tokens squeezed out by a moved class boundary) take the remaining
  // slots of their class, in position order.  A freshly built tile thus comes out sorted by
  // position inside each class, and a rebuild moves only as many tokens as it has to -- what
  // is stored for the tokens that stay is not written again.
  const int cls = tid < n_after ? qaq_class_of_bits(L.bits_new[tid]) : -1;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const unsigned long long bal = __ballot(cls == c);
    if (lane == 0) L.wave_cnt[c][wave] = __popcll(bal);
  }
  L.kept[tid] = 0;
  if (tid < 32) L.mask4[tid] = 0;
  if (HAS1 && tid < 16) L.mask1b[tid] = 0;
  __syncthreads();
  QaqCounts cn;
  {
    int n[QAQ_NCLASS];
    n[QC1] = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) n[c] = L.wave_cnt[c][0] + L.wave_cnt[c][1] + L.wave_cnt[c][2] + L.wave_cnt[c][3];
    cn.n3 = n[QC3]; cn.n2 = n[QC2]; cn.n4 = n[QC4]; cn.n8 = n[QC8]; cn.n1 = n[QC1];
  }
  int old_slot = -1;              // cached tokens: the slot held so far
  if (n_before == 0) {
    // nothing cached: a plain stable counting sort (rank inside the wavefront + wavefront offsets)
    int my_rank = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const unsigned long long bal = __ballot(cls == c);
      if (cls == c) my_rank = __popcll(bal & ((1ull << lane) - 1ull));
    }
    if (cls >= 0) {
      int sl = cn.start(cls) + my_rank;
      for (int w = 0; w < wave; ++w) sl += L.wave_cnt[cls][w];
      L.slot_of_pos[tid] = (uint16_t)sl;
      L.pos_of_slot[sl] = (uint16_t)tid;
    }
    __syncthreads();
  } else {
    const bool was_cached = tid < n_before;
    old_slot = was_cached ? (int)L.slot_of_pos[tid] : -1;
    bool keep = false;
    if (was_cached && cls == qaq_class_of_bits(L.bits_old[tid])) {
      const int lo = cn.start(cls);
      keep = old_slot >= lo && old_slot < lo + cn.count(cls);
    }
    if (keep) L.kept[old_slot] = 1;
    __syncthreads();
    // ranks: of the tokens that need a slot (by position), of the free slots (by slot)
    const bool need = cls >= 0 && !keep;
    const int slot_cls = tid < n_after ? qaq_class_of_bits(bits_at(cn, tid)) : -1;   // class owning slot `tid`
    const bool is_free = slot_cls >= 0 && !L.kept[tid];
    int need_rank = 0, free_rank = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const unsigned long long bn = __ballot(need && cls == c);
      const unsigned long long bf = __ballot(is_free && slot_cls == c);
      if (lane == 0) { L.wave_need[c][wave] = __popcll(bn); L.wave_free[c][wave] = __popcll(bf); }
      if (need && cls == c) need_rank = __popcll(bn & ((1ull << lane) - 1ull));
      if (is_free && slot_cls == c) free_rank = __popcll(bf & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    if (is_free) {
      int r = cn.start(slot_cls) + free_rank;
      for (int w = 0; w < wave; ++w) r += L.wave_free[slot_cls][w];
      L.freeslot[r] = (uint16_t)tid;
    }
    __syncthreads();
    if (cls >= 0) {
      int sl = old_slot;
      if (!keep) {
        int r = cn.start(cls) + need_rank;
        for (int w = 0; w < wave; ++w) r += L.wave_need[cls][w];
        sl = L.freeslot[r];
      }
      L.slot_of_pos[tid] = (uint16_t)sl;
      L.pos_of_slot[sl] = (uint16_t)tid;
      if (keep && L.bits_new[tid] == L.bits_old[tid] && was_cached) L.shf[tid] |= kKeptFlag;
    }
    __syncthreads();
  }

  // Which tokens are written again: those that do not keep slot and width, and those whose
  // region starts elsewhere than before.  A cached token among them that does not widen has
  // its stored code read back (the others are left alone); on the value side, where a stored
  // word holds one channel of up to 16 tokens, the slots to write are gathered per unit and
  // the tokens to read back into a list.
  int n_moved = 0;
  {
    const bool had = n_before > 0;
    const int n32 = cn.n32(), n32o = c_old.n32();
    bool same1, same4, same8;
    if (side == 0) {
      const QaqKRegions r = qaq_k_regions(cn, D), r0 = qaq_k_regions(c_old, D);
      same1 = had && r.r1 == r0.r1;
      same4 = had && n32 == n32o && r.r4 == r0.r4;
      same8 = same4 && c_old.n4 == cn.n4 && r.r8 == r0.r8;
    } else {
      const QaqVRegions r = qaq_v_regions(cn, D), r0 = qaq_v_regions(c_old, D);
      same1 = had && r.r1 == r0.r1;
      same4 = had && n32 == n32o && r.r4 == r0.r4;
      same8 = same4 && c_old.n4 == cn.n4 && r.r8 == r0.r8;
    }
    const bool same1b = same8 && c_old.n8 == cn.n8;
    auto written = [&](int pos, int c) {
      return !(L.shf[pos] & kKeptFlag) || (c == QC3 && !same1) || (c == QC4 && !same4) || (c == QC8 && !same8) ||
             (HAS1 && c == QC1 && !same1b);
    };
    if (side == 1 && had) {
      // by slot of the new layout
      const bool wr = tid < n_after && written(L.pos_of_slot[tid], qaq_class_of_bits(bits_at(cn, tid)));
      const unsigned long long bal = __ballot(wr && tid < n32);
      if (lane < 4) L.mask2[4 * wave + lane] = (uint32_t)(bal >> (16 * lane)) & 0xffffu;
      if (wr && tid >= n32 && tid < n32 + cn.n4) atomicOr(&L.mask4[(tid - n32) >> 3], 1u << ((tid - n32) & 7));
      if (HAS1 && wr && tid >= cn.first1()) atomicOr(&L.mask1b[(tid - cn.first1()) >> 4], 1u << ((tid - cn.first1()) & 15));
    }
    // by position
    int nd = 0;
    if (tid < n_before) nd = L.bits_new[tid] > L.bits_old[tid] ? 2 : written(tid, cls) ? 1 : 0;
    if (tid < n_after) L.need[tid] = (uint8_t)nd;
    if (side == 1 && had) {
      const unsigned long long bal = __ballot(nd == 1);
      if (lane == 0) L.wave_cnt[0][wave] = __popcll(bal);
      __syncthreads();
      int off = 0;
      for (int w = 0; w < wave; ++w) off += L.wave_cnt[0][w];
      if (nd == 1) {
        const int k = off + __popcll(bal & ((1ull << lane) - 1ull));
        L.freeslot[k] = (uint16_t)tid;       // position
        L.kept[k] = (uint8_t)old_slot;       // the slot it had (both arrays are free by now)
      }
      n_moved = L.wave_cnt[0][0] + L.wave_cnt[0][1] + L.wave_cnt[0][2] + L.wave_cnt[0][3];
    }
    __syncthreads();
    if (had) {
      if (side == 0) unpack_tile<D, MAXO, HAS1>(side, base, c_old, L);
      else unpack_moved_v<D, MAXO, HAS1>(base, c_old, n_moved, L);
      __syncthreads();
    }
  }

  // metadata in slot order, widths by position, class counts
  if (tid < n_after && !(L.shf[tid] & kKeptFlag)) {
    const int s = L.slot_of_pos[tid];
    const size_t gi = qaq_slot_index(v, b, h, tile, s);
    v.mm[side][gi] = L.mm[tid];
    v.perm[side][gi] = (uint8_t)tid;
    for (int k = 0; k < v.no2 && !csr; ++k) {
      v.oidx[side][gi * v.no2 + k] = L.oidx[tid][k];
      v.oval[side][gi * v.no2 + k] = L.oval[tid][k];
    }
    v.tags[side][qaq_slot_index(v, b, h, tile, tid)] = L.bits_new[tid];
  }
  if (csr && n_after > n_before) {
    // variable-length side store: the new tokens' entries go behind the tile's last one, in
    // position order (a prefix sum of their counts)
    const bool fresh = tid >= n_before && tid < n_after;
    int cnt = 0;
    if (fresh)
      for (int k = 0; k < v.no2; ++k) cnt += L.oidx[tid][k] != 0xffu;
    int inc = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(inc, o);
      if (lane >= o) inc += y;
    }
    if (lane == 63) L.wave_ocnt[wave] = inc;
    __syncthreads();
    int start = inc - cnt;
    for (int w = 0; w < wave; ++w) start += L.wave_ocnt[w];
    if (n_before > 0) {
      const size_t pl = qaq_slot_index(v, b, h, tile, n_before - 1);
      start += (int)v.ostart[side][pl] + (int)v.ocnt[side][pl];
    }
    if (fresh) {
      const size_t pi = qaq_slot_index(v, b, h, tile, tid);
      v.ostart[side][pi] = (uint16_t)start;
      v.ocnt[side][pi] = (uint8_t)cnt;
      for (int k = 0; k < cnt; ++k) {          // the row is sorted by channel, unused places last
        v.oidx[side][pool0 + start + k] = L.oidx[tid][k];
        v.oval[side][pool0 + start + k] = L.oval[tid][k];
      }
    }
  }
  if (tid == 0) {
    uint16_t* cp = v.counts + (((qaq_bh(v, b, h) * v.NT + tile) * 2 + side) * 4);
    cp[QC3] = (uint16_t)cn.n3; cp[QC2] = (uint16_t)cn.n2; cp[QC4] = (uint16_t)cn.n4; cp[QC8] = (uint16_t)cn.n8;
    if (side == 1)
      v.vbound[qaq_bh(v, b, h) * v.NT + tile] = fmaxf(fmaxf(L.wave_bound[0], L.wave_bound[1]), fmaxf(L.wave_bound[2], L.wave_bound[3]));
    else
      ((float2*)v.kthr)[qaq_bh(v, b, h) * v.NT + tile] =
          make_float2(fmaxf(fmaxf(L.wave_bound[0], L.wave_bound[1]), fmaxf(L.wave_bound[2], L.wave_bound[3])),
                      fminf(fminf(L.wave_bound2[0], L.wave_bound2[1]), fminf(L.wave_bound2[2], L.wave_bound2[3])));
  }
  if (side == 1 && n_before > 0) pack_masked_v<D, MAXO, HAS1>(base, cn, c_old, L);
  else pack_tile<D, MAXO, HAS1>(side, base, cn, c_old, L);
}

// Grid (units, tiles, 2 sides) -- heads are the fastest grid dimension: with tiles fastest and a
// tile count that is a multiple of eight, every die would see the same two tile indices of every
// head, which ran 30 % slower.
template <int D, bool ONE, bool HAS1>
__global__ __launch_bounds__(kThreads) void k_build(QaqBuildArgs a) {
  build_tile<D, ONE, HAS1>(a, (int)blockIdx.x, a.tile0 + (int)blockIdx.y, (int)blockIdx.z);
}

// The same for a list of tile sides (a.todo: entries (unit * NT + tile) * 2 + side, a.todo_count of
// them, both in device memory): a one-dimensional grid whose workgroups share out the entries.
template <int D, bool ONE, bool HAS1>
__global__ __launch_bounds__(kThreads) void k_build_listed(QaqBuildArgs a) {
  const uint32_t n = *a.todo_count;
#pragma unroll 1
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t e = a.todo[i];
    build_tile<D, ONE, HAS1>(a, (int)((e >> 1) / (uint32_t)a.v.NT), (int)((e >> 1) % (uint32_t)a.v.NT), (int)(e & 1u));
    __syncthreads();        // the next tile side reuses the staging memory
  }
}

// ---------------------------------------------------------------------------------
// Decode-step update, fast kernel (Section 4.2 "Integration in text generation process": the
// part of a step after the attention).  Same result as build_tile in mode 2, for the common
// configuration (one outlier per end, fixed-length side store, widths within {2,3,4,8}), built
// for what a decode step does to a tile: a few tokens change width, one token is appended to
// the last tile, everything else stays.  A workgroup evaluates the rules for its tile side,
// leaves at once if nothing moves, re-assigns slots so that as few tokens move as possible
// (a token keeps its place inside its region; tiles in which more than kMaxMoved tokens move
// are handed to the general kernel through a list), and carries only the moved tokens' codes
// through LDS.  A fifth of
// the general kernel's LDS and half its registers: eight workgroups per compute unit hide its
// two dependent round trips to memory.
// ---------------------------------------------------------------------------------
constexpr int kMaxMoved = 64;

template <int D>
struct UpdLds {
  static constexpr int SROW = D / 4 + 1;   // dwords per staged row (odd stride: rows spread over the banks)
  float pred[QAQ_TT];                      // value side: predicted score by position
  uint32_t stage[kMaxMoved * SROW];        // codes of the moved tokens at their new width, byte d = channel d
  uint32_t mv_a[kMaxMoved];                // moved list: token (thread) index | new slot << 16
  uint32_t mv_b[kMaxMoved];                // ... old width | new width << 8 | position << 16
  uint32_t mv_mm[kMaxMoved];               // ... fp16 min | max << 16
  uint8_t cls_new[QAQ_TT];                 // by token: class after this step (0xff: no token)
  uint8_t m_of_slot[QAQ_TT];               // by new slot: index in the moved list, 0xff = what is stored stays
  uint8_t freeslot[QAQ_TT];                // per class, in slot order: the slots no token keeps
  uint32_t mask2[16], mask4[32];           // value side: slots to write per unit of 16 (2-bit fields) / half-unit of 8 (4-bit)
  int wave_cnt[4][4], wave_need[4][4], wave_free[4][4];
  int wave_moved[4];
  int wave_wide[4];                        // widenings asked for, per wavefront
  int wave_any[4];                         // a token of the wavefront changes width or arrives
  float wave_bound[4], wave_bound2[4];
  uint32_t new_mm, new_oi, new_ov;         // the appended token: min | max, outlier channels, outlier values
  uint32_t newrow[D / 4];                  // ... its codes at the widest width, byte d = channel d
};

// unsigned wavefront reductions on the data-parallel-primitive path
__device__ __forceinline__ uint32_t wave_umax(uint32_t x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) { const uint32_t y = (uint32_t)__shfl_xor((int)x, o); x = x > y ? x : y; }
  return x;
}
__device__ __forceinline__ uint32_t wave_umin(uint32_t x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) { const uint32_t y = (uint32_t)__shfl_xor((int)x, o); x = x < y ? x : y; }
  return x;
}
__device__ __forceinline__ uint16_t key16_bits(uint32_t key) {     // fp16 bits of a key made by order_keys_pair (upper half)
  const uint32_t k = key >> 16;
  return (uint16_t)(k >= 0x8000u ? k - 0x8000u : ((0x8000u - k) | 0x8000u));
}
__device__ __forceinline__ uint32_t width_mask(int bits) { return 0x01010101u * ((1u << bits) - 1u); }

// Four codes (channels 4*c4 .. 4*c4+3, one per byte) of the token in old slot `slot`, keys.  The
// class only selects addresses, shifts and masks: the loads themselves are unconditional (two, the
// second one repeating the first where the token has no low-bit plane), so that they are in
// flight together.
template <int D>
__device__ __forceinline__ uint32_t k_old_codes(const uint8_t* base, const QaqCounts& c, const QaqKRegions& r, int slot, int c4) {
  constexpr int KS = D / 64;
  const int d = 4 * c4, ks = d / 64, g = (d % 64) / 16, vq = (d % 16) / 4;
  const int q = g * KS + ks;
  const int n32 = c.n32();
  const bool f2 = slot < n32, f3 = slot < c.n3, f4 = !f2 && slot < n32 + c.n4;
  const uint32_t off = f2 ? r.r2 + (uint32_t)slot * (D / 4) + 4u * (uint32_t)q
                     : f4 ? r.r4 + (uint32_t)(slot - n32) * (D / 2) + 4u * (uint32_t)(2 * q + (vq >> 1))
                          : r.r8 + (uint32_t)(slot - n32 - c.n4) * D + 4u * (uint32_t)(4 * q + vq);
  const uint32_t offl = f3 ? r.r1 + (uint32_t)slot * (D / 8) + 4u * (uint32_t)(q >> 1) : off;
  const uint32_t w = *(const uint32_t*)(base + off);
  const uint32_t wl = *(const uint32_t*)(base + offl);
  const int sh = f2 ? 2 * vq : f4 ? 4 * (vq & 1) : 0;
  const uint32_t msk = f2 ? 0x03030303u : f4 ? 0x0f0f0f0fu : 0xffffffffu;
  uint32_t code = ((w >> sh) & msk) ^ (f2 || f4 ? 0u : 0x80808080u);
  if (f3) code = (code << 1) | ((wl >> (4 * (q & 1) + vq)) & 0x01010101u);
  return code;
}

// The same for values (transposed units: one load per channel, and one more per channel for the
// low-bit plane of a 3-bit token; eight unconditional loads, or one for an 8-bit token).
template <int D>
__device__ __forceinline__ uint32_t v_old_codes(const uint8_t* base, const QaqCounts& c, const QaqVRegions& r, int slot, int c4) {
  const int n32 = c.n32();
  const int n0 = 4 * (c4 & 3), cg = c4 >> 2;
  if (slot >= n32 + c.n4) return *(const uint32_t*)(base + r.r8 + (uint32_t)(slot - n32 - c.n4) * D + 4u * (uint32_t)c4);
  const bool f2 = slot < n32, f3 = slot < c.n3;
  const int idx = f2 ? slot : slot - n32;
  const int u = f2 ? idx >> 4 : idx >> 3, i = f2 ? idx & 15 : idx & 7;
  const uint32_t off = (f2 ? r.r2 : r.r4) + (uint32_t)u * (4u * D) + 4u * (uint32_t)(n0 * (D / 16) + cg);
  const int sh = f2 ? 8 * (i & 3) + 2 * (i >> 2) : 8 * (i & 3) + 4 * (i >> 2);
  const uint32_t msk = f2 ? 3u : 15u;
  // low-bit plane of a 3-bit token: word (n, cg / 2) of unit u, bit 8*(i%4) + 4*(cg%2) + i/4
  const uint32_t offl = f3 ? r.r1 + (uint32_t)u * (2u * D) + 4u * (uint32_t)(n0 * (D / 32) + (cg >> 1)) : off;
  const uint32_t stl = f3 ? D / 8 : D / 4;
  uint32_t w[4], l[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) w[k] = *(const uint32_t*)(base + off + (uint32_t)k * (D / 4));
#pragma unroll
  for (int k = 0; k < 4; ++k) l[k] = *(const uint32_t*)(base + offl + (uint32_t)k * stl);
  uint32_t code = 0u;
#pragma unroll
  for (int k = 0; k < 4; ++k) code |= ((w[k] >> sh) & msk) << (8 * k);
  if (f3) {
    const int shl = 8 * (i & 3) + 4 * (cg & 1) + (i >> 2);
    uint32_t low = 0u;
#pragma unroll
    for (int k = 0; k < 4; ++k) low |= ((l[k] >> shl) & 1u) << (8 * k);
    code = (code << 1) | low;
  }
  return code;
}

template <int D>
__global__ __launch_bounds__(kThreads, 8) void k_update(QaqBuildArgs a) {
  __shared__ UpdLds<D> L;
  constexpr int SROW = UpdLds<D>::SROW, NQ = D / 16, KS = D / 64;
  const QaqView& v = a.v;
  const QaqRuleArgs& ru = a.rule;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bh = blockIdx.x, b = bh / v.Hkv, h = bh % v.Hkv;
  // value sides first: nearly every one of them has work (a token's predicted score moves every
  // step), most key sides leave after one load and fill in behind
  const int tile = blockIdx.y, side = 1 - (int)blockIdx.z;
  const int t0 = tile * QAQ_TT;
  const int len_before = qaq_seq_len(v, b, a.len_before), len_after = qaq_seq_len(v, b, a.len_after);   // of this sequence
  const int n_before = min(max(len_before - t0, 0), QAQ_TT);
  const int n_after = min(max(len_after - t0, 0), QAQ_TT);
  if (bh == 0 && tile == 0 && side == 0 && tid == 0) *a.todo_count_next = 0u;
  if (n_after == 0) return;
  const bool has_new = n_after > n_before;           // the appended token is position n_before of this tile
  const size_t tile_id = qaq_bh(v, b, h) * v.NT + tile;
  // keys: the tile recorded, when it was built, the interval of thresholds for which none of its
  // tokens changes width (one 8-byte load decides)
  if (side == 0 && !has_new && !ru.out_bits[0]) {
    const float2 keep = ((const float2*)v.kthr)[tile_id];
    const float tau = qaq_tau_k(ru, v, b, h);
    if (tau >= keep.x && tau < keep.y) return;
  }

  // ---- everything whose address is known up front ------------------------------------------------
  uint8_t* base = qaq_tile_codes(v, side, b, h, tile);
  // (the stored class counts are asked for with the rest and decoded behind the barrier: made wavefront
  // constants on the spot, they would be waited for before any other load is issued)
  const uint2 counts_raw = *(const uint2*)(v.counts + (tile_id * 2 + side) * 4);
  const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
  // thread t is token t: the cached token in old slot t, or (t == n_before) the appended one
  uint32_t mm = 0, oi = 0, ov = 0;
  int pos = tid;
  if (tid < n_before) {
    mm = v.mm[side][gi0 + tid];
    pos = v.perm[side][gi0 + tid];
    oi = *(const uint16_t*)(v.oidx[side] + (gi0 + tid) * 2);
    ov = *(const uint32_t*)(v.oval[side] + (gi0 + tid) * 2);
  }
  if (side == 1 && tid < n_after) {      // thread t as position t: the window (Section 4.2), this step's row stored
    const int t = t0 + tid;
    const size_t ring_row = (size_t)v.B * v.Hkv * v.Tmax;
    const size_t ri = qaq_bh(v, b, h) * v.Tmax + t;
    float s;
    const float pred = qaq_predicted<true>(v, qaq_rows_covering(v, ru.row_len, b, t), ru.new_row, ri, t, ru.scores, (size_t)b * v.Hq + h * ru.G, ru.G, ru.score_stride, &s);
    qaq_ring_store(v, (size_t)ru.new_row * ring_row + ri, s);
    L.pred[tid] = pred;
  }
  L.cls_new[tid] = 0xffu;
  L.m_of_slot[tid] = 0xffu;
  if (tid < 32) L.mask4[tid] = 0u;

  // ---- the appended token: outliers, range, codes at the widest width (Section 4.2 "Outliers",
  // Section 4.1 quantizer), by the last wavefront, two channels per lane -------------------------------
  if (has_new && wave == 3) {
    const bool act = 2 * lane < D;
    const uint32_t* src = (const uint32_t*)(a.newx[side] + (size_t)bh * a.n_new * D);
    const uint32_t w = act ? src[lane] : 0u;
    if (act && a.orig_put[side]) ((uint32_t*)(a.orig_put[side] + ((size_t)bh * a.orig_tokens + len_before) * D))[lane] = w;
    const uint32_t kk = order_keys_pair(w);
    const int ch0 = 2 * lane, ch1 = 2 * lane + 1;
    const uint32_t k0 = kk << 16, k1 = kk & 0xffff0000u;
    // largest value, lowest channel first; then the smallest of the rest, lowest channel first
    const uint32_t A1 = wave_umax(act ? max(k0 | (uint32_t)(127 - ch0), k1 | (uint32_t)(127 - ch1)) : 0u);
    const int ch_top = 127 - (int)(A1 & 127u);
    const uint32_t n0 = act && ch0 != ch_top ? (k0 | (uint32_t)ch0) : 0xffffffffu;
    const uint32_t n1 = act && ch1 != ch_top ? (k1 | (uint32_t)ch1) : 0xffffffffu;
    const uint32_t B1 = wave_umin(min(n0, n1));
    const int ch_bot = (int)(B1 & 127u);
    // [min, max] of what remains
    const bool in0 = act && ch0 != ch_top && ch0 != ch_bot, in1 = act && ch1 != ch_top && ch1 != ch_bot;
    const uint32_t A2 = wave_umax(max(in0 ? k0 : 0u, in1 ? k1 : 0u));
    const uint32_t B2 = wave_umin(min(in0 ? k0 : 0xffffffffu, in1 ? k1 : 0xffffffffu));
    const uint32_t mn_b = key16_bits(B2), mx_b = key16_bits(A2);
    const uint32_t wt = (uint32_t)__shfl((int)w, ch_top >> 1), wb = (uint32_t)__shfl((int)w, ch_bot >> 1);
    const uint32_t v_top = (wt >> (16 * (ch_top & 1))) & 0xffffu, v_bot = (wb >> (16 * (ch_bot & 1))) & 0xffffu;
    const float mn = h2f((uint16_t)mn_b), mx = h2f((uint16_t)mx_b);
    const float range = mx - mn;
    const float levels = (float)(1 << a.widest);
    const float inv = range > 0.0f ? levels / range : 0.0f;
    const float top_code = levels - 1.0f;
    uint32_t cw = 0u;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float diff = h2f((uint16_t)(w >> (16 * e))) - mn;
      const float prod = diff * inv;
      cw = __builtin_amdgcn_cvt_pk_u8_f32(fminf(floorf(prod), top_code), e, cw);
    }
    if (act) ((uint16_t*)L.newrow)[lane] = (uint16_t)cw;
    if (lane == 0) {
      L.new_mm = mn_b | (mx_b << 16);
      const bool top_first = ch_top < ch_bot;                 // the side store is ordered by channel
      L.new_oi = top_first ? ((uint32_t)ch_top | ((uint32_t)ch_bot << 8)) : ((uint32_t)ch_bot | ((uint32_t)ch_top << 8));
      L.new_ov = top_first ? (v_top | (v_bot << 16)) : (v_bot | (v_top << 16));
    }
  }
  __syncthreads();
  QaqCounts c_old;
  c_old.n3 = c_old.n2 = c_old.n4 = c_old.n8 = c_old.n1 = 0;
  if (n_before > 0) {
    const uint32_t c01 = (uint32_t)__builtin_amdgcn_readfirstlane((int)counts_raw.x), c23 = (uint32_t)__builtin_amdgcn_readfirstlane((int)counts_raw.y);
    static_assert(QC3 == 0 && QC2 == 1 && QC4 == 2 && QC8 == 3, "order of the stored counts");
    c_old.n3 = (int)(c01 & 0xffffu); c_old.n2 = (int)(c01 >> 16); c_old.n4 = (int)(c23 & 0xffffu); c_old.n8 = (int)(c23 >> 16);
  }
  const bool is_new = has_new && tid == n_before;
  if (is_new) { mm = L.new_mm; oi = L.new_oi; ov = L.new_ov; pos = n_before; }

  // ---- widths by the rules of Section 4.1 -----------------------------------------------------------
  const float mnf = h2f((uint16_t)(mm & 0xffffu)), mxf = h2f((uint16_t)(mm >> 16));
  const float range = mxf - mnf;
  int ob = 0, nb = 0;
  bool changed = false, wider = false;
  if (tid < n_after) {
    const float lhs = side == 0 ? range : range * L.pred[pos];
    const float thr = side == 0 ? qaq_tau_k(ru, v, b, h) : qaq_c_v(ru, v, b);
    int req = ru.bit_set[ru.nbits - 1];
    for (int i = ru.nbits - 1; i >= 0; --i)
      if (lhs <= ldexpf(thr, ru.bit_set[i])) req = ru.bit_set[i];
    if (ru.out_bits[side]) ru.out_bits[side][(size_t)bh * a.len_after + t0 + pos] = (uint8_t)req;
    if (is_new) {
      ob = a.widest; nb = req; changed = true;       // encoded at the widest width; narrowing drops low bits
    } else {
      ob = c_old.bits_of_slot4(tid);
      nb = ob;
      if (req < ob) nb = req;
      else if (req > ob) { wider = true; if (a.orig[side]) nb = req; }
      changed = nb != ob;
    }
  }
  const bool served = a.orig[side] != nullptr;
  note_widenings(L.wave_wide, wider);
  // ---- new class counts; what the attention kernel and the next step's skip test need of the tile
  // (ahead of the test whether the tile side has work at all, so that one barrier serves both) ------------
  const int cls = tid < n_after ? qaq_class_of_bits(nb) : -1;
  const int ocls = (tid < n_before) ? qaq_class_of_bits(ob) : -1;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const unsigned long long bal = __ballot(cls == c);
    if (lane == 0) L.wave_cnt[c][wave] = __popcll(bal);
  }
  if (tid < n_after) L.cls_new[tid] = (uint8_t)cls;
  if (side == 1) {
    float bnd = 0.0f;
    if (tid < n_after) {
      bnd = ldexpf(range, nb == 3 ? -2 : -nb);
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const float o = h2f((uint16_t)(ov >> (16 * k)));
        bnd = fmaxf(bnd, fmaxf(fabsf(o - mxf), fabsf(o - mnf)) + range);
      }
    }
    bnd = wave_max(bnd);
    if (lane == 0) L.wave_bound[wave] = bnd;
  } else {
    float lo = 0.0f, hi = INFINITY;
    if (tid < n_after) {
      int narrower = 0;
      for (int i = 0; i < ru.nbits; ++i)
        if (ru.bit_set[i] < nb) narrower = ru.bit_set[i];
      if (nb < ru.bit_set[ru.nbits - 1]) lo = ldexpf(range, -nb);
      if (narrower > 0) hi = ldexpf(range, -narrower);
    }
    lo = wave_max(lo); hi = wave_min(hi);
    if (lane == 0) { L.wave_bound[wave] = lo; L.wave_bound2[wave] = hi; }
  }
  // (one ballot per wavefront, one barrier, four flags: the library's workgroup OR is a reduction
  // across lanes and three barriers)
  const unsigned long long bal_changed = __ballot(changed);
  if (lane == 0) L.wave_any[wave] = bal_changed != 0ull ? 1 : 0;
  __syncthreads();
  if (!(L.wave_any[0] | L.wave_any[1] | L.wave_any[2] | L.wave_any[3])) {          // nothing moves and nothing is appended
    if (tid == 0) add_widenings(v, tile_id * 2 + side, L.wave_wide, served);
    return;
  }

  QaqCounts cn;
  cn.n3 = L.wave_cnt[QC3][0] + L.wave_cnt[QC3][1] + L.wave_cnt[QC3][2] + L.wave_cnt[QC3][3];
  cn.n2 = L.wave_cnt[QC2][0] + L.wave_cnt[QC2][1] + L.wave_cnt[QC2][2] + L.wave_cnt[QC2][3];
  cn.n4 = L.wave_cnt[QC4][0] + L.wave_cnt[QC4][1] + L.wave_cnt[QC4][2] + L.wave_cnt[QC4][3];
  cn.n8 = L.wave_cnt[QC8][0] + L.wave_cnt[QC8][1] + L.wave_cnt[QC8][2] + L.wave_cnt[QC8][3];
  cn.n1 = 0;

  // ---- slots.  A token's codes sit at an index inside its class's region (2- and 3-bit tokens: the
  // slot; 4-bit: slot minus the 2/3-bit tokens; 8-bit: minus the 4-bit ones as well).  A cached token
  // that stays in its class keeps that index if the region still reaches it; the others -- tokens that
  // change class, tokens squeezed out, the appended one -- take the free indices of their class in order.
  const int n32o = c_old.n32(), n32n = cn.n32();
  bool mv3, mv4, mv8;       // the region a class alone owns starts elsewhere than before (the 2-bit fields start the tile side)
  if (side == 0) {
    const QaqKRegions r0 = qaq_k_regions(c_old, D), r1 = qaq_k_regions(cn, D);
    mv3 = r0.r1 != r1.r1; mv4 = r0.r4 != r1.r4; mv8 = r0.r8 != r1.r8;
  } else {
    const QaqVRegions r0 = qaq_v_regions(c_old, D), r1 = qaq_v_regions(cn, D);
    mv3 = r0.r1 != r1.r1; mv4 = r0.r4 != r1.r4; mv8 = r0.r8 != r1.r8;
  }
  auto old_index = [&](int c, int slot) { return c == QC4 ? slot - n32o : c == QC8 ? slot - n32o - c_old.n4 : slot; };
  auto new_slot_of = [&](int c, int idx) { return c == QC4 ? n32n + idx : c == QC8 ? n32n + cn.n4 + idx : idx; };
  // (a region whose start moves -- a count before it crossed a multiple of 16 -- keeps nobody: its
  // tokens are written again at the new place like any other moved token)
  auto region_moved = [&](int c) { return (c == QC3 && mv3) || (c == QC4 && mv4) || (c == QC8 && mv8); };
  bool keep = false;
  int my_slot = -1;
  if (ocls >= 0 && cls == ocls && !region_moved(cls)) {
    const int idx = old_index(cls, tid);
    keep = cls == QC3 ? idx < cn.n3 : cls == QC2 ? (idx >= cn.n3 && idx < n32n) : cls == QC4 ? idx < cn.n4 : idx < cn.n8;
    if (keep) my_slot = new_slot_of(cls, idx);
  }
  const bool need = cls >= 0 && !keep;
  // thread s as slot s of the new order: free unless the token that could keep it does
  int slot_cls = -1;
  bool is_free = false;
  if (tid < n_after) {
    slot_cls = qaq_class_of_bits(cn.bits_of_slot4(tid));
    const int idx = slot_cls == QC4 ? tid - n32n : slot_cls == QC8 ? tid - n32n - cn.n4 : tid;
    const int cand = slot_cls == QC4 ? idx + n32o : slot_cls == QC8 ? idx + n32o + c_old.n4 : idx;    // the old slot with that index
    const bool taken = cand < n_before && !region_moved(slot_cls) && qaq_class_of_bits(c_old.bits_of_slot4(cand)) == slot_cls &&
                       L.cls_new[cand] == slot_cls;
    is_free = !taken;
  }
  int need_rank = 0, free_rank = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const unsigned long long bn = __ballot(need && cls == c);
    const unsigned long long bf = __ballot(is_free && slot_cls == c);
    if (lane == 0) { L.wave_need[c][wave] = __popcll(bn); L.wave_free[c][wave] = __popcll(bf); }
    if (need && cls == c) need_rank = __popcll(bn & ((1ull << lane) - 1ull));
    if (is_free && slot_cls == c) free_rank = __popcll(bf & ((1ull << lane) - 1ull));
  }
  const unsigned long long bal_need = __ballot(need);
  if (lane == 0) L.wave_moved[wave] = __popcll(bal_need);
  __syncthreads();
  const int n_moved = L.wave_moved[0] + L.wave_moved[1] + L.wave_moved[2] + L.wave_moved[3];
  if (n_moved > kMaxMoved) {
    // nothing of the cache has been written yet (the window row and the width outputs are the same
    // numbers when the general kernel writes them again)
    if (tid == 0) a.todo[atomicAdd(a.todo_count, 1u)] = (uint32_t)(tile_id * 2 + side);
    return;
  }
  if (is_free) {
    int r = cn.start(slot_cls) + free_rank;
    for (int w = 0; w < wave; ++w) r += L.wave_free[slot_cls][w];
    L.freeslot[r] = (uint8_t)tid;
  }
  __syncthreads();
  int m_idx = -1;
  if (need) {
    int r = cn.start(cls) + need_rank;
    for (int w = 0; w < wave; ++w) r += L.wave_need[cls][w];
    my_slot = L.freeslot[r];
    m_idx = __popcll(bal_need & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) m_idx += L.wave_moved[w];
    L.mv_a[m_idx] = (uint32_t)tid | ((uint32_t)my_slot << 16);
    L.mv_b[m_idx] = (uint32_t)ob | ((uint32_t)nb << 8) | ((uint32_t)pos << 16);
    L.mv_mm[m_idx] = mm;
    L.m_of_slot[my_slot] = (uint8_t)m_idx;
  }
  __syncthreads();

  // ---- value side: which slots of which units are written ---------------------------------------------
  if (side == 1) {
    const bool wr = tid < n_after && L.m_of_slot[tid] != 0xffu;
    const unsigned long long bal = __ballot(wr && tid < n32n);
    if (lane < 4) L.mask2[4 * wave + lane] = (uint32_t)(bal >> (16 * lane)) & 0xffffu;
    if (wr && tid >= n32n && tid < n32n + cn.n4) atomicOr(&L.mask4[(tid - n32n) >> 3], 1u << ((tid - n32n) & 7));
  }

  // ---- codes of the moved tokens -> LDS, at the new width: four channels per work item -----------------
  {
    const QaqKRegions rk0 = qaq_k_regions(c_old, D);
    const QaqVRegions rv0 = qaq_v_regions(c_old, D);
    for (int it = tid; it < n_moved * (D / 4); it += kThreads) {
      const int m = it / (D / 4), c4 = it % (D / 4);
      const uint32_t ma = L.mv_a[m], mb = L.mv_b[m];
      const int tok = (int)(ma & 0xffffu), o_b = (int)(mb & 0xffu), n_b = (int)((mb >> 8) & 0xffu), p = (int)(mb >> 16);
      uint32_t codes;
      if (has_new && tok == n_before) {
        codes = (L.newrow[c4] >> (o_b - n_b)) & width_mask(n_b);
      } else if (n_b > o_b) {
        // wider: from the unquantized copy, with the stored [min, max] (Section 4.2 "Integration")
        const uint2 raw = *(const uint2*)(a.orig[side] + ((size_t)bh * a.orig_tokens + (t0 + p)) * D + 4 * c4);
        const uint32_t m2 = L.mv_mm[m];
        const float mn = h2f((uint16_t)(m2 & 0xffffu)), mx = h2f((uint16_t)(m2 >> 16));
        const float rg = mx - mn;
        const float levels = (float)(1 << n_b);
        const float inv = rg > 0.0f ? levels / rg : 0.0f;
        const float top_code = levels - 1.0f;
        codes = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t hw = e < 2 ? raw.x : raw.y;
          const float diff = h2f((uint16_t)(hw >> (16 * (e & 1)))) - mn;
          const float prod = diff * inv;
          codes = __builtin_amdgcn_cvt_pk_u8_f32(fminf(floorf(prod), top_code), e, codes);
        }
      } else {
        codes = side == 0 ? k_old_codes<D>(base, c_old, rk0, tok, c4) : v_old_codes<D>(base, c_old, rv0, tok, c4);
        codes = (codes >> (o_b - n_b)) & width_mask(n_b);
      }
      L.stage[m * SROW + c4] = codes;
    }
  }
  __syncthreads();      // every read of the old layout is done

  // ---- metadata: tokens whose slot changed (moved ones, and 4-/8-bit tokens behind a moved class
  // border), widths by position, class counts, the tile's bounds --------------------------------------
  if (tid < n_after && (my_slot != tid || need)) {
    const size_t gi = gi0 + my_slot;
    v.mm[side][gi] = mm;
    v.perm[side][gi] = (uint8_t)pos;
    *(uint16_t*)(v.oidx[side] + gi * 2) = (uint16_t)oi;
    *(uint32_t*)(v.oval[side] + gi * 2) = ov;
  }
  if (tid < n_after && (changed || is_new)) v.tags[side][gi0 + pos] = (uint8_t)nb;
  if (tid == 0) {
    uint16_t* cp = v.counts + ((tile_id * 2 + side) * 4);
    cp[QC3] = (uint16_t)cn.n3; cp[QC2] = (uint16_t)cn.n2; cp[QC4] = (uint16_t)cn.n4; cp[QC8] = (uint16_t)cn.n8;
    if (side == 1)
      v.vbound[tile_id] = fmaxf(fmaxf(L.wave_bound[0], L.wave_bound[1]), fmaxf(L.wave_bound[2], L.wave_bound[3]));
    else
      ((float2*)v.kthr)[tile_id] = make_float2(fmaxf(fmaxf(L.wave_bound[0], L.wave_bound[1]), fmaxf(L.wave_bound[2], L.wave_bound[3])),
                                               fminf(fminf(L.wave_bound2[0], L.wave_bound2[1]), fminf(L.wave_bound2[2], L.wave_bound2[3])));
  }
  if (tid == 0) add_widenings(v, tile_id * 2 + side, L.wave_wide, served);

  // ---- codes of the moved tokens -> their new places ----------------------------------------------------
  if (side == 0) {
    const QaqKRegions r = qaq_k_regions(cn, D);
    for (int it = tid; it < n_moved * NQ; it += kThreads) {
      const int m = it / NQ, q = it % NQ;
      const uint32_t ma = L.mv_a[m];
      const int sl = (int)(ma >> 16), n_b = (int)((L.mv_b[m] >> 8) & 0xffu);
      const uint32_t* row = &L.stage[m * SROW + 16 * (q % KS) + 4 * (q / KS)];
      if (n_b <= 3) {
        const int sh = n_b == 3 ? 1 : 0;
        uint32_t w = 0;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) w |= ((row[vq] >> sh) & 0x03030303u) << (2 * vq);
        *(uint32_t*)(base + r.r2 + (uint32_t)sl * (D / 4) + 4u * (uint32_t)q) = w;
        if (n_b == 3 && !(q & 1)) {       // the low bits of slices q and q+1 share a word
          const uint32_t* row1 = &L.stage[m * SROW + 16 * ((q + 1) % KS) + 4 * ((q + 1) / KS)];
          uint32_t w1 = 0;
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) w1 |= ((row[vq] & 0x01010101u) << vq) | ((row1[vq] & 0x01010101u) << (4 + vq));
          *(uint32_t*)(base + r.r1 + (uint32_t)sl * (D / 8) + 4u * (uint32_t)(q >> 1)) = w1;
        }
      } else if (n_b == 4) {
        const uint2 w = make_uint2((row[0] & 0x0f0f0f0fu) | ((row[1] & 0x0f0f0f0fu) << 4), (row[2] & 0x0f0f0f0fu) | ((row[3] & 0x0f0f0f0fu) << 4));
        *(uint2*)(base + r.r4 + (uint32_t)(sl - n32n) * (D / 2) + 8u * (uint32_t)q) = w;
      } else {
        *(uint4*)(base + r.r8 + (uint32_t)(sl - n32n - cn.n4) * D + 16u * (uint32_t)q) =
            make_uint4(row[0] ^ 0x80808080u, row[1] ^ 0x80808080u, row[2] ^ 0x80808080u, row[3] ^ 0x80808080u);
      }
    }
    return;
  }
  // value side: a stored word holds one channel of up to 16 tokens, so the fields of the written slots
  // are put into the words as they are stored (a word of a unit that did not exist starts from zero;
  // so does one whose region moved: then no token was kept in it and every slot of it is written)
  {
    const QaqVRegions r = qaq_v_regions(cn, D), r0 = qaq_v_regions(c_old, D);
    const int units2_old = (n32o + 15) / 16;
    const int units1_old = r.r1 == r0.r1 ? (c_old.n3 + 15) / 16 : 0;
    const int half4_old = r.r4 == r0.r4 ? (c_old.n4 + 7) / 8 : 0;
    for (int it = tid; it < ((n32n + 15) / 16) * (D / 4); it += kThreads) {
      const int u = it / (D / 4), c4 = it % (D / 4), cg = c4 >> 2;
      uint32_t msk = L.mask2[u];
      if (!msk) continue;
      uint32_t* wp = (uint32_t*)(base + r.r2 + (uint32_t)u * (4 * D)) + (4 * (c4 & 3)) * (D / 16) + cg;
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = u < units2_old ? wp[k * (D / 16)] : 0u;
      while (msk) {
        const int i = __ffs(msk) - 1;
        msk &= msk - 1;
        const int sl = 16 * u + i;
        const uint32_t w = (L.stage[L.m_of_slot[sl] * SROW + c4] >> (sl < cn.n3 ? 1 : 0)) & 0x03030303u;
        const int bp = 8 * (i & 3) + 2 * (i >> 2);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(3u << bp)) | (((w >> (8 * k)) & 3u) << bp);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) wp[k * (D / 16)] = o[k];
    }
    for (int it = tid; it < ((cn.n3 + 15) / 16) * (D / 8); it += kThreads) {
      const int u = it / (D / 8), rest = it % (D / 8), cgp = rest >> 2, n4 = rest & 3;
      const int in3 = cn.n3 - 16 * u;                      // slots of this unit inside the 3-bit class
      uint32_t msk = L.mask2[u] & (in3 >= 16 ? 0xffffu : (1u << in3) - 1u);
      if (!msk) continue;
      uint32_t* wp = (uint32_t*)(base + r.r1 + (uint32_t)u * (2 * D)) + (4 * n4) * (D / 32) + cgp;
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = u < units1_old ? wp[k * (D / 32)] : 0u;
      while (msk) {
        const int i = __ffs(msk) - 1;
        msk &= msk - 1;
        const int mi = L.m_of_slot[16 * u + i];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const uint32_t w = L.stage[mi * SROW + 4 * (2 * cgp + hh) + n4] & 0x01010101u;
          const int bp = 8 * (i & 3) + 4 * hh + (i >> 2);
#pragma unroll
          for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(1u << bp)) | (((w >> (8 * k)) & 1u) << bp);
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) wp[k * (D / 32)] = o[k];
    }
    for (int it = tid; it < ((cn.n4 + 7) / 8) * (D / 4); it += kThreads) {
      const int hu = it / (D / 4), c4 = it % (D / 4), cg = c4 >> 2;
      uint32_t msk = L.mask4[hu];
      if (!msk) continue;
      uint32_t* wp = (uint32_t*)(base + r.r4 + (uint32_t)hu * (4 * D)) + (4 * (c4 & 3)) * (D / 16) + cg;
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = hu < half4_old ? wp[k * (D / 16)] : 0u;
      while (msk) {
        const int i = __ffs(msk) - 1;
        msk &= msk - 1;
        const uint32_t w = L.stage[L.m_of_slot[n32n + 8 * hu + i] * SROW + c4] & 0x0f0f0f0fu;
        const int bp = 8 * (i & 3) + 4 * (i >> 2);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (o[k] & ~(15u << bp)) | (((w >> (8 * k)) & 15u) << bp);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) wp[k * (D / 16)] = o[k];
    }
    for (int it = tid; it < n_moved * (D / 16); it += kThreads) {        // 8-bit tokens: token-major bytes, 16 per item
      const int m = it / (D / 16), dq = 4 * (it % (D / 16));
      if (((L.mv_b[m] >> 8) & 0xffu) != 8u) continue;
      const int sl = (int)(L.mv_a[m] >> 16);
      const uint32_t* row = &L.stage[m * SROW + dq];
      *(uint4*)(base + r.r8 + (uint32_t)(sl - n32n - cn.n4) * D + 4u * (uint32_t)dq) = make_uint4(row[0], row[1], row[2], row[3]);
    }
  }
}

// ---------------------------------------------------------------------------------
// Width selection (Section 4.1 bit rules written as comparisons, Section 4.2 window).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_select(QaqSelectArgs a) {
  __shared__ float rk[QAQ_TT], rv[QAQ_TT];
  const QaqView& v = a.v;
  const int tid = threadIdx.x;
  const int tile = blockIdx.x, bh = blockIdx.y, b = bh / v.Hkv, h = bh % v.Hkv;
  const int t0 = tile * QAQ_TT;
  const int n_tok = min(qaq_seq_len(v, b, a.len) - t0, QAQ_TT);
  if (n_tok <= 0) return;
  // all loads first (slot-order ranges, this step's scores, the window rows), one barrier,
  // then the comparisons
  const int t = t0 + tid;
  const size_t ring_row = (size_t)v.B * v.Hkv * v.Tmax;
  const size_t ri = qaq_bh(v, b, h) * v.Tmax + t;
  float pred = 0.0f;
  if (tid < n_tok) {
    const size_t gi = qaq_slot_index(v, b, h, tile, tid);
    const uint32_t mk = v.mm[0][gi], mv = v.mm[1][gi];
    const int pk = v.perm[0][gi], pv = v.perm[1][gi];
    float s;
    const uint32_t covered = qaq_rows_covering(v, a.row_len, b, t);
    pred = a.scores ? qaq_predicted<true>(v, covered, a.new_row, ri, t, a.scores, (size_t)b * v.Hq + h * a.G, a.G, (size_t)a.len, &s)
                    : qaq_predicted<false>(v, covered, -1, ri, t, nullptr, 0, 0, 0, &s);
    if (a.scores) qaq_ring_store(v, (size_t)a.new_row * ring_row + ri, s);
    rk[pk] = h2f((uint16_t)(mk >> 16)) - h2f((uint16_t)(mk & 0xffffu));
    rv[pv] = h2f((uint16_t)(mv >> 16)) - h2f((uint16_t)(mv & 0xffffu));
  }
  __syncthreads();
  if (tid >= n_tok) return;
  const float tau = a.tau_k[v.ragged ? b * v.Hkv + h : h];
  const float c_v = a.c_v[v.ragged ? b : 0];
  const float lhs_v = rv[tid] * pred;
  int bk = a.bit_set[a.nbits - 1], bv = a.bit_set[a.nbits - 1];
  for (int i = a.nbits - 1; i >= 0; --i) {
    const int bb = a.bit_set[i];
    if (rk[tid] <= ldexpf(tau, bb)) bk = bb;
    if (lhs_v <= ldexpf(c_v, bb)) bv = bb;
  }
  a.out_bits[0][(size_t)bh * a.len + t] = (uint8_t)bk;
  a.out_bits[1][(size_t)bh * a.len + t] = (uint8_t)bv;
}

// ---------------------------------------------------------------------------------
// Canonical export and dequantization (tests, export; not on the decode path).
// ---------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void k_export(QaqExportArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  TileLds<D>& L = *reinterpret_cast<TileLds<D>*>(smem_raw);
  const QaqView& v = a.v;
  const int tid = threadIdx.x;
  const int tile = blockIdx.x, bh = blockIdx.y, b = bh / v.Hkv, h = bh % v.Hkv;
  const int t0 = tile * QAQ_TT;
  const int n_tok = min(qaq_seq_len(v, b, a.len) - t0, QAQ_TT);
  if (n_tok <= 0) return;
  tile_load<D>(v, a.side, b, h, tile, n_tok, L);
  if (tid < n_tok) {
    const size_t o = (size_t)bh * a.len + t0 + tid;
    if (a.bits) a.bits[o] = L.bits_old[tid];
    if (a.minmax) { a.minmax[2 * o] = (uint16_t)(L.mm[tid] & 0xffffu); a.minmax[2 * o + 1] = (uint16_t)(L.mm[tid] >> 16); }
    for (int k = 0; k < v.no2; ++k) {
      if (a.oidx) a.oidx[o * v.no2 + k] = L.oidx[tid][k];
      if (a.oval) a.oval[o * v.no2 + k] = L.oval[tid][k];
    }
  }
  if (a.codes) {
    for (int e = tid; e < n_tok * D; e += kThreads) {
      const int pos = e / D, k = e % D;
      const int bits = L.bits_old[pos];
      uint32_t byte = 0;
      if (k < D * bits / 8) {
        for (int j = 0; j < 8; ++j) {
          const int gb = 8 * k + j;
          const int d = gb / bits, bit = gb % bits;
          byte |= ((L.stage[pos][d] >> bit) & 1u) << j;
        }
      }
      a.codes[((size_t)bh * a.len + t0 + pos) * D + k] = (uint8_t)byte;
    }
  }
}

template <int D>
__global__ __launch_bounds__(kThreads) void k_dequant(QaqDequantArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  TileLds<D>& L = *reinterpret_cast<TileLds<D>*>(smem_raw);
  const QaqView& v = a.v;
  const int tid = threadIdx.x;
  const int tile = a.t0 / QAQ_TT + blockIdx.x;
  const int bh = blockIdx.y, b = bh / v.Hkv, h = bh % v.Hkv;
  const int side = blockIdx.z;
  if (a.out[side] == nullptr) return;
  const int t0 = tile * QAQ_TT;
  const int n_tok = min(qaq_seq_len(v, b, a.len) - t0, QAQ_TT);
  if (n_tok <= 0) return;
  tile_load<D>(v, side, b, h, tile, n_tok, L);
  const int nt = a.t1 - a.t0;
  for (int e = tid; e < n_tok * D; e += kThreads) {
    const int pos = e / D, d = e % D;
    const int t = t0 + pos;
    if (t < a.t0 || t >= a.t1) continue;
    const int bits = L.bits_old[pos];
    const float mn = h2f((uint16_t)(L.mm[pos] & 0xffffu)), mx = h2f((uint16_t)(L.mm[pos] >> 16));
    const float range = mx - mn;
    const float scale = ldexpf(range, -bits);
    const float half_c = (float)L.stage[pos][d] + 0.5f;
    const float prod = half_c * scale;
    float xh = prod + mn;
    uint16_t hb = f2h(xh);
    for (int k = 0; k < v.no2; ++k)
      if (L.oidx[pos][k] == d) hb = L.oval[pos][k];
    a.out[side][((size_t)bh * nt + (t - a.t0)) * D + d] = __ushort_as_half(hb);
  }
}

// ---------------------------------------------------------------------------------
// Accounting.
// statbuf: [0..3] hist K (2,3,4,8), [4..7] hist V, [8] layout code bytes, [9] meta bytes,
// [10], [11] 1-bit token-heads K, V, [12], [13] widenings refused / served since the cache was made
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_stats(QaqView v, int len) {
  __shared__ unsigned long long acc[14];
  const int tid = threadIdx.x;
  if (tid < 14) acc[tid] = 0;
  __syncthreads();
  const int ntile = (len + QAQ_TT - 1) / QAQ_TT;
  const long long total = (long long)v.B * v.Hkv * ntile * 2;
  unsigned long long loc[14] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  for (long long i = (long long)blockIdx.x * kThreads + tid; i < total; i += (long long)gridDim.x * kThreads) {
    const int side = (int)(i & 1);
    const long long j = i >> 1;
    const int tile = (int)(j % ntile);
    const int bh = (int)(j / ntile);
    const int n_tok = min(qaq_seq_len(v, bh / v.Hkv, len) - tile * QAQ_TT, QAQ_TT);
    if (n_tok <= 0) continue;      // past the end of a shorter sequence
    const QaqCounts c = qaq_load_counts(v, side, bh / v.Hkv, bh % v.Hkv, tile, n_tok);
    loc[side * 4 + 0] += c.n2; loc[side * 4 + 1] += c.n3; loc[side * 4 + 2] += c.n4; loc[side * 4 + 3] += c.n8;
    loc[10 + side] += c.n1;

    // bytes a scan reads: key records one by one, value planes in whole units
    loc[8] += side == 0 ? (unsigned long long)c.n32() * (v.D / 4) + (c.n3 + c.n1) * (v.D / 8) + c.n4 * (v.D / 2) + c.n8 * v.D
                        : qaq_v_regions(c, v.D).end;
    if (!v.csr) loc[9] += (unsigned long long)c.total() * (4 + 1 + 3 * v.no2);
    else {   // min/max, order byte, (offset, count), and the entries the tile's pool holds
      const size_t pl = qaq_slot_index(v, bh / v.Hkv, bh % v.Hkv, tile, c.total() - 1);
      loc[9] += (unsigned long long)c.total() * (4 + 1 + 3) + 3ull * ((unsigned)v.ostart[side][pl] + (unsigned)v.ocnt[side][pl]);
    }
  }
  // widenings: every tile side the cache has room for (a cache that was reset keeps its history)
  const long long sides = (long long)v.B * v.Hkv * v.NT * 2;
  for (long long i = (long long)blockIdx.x * kThreads + tid; i < sides; i += (long long)gridDim.x * kThreads) {
    loc[12] += v.refused[2 * i]; loc[13] += v.refused[2 * i + 1];
  }
  for (int k = 0; k < 14; ++k) if (loc[k]) atomicAdd(&acc[k], loc[k]);
  __syncthreads();
  if (tid < 14 && acc[tid]) atomicAdd((unsigned long long*)&v.statbuf[tid], acc[tid]);
}

__global__ void k_init(QaqView v) {
  const size_t n = (size_t)v.B * v.Hkv * v.NT * 2 * 4;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) v.counts[i] = 0;
  if (blockIdx.x == 0 && threadIdx.x < 32) v.statbuf[threadIdx.x] = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < (size_t)v.B * v.Hkv * v.NT * 4; i += (size_t)gridDim.x * blockDim.x) v.refused[i] = 0;
  if (blockIdx.x == 0 && threadIdx.x < 2) v.todo_count[threadIdx.x] = 0;
}

__global__ void k_clear_stats(QaqView v) {
  if (threadIdx.x < 32) v.statbuf[threadIdx.x] = 0;
}

}  // namespace

hipError_t qaq_launch_init(const QaqView& v, hipStream_t s) {
  hipLaunchKernelGGL(k_init, dim3(64), dim3(256), 0, s, v);
  return hipGetLastError();
}

hipError_t qaq_launch_build(const QaqBuildArgs& a, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  dim3 grid(a.v.B * a.v.Hkv, ntiles, 2);
  const bool one = a.v.no2 == 2 && !a.v.csr;      // (the one-per-end search has no threshold test)
  if (a.v.D == 128) {
    if (a.v.has1) {
      if (one) hipLaunchKernelGGL((k_build<128, true, true>), grid, dim3(kThreads), 0, s, a);
      else hipLaunchKernelGGL((k_build<128, false, true>), grid, dim3(kThreads), 0, s, a);
    } else {
      if (one) hipLaunchKernelGGL((k_build<128, true, false>), grid, dim3(kThreads), 0, s, a);
      else hipLaunchKernelGGL((k_build<128, false, false>), grid, dim3(kThreads), 0, s, a);
    }
  } else {
    if (a.v.has1) {
      if (one) hipLaunchKernelGGL((k_build<64, true, true>), grid, dim3(kThreads), 0, s, a);
      else hipLaunchKernelGGL((k_build<64, false, true>), grid, dim3(kThreads), 0, s, a);
    } else {
      if (one) hipLaunchKernelGGL((k_build<64, true, false>), grid, dim3(kThreads), 0, s, a);
      else hipLaunchKernelGGL((k_build<64, false, false>), grid, dim3(kThreads), 0, s, a);
    }
  }
  return hipGetLastError();
}

hipError_t qaq_launch_update(const QaqBuildArgs& a_in, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  QaqBuildArgs a = a_in;
  const bool fast = a.mode == 2 && a.v.no2 == 2 && !a.v.csr && !a.v.has1 && a.todo && a.todo_count && a.todo_count_next;
  if (!fast) {
    a.todo = nullptr;
    return qaq_launch_build(a, ntiles, s);
  }
  const dim3 grid(a.v.B * a.v.Hkv, ntiles, 2);
  if (a.v.D == 128) hipLaunchKernelGGL(k_update<128>, grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(k_update<64>, grid, dim3(kThreads), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the tile sides the fast kernel handed over (their number is only known on the device)
  const long long sides = (long long)a.v.B * a.v.Hkv * ntiles * 2;
  const dim3 grid2((unsigned)(sides < 512 ? sides : 512));
  if (a.v.D == 128) hipLaunchKernelGGL((k_build_listed<128, true, false>), grid2, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL((k_build_listed<64, true, false>), grid2, dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t qaq_launch_select(const QaqSelectArgs& a, hipStream_t s) {
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  if (ntile <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_select, dim3(ntile, a.v.B * a.v.Hkv), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t qaq_launch_export(const QaqExportArgs& a, hipStream_t s) {
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  if (ntile <= 0) return hipSuccess;
  dim3 grid(ntile, a.v.B * a.v.Hkv);
  if (a.v.D == 128) hipLaunchKernelGGL(k_export<128>, grid, dim3(kThreads), sizeof(TileLds<128>), s, a);
  else hipLaunchKernelGGL(k_export<64>, grid, dim3(kThreads), sizeof(TileLds<64>), s, a);
  return hipGetLastError();
}

hipError_t qaq_launch_dequant(const QaqDequantArgs& a, hipStream_t s) {
  if (a.t1 <= a.t0) return hipSuccess;
  const int tile_lo = a.t0 / QAQ_TT, tile_hi = (a.t1 - 1) / QAQ_TT;
  dim3 grid(tile_hi - tile_lo + 1, a.v.B * a.v.Hkv, 2);
  if (a.v.D == 128) hipLaunchKernelGGL(k_dequant<128>, grid, dim3(kThreads), sizeof(TileLds<128>), s, a);
  else hipLaunchKernelGGL(k_dequant<64>, grid, dim3(kThreads), sizeof(TileLds<64>), s, a);
  return hipGetLastError();
}

hipError_t qaq_launch_stats(const QaqView& v, int len, hipStream_t s) {
  hipLaunchKernelGGL(k_clear_stats, dim3(1), dim3(64), 0, s, v);
  hipLaunchKernelGGL(k_stats, dim3(64), dim3(kThreads), 0, s, v, len);
  return hipGetLastError();
}

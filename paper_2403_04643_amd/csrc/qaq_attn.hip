// Decode-step attention over the quantized cache (Section 2.1 attention evaluated on
// the midpoint reconstruction of Section 4.1 with the outlier side store of Section 4.2).
//
// k_attn_tile scans the cache: the 256-position tiles of a (sequence, query head) are cut
// into parts of consecutive tiles; a part is 256 threads that compute logits, a softmax with
// a running max and sum over their tiles and the unnormalised output, with the next tile's
// loads in flight while the current tile is computed.  Where a head has at most four parts
// they are the 256-thread groups of one workgroup, which merges them in LDS, adds the
// unquantized new token and writes output and normalised scores itself (one kernel per
// call).  Otherwise every part is a workgroup of its own, writes a partial (max, sum, X), and
// k_attn_combine merges the parts, adds the new token and normalises the scores.
//
// Arithmetic.  With per-token scale_t = range_t / 2^B and codes c_td,
//   q.K^_t  = min_t * sum(q) + scale_t * (sum_d q_d c_td + sum(q)/2) + outlier terms
//   X_d     = sum_t [p_t*min_t + w_t*(c_td + 1/2)] + outlier terms,   w_t = p_t*scale_t
// The sums over code fields are exact integer contractions: q (per head) and w (per tile)
// are written in fixed point, split into signed base-256 digits, and each digit plane
// goes through the 16x16x64 int8 matrix instruction as one row of the A operand, the code
// bytes being the B operand.  Only one query row exists per KV head here, so the other
// rows of the 16-row tile carry the further digits (and, on the key side, three more
// groups of 16 tokens): the matrix unit serves as a wide integer dot engine because the
// vector ALU cannot both unpack and multiply 2-bit codes at HBM rate.
//
// Spreading fields to bytes costs one AND per four codes where the mask can stay in
// place: (w & 0x0c0c0c0c) is 4*code, (w & 0x30303030) is 16*code, and the factor is taken
// out of the other operand's fixed-point digits (the top field of a byte would overflow a
// signed byte, so it is shifted down instead).  One-bit planes use masks 1,2,4,8 after at
// most one shift of the dword.
#include "qaq_internal.h"
#include <hip/hip_ext.h>

namespace {

constexpr int kThreads = 256;
constexpr int QAQ_MAX_NTC = 64;   // tiles per workgroup at most
constexpr int kFusedMaxTiles = 32;   // fused form: tiles of one head whose raw logits are kept in LDS (1 KB each)
typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float h2f(uint16_t b) { return __half2float(__ushort_as_half(b)); }
__device__ __forceinline__ v4i mma(v4i a, v4i b, v4i c) { return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }

// log2 of the factor the in-place masks leave on element group v (elements 4v..4v+3 of a
// slice) of a 2-bit resp. 1-bit field word
__device__ __forceinline__ int shift2(int v) { return v == 1 ? 2 : v == 2 ? 4 : 0; }
__device__ __forceinline__ int shift1(int v) { return v; }

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

// Global-memory pointer whose value is the same in every lane: goes through scalar
// registers, keeps the global address space (a pointer rebuilt from integers would
// otherwise become a generic one, whose loads also count as LDS traffic), and lets loads
// take the scalar-base + 32-bit-lane-offset form.
typedef const __attribute__((address_space(1))) uint8_t* gbytes_t;
__device__ __forceinline__ gbytes_t uniform_ptr(const void* p) {
  const uint64_t x = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
  return (gbytes_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t gload32(gbytes_t base, uint32_t off) {
  return *(const __attribute__((address_space(1))) uint32_t*)(base + off);
}
template <int N>
__device__ __forceinline__ void gload_dwords(gbytes_t p, uint32_t (&w)[N]) {
  typedef uint32_t u2 __attribute__((ext_vector_type(2)));
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  if constexpr (N == 1) {
    w[0] = *(const __attribute__((address_space(1))) uint32_t*)p;
  } else if constexpr (N == 2) {
    const u2 t = *(const __attribute__((address_space(1))) u2*)p;
    w[0] = t.x; w[1] = t.y;
  } else {
    static_assert(N % 4 == 0, "dword count");
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      const u4 t = ((const __attribute__((address_space(1))) u4*)p)[i];
      w[4 * i] = t.x; w[4 * i + 1] = t.y; w[4 * i + 2] = t.z; w[4 * i + 3] = t.w;
    }
  }
}

// Workgroup barrier that orders LDS traffic only.  All communication between the threads
// of these kernels goes through LDS, and __syncthreads() would also wait for every global
// load in flight -- including the loads of the next tile that are meant to stay in flight
// across the barrier.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// (wave_max, wave_sum: the one-instruction-per-step wavefront reductions of qaq_internal.h)
// max of two numbers that are known not to be NaN: one instruction
__device__ __forceinline__ float vmaxf(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Signed base-256 digits of an integer (each in [-128, 127]), packed little endian.
__device__ __forceinline__ uint32_t digits_packed(int x) {
  const int d0 = ((x + 128) & 255) - 128;
  const int r = (x - d0) >> 8;
  const int d1 = ((r + 128) & 255) - 128;
  const int r2 = (r - d1) >> 8;
  const int d2 = ((r2 + 128) & 255) - 128;
  const int d3 = (r2 - d2) >> 8;
  return (uint32_t)(d0 & 255) | ((uint32_t)(d1 & 255) << 8) | ((uint32_t)(d2 & 255) << 16) | ((uint32_t)(d3 & 255) << 24);
}

// B operand (16 byte-spread codes of one slice).  "Scaled" variants leave the factors
// 1, 4, 16, 1 (2-bit) resp. 1, 2, 4, 8 (1-bit) on the four element groups.
template <int BF>
__device__ __forceinline__ v4i spread(const uint32_t* w, int nib) {
  v4i b;
  if constexpr (BF == 2) {
    b[0] = (int)(w[0] & 0x03030303u); b[1] = (int)(w[0] & 0x0c0c0c0cu);
    b[2] = (int)(w[0] & 0x30303030u); b[3] = (int)((w[0] >> 6) & 0x03030303u);
  } else if constexpr (BF == 1) {
    const uint32_t x = nib ? (w[0] >> 4) : w[0];
    b[0] = (int)(x & 0x01010101u); b[1] = (int)(x & 0x02020202u);
    b[2] = (int)(x & 0x04040404u); b[3] = (int)(x & 0x08080808u);
  } else if constexpr (BF == 4) {
    b[0] = (int)(w[0] & 0x0f0f0f0fu); b[1] = (int)((w[0] >> 4) & 0x0f0f0f0fu);
    b[2] = (int)(w[1] & 0x0f0f0f0fu); b[3] = (int)((w[1] >> 4) & 0x0f0f0f0fu);
  } else {
    b[0] = (int)w[0]; b[1] = (int)w[1]; b[2] = (int)w[2]; b[3] = (int)w[3];
  }
  return b;
}

// One key record of field width BF, read whole by the lane that owns the token.
// Slice q of the record (16 channels, see the layout header) is one step of the
// contraction: the A operand holds the query digits of those 16 channels.
template <int D, int BF>
struct KRec {
  static constexpr int NQ = D / 16;                 // slices = contraction steps
  static constexpr int REC = D * BF / 8;
  static constexpr int RDW = D * BF / 32;           // dwords per record
  static __device__ __forceinline__ void load(const uint8_t* rbase, int ridx, uint32_t (&w)[RDW]) {
    load_dwords<RDW>(rbase + (uint32_t)ridx * (uint32_t)REC, w);
  }
  static __device__ __forceinline__ v4i operand(const uint32_t (&w)[RDW], int q) {
    if constexpr (BF == 1) return spread<1>(&w[q >> 1], q & 1);
    else return spread<BF>(&w[q * (BF / 2)], 0);
  }
};

template <int D>
struct TileLds {
  float qf[D];
  // Rows that different lanes of one 16-byte LDS read address together (digit rows of the
  // query, digit rows of the weights) are 16 bytes longer than their payload, so that equal
  // offsets in different rows fall into different banks.
  alignas(16) int8_t ql[3][4][D + 16];  // query digits [format][digit][position in record order]
  alignas(16) int8_t zrow[256];         // zeros: A operand of lanes whose row carries nothing
  alignas(16) uint16_t cnt[QAQ_MAX_NTC][8]; // class counts of the workgroup's tiles: keys, values
  float vb[QAQ_MAX_NTC];                // per tile: bound on the value-side weights and outlier corrections
  float logit[QAQ_TT];                  // raw logits by position
  alignas(16) int8_t wl2[4][QAQ_TT + 16];   // weight digits per slot of the 2-bit field region
  alignas(16) int8_t wl1[4][QAQ_TT + 16];   // ... of the 1-bit field region
  alignas(16) int8_t wl4[4][QAQ_TT + 16];   // ... of the 4-bit region
  alignas(16) int8_t wl1b[4][QAQ_TT + 16];  // ... of the 1-bit tokens' region
  float w8[QAQ_TT];                     // fp32 weights of the 8-bit slots
  float xw[4][D / 4];                   // per-wavefront 8-bit-class outputs (its own channels)
  float xcorr[D];                       // outlier corrections of the output (end of the chunk)
  alignas(16) int xc[D][16];            // ... of one tile, fixed point, 16 copies per channel (by lane % 16):
                                        // integer LDS atomics are several times faster than float ones, the
                                        // copies keep tokens that share a hot channel off one address, and
                                        // the sums do not depend on the order of arrival.  Copy c of channel
                                        // ch sits at column (c + 4*(ch/2)) % 16, so that neighbouring channels'
                                        // 16-byte reads of their copies start in different banks.
  float red[16];
  float part[D + 4];                    // fused form: this part's partial (output, then max, sum)
  float newv[D];                        // fused form, first part: the new token's value row (fetched in the prologue)
};

// 64 key records through the matrix unit, one per lane.  Lane (n, g) of the wavefront
// feeds its own record as column n of lane group g's share of the contraction index; row
// 4*tg + L of the A operand holds digit L of the query in lane group tg only, so row block
// tg of the result is the dot product with the records of lane group tg: lane l ends with
// the three digit sums (c[0..2]) of its own record.  `abase` is the lane's digit row in
// LDS (or a row of zeros for lanes whose A row is empty).
template <int D, int BF>
__device__ __forceinline__ v4i k_contract(const uint32_t (&w)[KRec<D, BF>::RDW], const int8_t* abase) {
  v4i c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
#pragma unroll
  for (int q = 0; q < KRec<D, BF>::NQ; ++q) {
    const v4i a = *(const v4i*)(abase + 16 * q);
    const v4i bb = KRec<D, BF>::operand(w, q);
    if (q & 1) c1 = mma(a, bb, c1); else c0 = mma(a, bb, c0);
  }
  return c0 + c1;
}

// Outlier side store of one slot: NO2 entries known at compile time (0 or 2), or up to 8
// with a run-time count.  Loads only move raw words; unpacking happens where the values
// are used, so that a load issued ahead of time is not waited for at its issue point.
template <int NO2>
struct Outl {
  static constexpr int CAP = NO2 ? NO2 : 1;
  static constexpr int NI = (CAP + 3) / 4, NV = (CAP + 1) / 2;
  uint32_t i2, v2;            // NO2 == 2: word holding the two channel bytes, two fp16 values
  int nmax = CAP;             // NO2 > 2: places any lane of the wavefront uses (uniform)
  uint32_t ip[NI], vp[NV];    // NO2 > 2: channel bytes and fp16 values, packed (place j: byte j, half j)
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int k = 0; k < NI; ++k) ip[k] = 0xffffffffu;
#pragma unroll
    for (int k = 0; k < NV; ++k) vp[k] = 0u;
  }
  __device__ __forceinline__ void put(int j, uint32_t ch, uint32_t hv) {      // j is a compile-time constant at every call
    ip[j >> 2] = (ip[j >> 2] & ~(0xffu << (8 * (j & 3)))) | (ch << (8 * (j & 3)));
    vp[j >> 1] = (vp[j >> 1] & ~(0xffffu << (16 * (j & 1)))) | (hv << (16 * (j & 1)));
  }
  // gi0: first slot of the tile (uniform), slot: the lane's slot inside the tile
  __device__ __forceinline__ void load(const QaqView& v, int side, size_t gi0, uint32_t slot, int no2) {
    if constexpr (NO2 == 2) {
      // whole aligned words only (the channel pair is one half of its word): nothing has
      // to be done to the loaded register until it is used
      i2 = gload32(uniform_ptr(v.oidx[side] + gi0 * 2), (2u * slot) & ~3u);
      v2 = gload32(uniform_ptr(v.oval[side] + gi0 * 2), 4u * slot);
    } else if constexpr (NO2 > 2) {
      if (v.csr) return;              // variable-length side store: fetched when the position is known (load_csr)
      const size_t gi = gi0 + slot;
      clear();
      if (no2 == 8) {                 // a row is two aligned words of channels and four of values
        const uint2 ci = *(const uint2*)(v.oidx[side] + gi * 8);
        const uint4 cv = *(const uint4*)(v.oval[side] + gi * 8);
        ip[0] = ci.x; ip[NI - 1] = ci.y;
        vp[0] = cv.x; vp[1 % NV] = cv.y; vp[2 % NV] = cv.z; vp[NV - 1] = cv.w;
      } else if (no2 == 4) {          // one word of channels, two of values
        ip[0] = *(const uint32_t*)(v.oidx[side] + gi * 4);
        const uint2 cv = *(const uint2*)(v.oval[side] + gi * 4);
        vp[0] = cv.x; vp[1 % NV] = cv.y;
      } else {
#pragma unroll
        for (int j = 0; j < NO2; ++j)
          if (j < no2) put(j, v.oidx[side][gi * no2 + j], v.oval[side][gi * no2 + j]);
      }
    }
  }
  // Variable-length side store (outliers by thresholds): the tile's pool is in position order;
  // `pos` = the token's position inside the tile.  Unused places keep channel 255.
  __device__ __forceinline__ void load_csr(const QaqView& v, int side, size_t gi0, uint32_t pos, int no2) {
    if constexpr (NO2 > 2) {
      const int cnt = v.ocnt[side][gi0 + pos], st = v.ostart[side][gi0 + pos];
      nmax = 0;
      clear();
#pragma unroll
      for (int j = 0; j < NO2; ++j) {
        const bool have = j < cnt && j < no2;
        if (__ballot(have) != 0ull) {        // uniform: most tokens have one or two, the row has room for eight
          nmax = j + 1;
          if (have) put(j, v.oidx[side][gi0 * no2 + st + j], v.oval[side][gi0 * no2 + st + j]);
        }
      }
    }
  }
  // slot: the slot the store was loaded for (selects the half of the channel word)
  __device__ __forceinline__ int idx(int j, uint32_t slot) const {
    if constexpr (NO2 == 2) return (int)((i2 >> (16 * (slot & 1u) + 8 * j)) & 0xffu);
    else return (int)((ip[j >> 2] >> (8 * (j & 3))) & 0xffu);
  }
  __device__ __forceinline__ bool used(int j) const {
    if constexpr (NO2 > 2) return j < nmax && ((ip[j >> 2] >> (8 * (j & 3))) & 0xffu) != 0xffu;
    else return true;
  }
  __device__ __forceinline__ float val(int j) const {
    if constexpr (NO2 == 2) return h2f((uint16_t)(v2 >> (16 * j)));
    else return h2f((uint16_t)(vp[j >> 1] >> (16 * (j & 1))));
  }
};

// Everything of one tile that is loaded ahead of its arithmetic, in two halves: what the
// key phase reads and what the softmax / value phases read.  Each half is reloaded for the
// next tile as soon as its phase is over, so one register set serves the whole chunk and the
// loads still have more than half a tile of arithmetic to arrive.  Addresses are a per-tile
// uniform base (scalar registers) plus a 32-bit lane offset.
template <int D, int NO2>
struct KeyRegs {
  QaqCounts c;
  int n_tok;
  // code words of the lane's own slot: a 2-bit field record in ka, the 1-bit record of a 3-bit
  // token in kb, or a 4-bit record in ka followed by kb.  8-bit records are four times that:
  // the first four 8-bit slots of a wavefront are fetched by its four groups of 16 lanes, 8
  // bytes per lane (k8); further ones, rare, are fetched when needed.
  static constexpr int HALF = KRec<D, 2>::RDW;
  uint32_t ka[HALF], kb[HALF];
  uint32_t k8[2];
  uint32_t mm, pos;
  Outl<NO2> o;
  template <bool H1>
  __device__ __forceinline__ void load(const QaqView& v, int len, int b, int h, int tile, const QaqCounts& ck, int tid) {
    c = ck;
    n_tok = min(len - tile * QAQ_TT, QAQ_TT);
    const uint8_t* base = qaq_tile_codes(v, 0, b, h, tile);
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    const uint32_t slot = (uint32_t)min(tid, n_tok - 1);
    mm = gload32(uniform_ptr(v.mm[0] + gi0), 4u * slot);
    pos = gload32(uniform_ptr(v.perm[0] + gi0), slot & ~3u);   // aligned word; byte slot%4 is the position
    o.load(v, 0, gi0, slot, v.no2);
    // one straight-line sequence of loads for every lane, whatever its class: only the offsets
    // differ (lanes with nothing to fetch read the first bytes of the tile side)
    const QaqKRegions rK = qaq_k_regions(c, D);
    const int n32 = c.n32();
    const bool is3 = tid < c.n3, is23 = tid < n32, is4 = !is23 && tid < n32 + c.n4;
    const bool is8 = !is23 && !is4 && tid < n_tok - c.n1;
    // a 4-bit record, or the first half of an 8-bit one (the other half is fetched where it is used)
    const uint32_t rec4 = is8 ? rK.r8 + (uint32_t)(tid - n32 - c.n4) * (uint32_t)KRec<D, 8>::REC
                              : rK.r4 + (uint32_t)(tid - n32) * (uint32_t)KRec<D, 4>::REC;
    const bool wide = is4 || is8;
    const uint32_t off_a = is23 ? (uint32_t)tid * (uint32_t)KRec<D, 2>::REC : wide ? rec4 : 0u;
    uint32_t off_b0 = is3 ? rK.r1 + (uint32_t)tid * (uint32_t)KRec<D, 1>::REC : wide ? rec4 + 4u * HALF : 0u;
    if (H1 && c.n1 > 0 && tid >= c.first1())          // a 1-bit token's record (lanes past the tile's tokens: the last one)
      off_b0 = rK.r1b + (uint32_t)min(tid - c.first1(), c.n1 - 1) * (uint32_t)KRec<D, 1>::REC;
    const uint32_t off_b1 = wide ? rec4 + 4u * HALF + 2u * HALF : 0u;
    const gbytes_t ubase = uniform_ptr(base);
    gload_dwords<HALF>(ubase + off_a, ka);
    uint32_t b0[HALF / 2], b1[HALF / 2];
    gload_dwords<HALF / 2>(ubase + off_b0, b0);
    gload_dwords<HALF / 2>(ubase + off_b1, b1);
#pragma unroll
    for (int i = 0; i < HALF / 2; ++i) { kb[i] = b0[i]; kb[HALF / 2 + i] = b1[i]; }
    // lane group g of the wavefront: bytes 8*(lane%16) .. +8 of the record of its g-th 8-bit slot
    const int first8 = n32 + c.n4;
    const int s8 = max(first8, tid & ~63) + ((tid & 63) >> 4);
    const uint32_t off8 = s8 < n_tok - c.n1 && 8 * (tid & 15) < D ? rK.r8 + (uint32_t)(s8 - first8) * (uint32_t)KRec<D, 8>::REC + 8u * (uint32_t)(tid & 15) : 0u;
    if (c.n8 > 0) gload_dwords<2>(ubase + off8, k8);      // uniform over the workgroup
  }
  // The first tile of a part, in two steps, so that its bytes are on their way while the class counts
  // are: `head` asks for what can be addressed without the counts -- the slot's metadata and the 2-bit
  // field record of slot `tid`, which is where the record of a 2- or 3-bit token is -- and `tail`, once
  // the counts are known, for the rest (and for the first word group again where the tile has 4-bit
  // tokens, whose records are elsewhere: rare, and uniform over the workgroup).
  __device__ __forceinline__ void load_head(const QaqView& v, int len, int b, int h, int tile, int tid) {
    n_tok = min(len - tile * QAQ_TT, QAQ_TT);
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    const uint32_t slot = (uint32_t)min(tid, n_tok - 1);
    mm = gload32(uniform_ptr(v.mm[0] + gi0), 4u * slot);
    pos = gload32(uniform_ptr(v.perm[0] + gi0), slot & ~3u);
    o.load(v, 0, gi0, slot, v.no2);
    gload_dwords<HALF>(uniform_ptr(qaq_tile_codes(v, 0, b, h, tile)) + (uint32_t)tid * (uint32_t)KRec<D, 2>::REC, ka);
  }
  template <bool H1>
  __device__ __forceinline__ void load_tail(const QaqView& v, int b, int h, int tile, const QaqCounts& ck, int tid) {
    c = ck;
    const QaqKRegions rK = qaq_k_regions(c, D);
    const int n32 = c.n32();
    const bool is3 = tid < c.n3, is23 = tid < n32, is4 = !is23 && tid < n32 + c.n4;
    const bool is8 = !is23 && !is4 && tid < n_tok - c.n1;
    // a 4-bit record, or the first half of an 8-bit one (the other half is fetched where it is used)
    const uint32_t rec4 = is8 ? rK.r8 + (uint32_t)(tid - n32 - c.n4) * (uint32_t)KRec<D, 8>::REC
                              : rK.r4 + (uint32_t)(tid - n32) * (uint32_t)KRec<D, 4>::REC;
    const bool wide = is4 || is8;
    const uint32_t off_a = is23 ? (uint32_t)tid * (uint32_t)KRec<D, 2>::REC : wide ? rec4 : 0u;
    uint32_t off_b0 = is3 ? rK.r1 + (uint32_t)tid * (uint32_t)KRec<D, 1>::REC : wide ? rec4 + 4u * HALF : 0u;
    if (H1 && c.n1 > 0 && tid >= c.first1())
      off_b0 = rK.r1b + (uint32_t)min(tid - c.first1(), c.n1 - 1) * (uint32_t)KRec<D, 1>::REC;
    const uint32_t off_b1 = wide ? rec4 + 4u * HALF + 2u * HALF : 0u;
    const gbytes_t ubase = uniform_ptr(qaq_tile_codes(v, 0, b, h, tile));
    if (c.n4 + c.n8 > 0) {     // (into other registers first: a load into registers that an earlier load is still on its way to is held back until that one has arrived)
      uint32_t t[HALF];
      gload_dwords<HALF>(ubase + off_a, t);
#pragma unroll
      for (int i = 0; i < HALF; ++i) ka[i] = t[i];
    }
    uint32_t b0[HALF / 2], b1[HALF / 2];
    gload_dwords<HALF / 2>(ubase + off_b0, b0);
    gload_dwords<HALF / 2>(ubase + off_b1, b1);
#pragma unroll
    for (int i = 0; i < HALF / 2; ++i) { kb[i] = b0[i]; kb[HALF / 2 + i] = b1[i]; }
    const int first8 = n32 + c.n4;
    const int s8 = max(first8, tid & ~63) + ((tid & 63) >> 4);
    const uint32_t off8 = s8 < n_tok - c.n1 && 8 * (tid & 15) < D ? rK.r8 + (uint32_t)(s8 - first8) * (uint32_t)KRec<D, 8>::REC + 8u * (uint32_t)(tid & 15) : 0u;
    if (c.n8 > 0) gload_dwords<2>(ubase + off8, k8);
  }
};

template <int D, int NO2>
struct ValRegs {
  static constexpr int NCG = D / 16;
  static constexpr int CGW = NCG / 4;
  QaqCounts c;
  uint32_t mm, pos;
  Outl<NO2> o;
  uint32_t vw2[4][CGW], vw1[4];
  // vw1: blocks (of 4 units) of the 3-bit tokens' low planes from entry 0 up; with a width set
  // that has 1, blocks of the 1-bit tokens' units from entry 3 down as far as entries are free
  // PRE8 (the grouped-query kernel; in k_attn_tile the two registers cost the common case more than
  // the rare classes gain):
  uint32_t v4p;  // D = 128: one word of the first two half-units (16 slots) of the 4-bit region: lane
                 // group g holds word g & 1 of half-unit g >> 1 (handed to the lanes that need it when it is used)
  uint32_t v8;   // 8-bit values (token-major rows): this lane's four channels of row lane / (D/16), so
                 // that the first 64 / (D/16) such tokens of a tile -- a tile of a cache the rules shaped rarely
                 // has more -- cost no load inside the tile loop
  template <bool H1, bool PRE8 = false>
  __device__ __forceinline__ void load(const QaqView& v, int len, int b, int h, int tile, const QaqCounts& cv, int tid, int wave, int nn, int g) {
    c = cv;
    const int n_tok = min(len - tile * QAQ_TT, QAQ_TT);
    const uint8_t* base = qaq_tile_codes(v, 1, b, h, tile);
    const gbytes_t ubase = uniform_ptr(base);
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    const uint32_t slot = (uint32_t)min(tid, n_tok - 1);
    mm = gload32(uniform_ptr(v.mm[1] + gi0), 4u * slot);
    pos = gload32(uniform_ptr(v.perm[1] + gi0), slot & ~3u);
    o.load(v, 1, gi0, slot, v.no2);
    const uint32_t voff = (uint32_t)g * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
      if (!H1 || blk * 64 < c.n32()) gload_dwords<CGW>(ubase + voff + (uint32_t)blk * (16u * D), vw2[blk]);   // (blocks past the region are not used)
    const QaqVRegions rV = qaq_v_regions(c, D);
    if (PRE8 && CGW == 2) {
      const int nhu = (c.n4 + 7) >> 3;
      v4p = gload32(ubase, c.n4 > 0 ? rV.r4 + (uint32_t)min(g >> 1, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * (uint32_t)(CGW * wave + (g & 1)) : 0u);
    }
    if (PRE8) {
      const int lane = tid & 63;
      v8 = gload32(ubase, c.n8 > 0 ? rV.r8 + (uint32_t)min(lane / (D / 16), c.n8 - 1) * D + (D / 4) * wave + 4 * (lane % (D / 16)) : 0u);
    }
    const int nu1 = (c.n3 + 15) >> 4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
      if (blk * 4 < nu1)
        vw1[blk] = *(const uint32_t*)(base + rV.r1 + (uint32_t)min(blk * 4 + g, nu1 - 1) * (2u * D) + (uint32_t)nn * (NCG * 2) + 4u * ((CGW * wave) >> 1));
    if (H1) {
      const int nb3 = (nu1 + 3) >> 2, nu1b = (c.n1 + 15) >> 4;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
        if (blk * 4 < nu1b && 3 - blk >= nb3)
          vw1[3 - blk] = *(const uint32_t*)(base + rV.r1b + (uint32_t)min(blk * 4 + g, nu1b - 1) * (2u * D) + (uint32_t)nn * (NCG * 2) + 4u * ((CGW * wave) >> 1));
    }
  }
  // the first tile of a part in two steps, as for the keys: the 2-bit field units start the tile side
  template <bool H1>
  __device__ __forceinline__ void load_head(const QaqView& v, int len, int b, int h, int tile, int tid, int wave, int nn, int g) {
    const int n_tok = min(len - tile * QAQ_TT, QAQ_TT);
    const gbytes_t ubase = uniform_ptr(qaq_tile_codes(v, 1, b, h, tile));
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    const uint32_t slot = (uint32_t)min(tid, n_tok - 1);
    mm = gload32(uniform_ptr(v.mm[1] + gi0), 4u * slot);
    pos = gload32(uniform_ptr(v.perm[1] + gi0), slot & ~3u);
    o.load(v, 1, gi0, slot, v.no2);
    if (!H1) {
      const uint32_t voff = (uint32_t)g * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) gload_dwords<CGW>(ubase + voff + (uint32_t)blk * (16u * D), vw2[blk]);
    }
  }
  template <bool H1>
  __device__ __forceinline__ void load_tail(const QaqView& v, int b, int h, int tile, const QaqCounts& cv, int wave, int nn, int g) {
    c = cv;
    const uint8_t* base = qaq_tile_codes(v, 1, b, h, tile);
    if (H1) {
      const gbytes_t ubase = uniform_ptr(base);
      const uint32_t voff = (uint32_t)g * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
        if (blk * 64 < c.n32()) gload_dwords<CGW>(ubase + voff + (uint32_t)blk * (16u * D), vw2[blk]);
    }
    const QaqVRegions rV = qaq_v_regions(c, D);
    const int nu1 = (c.n3 + 15) >> 4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
      if (blk * 4 < nu1)
        vw1[blk] = *(const uint32_t*)(base + rV.r1 + (uint32_t)min(blk * 4 + g, nu1 - 1) * (2u * D) + (uint32_t)nn * (NCG * 2) + 4u * ((CGW * wave) >> 1));
    if (H1) {
      const int nb3 = (nu1 + 3) >> 2, nu1b = (c.n1 + 15) >> 4;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
        if (blk * 4 < nu1b && 3 - blk >= nb3)
          vw1[3 - blk] = *(const uint32_t*)(base + rV.r1b + (uint32_t)min(blk * 4 + g, nu1b - 1) * (2u * D) + (uint32_t)nn * (NCG * 2) + 4u * ((CGW * wave) >> 1));
    }
  }
};

// ---------------------------------------------------------------------------------------
// One workgroup: one (sequence, query head), part `chunk` of its tiles: the tiles are split
// into nparts runs whose lengths differ by at most one, the longer runs last (the last tile
// is the one that may be partly filled).  The loads
// of tile t+1 are in flight while tile t is computed; the output, the softmax sum and the
// constant terms are carried in registers across the tiles with the usual rescaling by
// exp(old max - new max), and one partial is written per workgroup.
//
// Two forms.  P = 0: one part per workgroup of 256 threads; the partial goes to HBM and
// k_attn_combine merges the parts.  P = 1..4 (fused): the P parts of a head are the P groups
// of 256 threads of one workgroup, each with its own LDS block, in lockstep (every group runs
// the same number of iterations and skips the work of those past its last tile, so that all
// barriers are met by all wavefronts); raw logits stay in LDS, the parts are merged in LDS,
// and the workgroup writes the output and the normalised scores itself: no second kernel.
// H1: the width set contains 1 (a fifth class at the end of every tile); without it that
// class costs nothing.
// PP = 5: the fused form with four parts whose raw logits wait in the score buffer instead of LDS
// (a head with more tiles than the LDS store holds; a form of its own so that the common one carries
// no test for it: as a run-time flag it cost the call 0.4 us).
template <int D, int NO2, int PP, bool H1>
__global__ __launch_bounds__((PP == 5 ? 4 : PP ? PP : 1) * kThreads, 4) void k_attn_tile(QaqAttnArgs a) {   // four wavefronts per SIMD
  constexpr int P = PP == 5 ? 4 : PP;
  constexpr bool LDS_LOGITS = PP != 5;
  constexpr int KS = D / 64;
  constexpr int NCG = D / 16;
  constexpr int CGW = NCG / 4;              // channel groups per wavefront on the value side
  __shared__ TileLds<D> S_all[P ? P : 1];
  extern __shared__ float lg_all[];         // fused form: raw logits [part][iteration][position]
  const QaqView& v = a.v;
  const int chunk = P ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8)) : (int)blockIdx.x;
  TileLds<D>& S = S_all[P ? chunk : 0];
  const int tid = threadIdx.x & (kThreads - 1), lane = tid & 63, wave = tid >> 6;
  const int nn = lane & 15, g = lane >> 4;
  // Key side: which quarter of a tile's slots a wavefront takes rotates with the part, so that the
  // wavefronts one SIMD hosts (the same wavefront index of the parts that share a compute unit) do not
  // all get the quarter with the widest keys: slots are sorted by width, and a quarter of 3-bit
  // keys costs twice the contractions of a quarter of 2-bit keys.  The threads that sum the
  // outlier corrections of the output rotate the same way.
  const int kwave = (wave + chunk) & 3, ktid = 64 * kwave + lane;
  // Grouped queries, fused form: workgroups are dealt to the eight dies round-robin, so the G
  // query heads of a KV head, which read the same codes, are given indices that land on one
  // die (the reads after the first are served by that die's L2): die x takes the x-th eighth
  // of the (sequence, query head) pairs.
  int bq = blockIdx.y;
  if (P && a.G > 1 && (gridDim.y & 7) == 0) bq = (int)(blockIdx.y & 7) * (int)(gridDim.y >> 3) + (int)(blockIdx.y >> 3);
  const int b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
  const int len = qaq_seq_len(v, b, a.len);          // cached tokens of this sequence
  const int ntile = (len + QAQ_TT - 1) / QAQ_TT;
  const int tile_begin = (int)((long long)chunk * ntile / a.nparts);
  const int tile_end = (int)((long long)(chunk + 1) * ntile / a.nparts);
  if (!P && tile_begin >= tile_end) {
    // a sequence shorter than the longest can leave a part without tiles: a partial that the merge ignores
    float* part = a.partial + ((size_t)bq * a.part_stride + chunk) * (D + 4);
    if (tid < D) part[tid] = 0.0f;
    if (tid == 0) { part[D] = -INFINITY; part[D + 1] = 0.0f; }
    return;
  }
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const int no2 = v.no2;
  const v4i zero4 = {0, 0, 0, 0};

  // (no load of the prologue sits behind a branch: the compiler places its waits by counting the loads
  // issued after the one it waits for, and where that number depends on a branch it waits for all of them
  // -- here for the first tile's codes, before the barrier that everything else is behind)
  const __half q_raw = a.q[(size_t)bq * D + min(tid, D - 1)];
  // class counts of all tiles of the chunk -> LDS (one 16-byte load per tile), so that the
  // tile loop needs no dependent global load to place its 1-bit regions
  const int my_tile = tile_begin + min(tid, tile_end - tile_begin - 1);
  const uint4 cnt_raw = *(const uint4*)(v.counts + ((qaq_bh(v, b, h) * v.NT + my_tile) * 2) * 4);
  const float vb_raw = v.vbound[qaq_bh(v, b, h) * v.NT + my_tile];
  // fused form: the new token's key and value rows are needed at the very end, by the first part; asked for
  // there, each would be a memory round trip with nothing left to hide it behind
  // (where they are not needed, the query row is read again instead: no load behind a branch)
  const bool new_here = P && chunk == 0 && a.k_new;
  const __half kn_raw = (new_here ? a.k_new + ((size_t)b * v.Hkv + h) * D : a.q + (size_t)bq * D)[min(tid, D - 1)];
  const __half vn_raw = (new_here ? a.v_new + ((size_t)b * v.Hkv + h) * D : a.q + (size_t)bq * D)[min(tid, D - 1)];
  asm volatile("" ::: "memory");      // these first: what follows is the bulk, and loads come back in the order of issue
  // the first tile: what its class counts are not needed for is requested at once
  KeyRegs<D, NO2> kr;
  ValRegs<D, NO2> vr;
  kr.load_head(v, len, b, h, tile_begin, ktid);
  vr.template load_head<H1>(v, len, b, h, tile_begin, tid, wave, nn, g);
  const float qv = tid < D ? __half2float(q_raw) : 0.0f;
  if (new_here) {
    const float qk = wave_sum(tid < D ? __half2float(q_raw) * __half2float(kn_raw) : 0.0f);
    if (lane == 0) S.red[12 + wave] = qk;
    if (tid < D) S.newv[tid] = __half2float(vn_raw);
  }
  if (tid < tile_end - tile_begin) {
    *(uint4*)&S.cnt[tid][0] = cnt_raw;
    S.vb[tid] = vb_raw;
  }

  // ---- query: fixed point, signed base-256 digits, one table per spreading format ------------
  if (wave < KS) {          // the wavefronts that hold the D query channels
    const float am = wave_max(fabsf(qv));
    const float sm = wave_sum(qv);
    if (lane == 0) { S.red[wave] = am; S.red[4 + wave] = sm; }
    S.qf[tid] = qv;
  }
  S.zrow[tid] = 0;
  for (int e = tid; e < D * 16; e += kThreads) (&S.xc[0][0])[e] = 0;
  lds_barrier();
  // the rest of the first tile is requested before the query digits are made
  auto counts_of = [&](int t, int side) {
    const uint2 c = *(const uint2*)&S.cnt[t - tile_begin][4 * side];
    const uint32_t lo = __builtin_amdgcn_readfirstlane(c.x), hi = __builtin_amdgcn_readfirstlane(c.y);
    QaqCounts r;
    r.n3 = lo & 0xffffu; r.n2 = lo >> 16; r.n4 = hi & 0xffffu; r.n8 = hi >> 16;
    r.n1 = H1 ? min(len - t * QAQ_TT, QAQ_TT) - (r.n3 + r.n2 + r.n4 + r.n8) : 0;      // the 1-bit class is the rest of the tile
    return r;
  };
  kr.template load_tail<H1>(v, b, h, tile_begin, counts_of(tile_begin, 0), ktid);
  vr.template load_tail<H1>(v, b, h, tile_begin, counts_of(tile_begin, 1), wave, nn, g);
  const float qmax = KS == 1 ? S.red[0] : fmaxf(S.red[0], S.red[1]);
  const float sumq = KS == 1 ? S.red[4] : S.red[4] + S.red[5];
  int qexp = 0;
  if (qmax > 0.0f) (void)frexpf(qmax, &qexp);
  const float qscale = qmax > 0.0f ? ldexpf(1.0f, qexp - 22) : 0.0f;
  if (wave < KS) {
    // channel tid sits at position 16*(g'*KS + ks) + i of a record
    const int i = tid & 15, vgr = i >> 2;
    const int pos = 16 * (((tid & 63) >> 4) * KS + (tid >> 6)) + i;
#pragma unroll
    for (int f = 0; f < 3; ++f) {
      const int sh = f == 0 ? shift2(vgr) : f == 1 ? shift1(vgr) : 0;
      const int x = qmax > 0.0f ? (int)rintf(ldexpf(qv, 22 - qexp - sh)) : 0;
      const uint32_t dg = digits_packed(x);
      S.ql[f][0][pos] = (int8_t)dg; S.ql[f][1][pos] = (int8_t)(dg >> 8); S.ql[f][2][pos] = (int8_t)(dg >> 16);
    }
  }
  lds_barrier();
  // A rows: row r = 4*tg + L is switched on in lane group tg only
  const bool arow = (g == (nn >> 2)) && ((nn & 3) < 3);
  const int8_t* abase0 = arow ? &S.ql[0][nn & 3][0] : &S.zrow[0];
  const int8_t* abase1 = arow ? &S.ql[1][nn & 3][0] : &S.zrow[0];
  const int8_t* abase2 = arow ? &S.ql[2][nn & 3][0] : &S.zrow[0];
  const int8_t* wb2 = nn < 4 ? &S.wl2[nn][16 * g] : &S.zrow[0];
  const int8_t* wb1 = nn < 4 ? &S.wl1[nn][16 * g] : &S.zrow[0];
  const int8_t* wb4 = nn < 4 ? &S.wl4[nn][16 * g] : &S.zrow[0];
  const int8_t* wb1b = nn < 4 ? &S.wl1b[nn][16 * g] : &S.zrow[0];

  auto real_of = [&](const v4i& c) { return (((float)c[2] * 65536.0f + (float)c[1] * 256.0f) + (float)c[0]) * qscale; };
  auto key_logit = [&](uint32_t m, const Outl<NO2>& o, uint32_t slot, int bits, float dotq) {
    const float mn = h2f((uint16_t)(m & 0xffffu)), mx = h2f((uint16_t)(m >> 16));
    const float range = mx - mn;
    const float scale = ldexpf(range, -bits);
    float val = mn * sumq + scale * (dotq + 0.5f * sumq);
    // an outlier above the range was coded 2^B-1 (reconstruction max - scale/2), one below
    // it 0 (min + scale/2): replace that reconstruction by the stored value
    const float hs = 0.5f * scale;
#pragma unroll
    for (int j = 0; j < Outl<NO2>::CAP; ++j) {
      if (j < NO2 && j < no2 && o.used(j)) {
        const float ov = o.val(j);
        const bool top = ov >= mx;
        val += S.qf[o.idx(j, slot)] * ((ov - (top ? mx : mn)) + (top ? hs : -hs));
      }
    }
    return val * inv_sqrt_d;
  };


  // carried across the tiles
  float m_run = -INFINITY;          // reference of everything below
  float l_run = 0.0f, bias_run = 0.0f;    // per thread: softmax sum and constant terms of its slots
  float c_run = 0.0f;               // threads with ktid < D: outlier correction of channel ktid
  float xrun[CGW];                  // lanes of group 0: output of channel 16*(CGW*wave+j)+n
#pragma unroll
  for (int j = 0; j < CGW; ++j) xrun[j] = 0.0f;

  const int n_iter = P ? a.ntc : tile_end - tile_begin;
  for (int it = 0; it < n_iter; ++it) {
    const int tile = tile_begin + it;
    const bool on = !P || tile < tile_end;       // uniform over the part's 256 threads
    const QaqCounts cK = kr.c, cV = vr.c;
    const int n_tok = kr.n_tok;
    const uint32_t slot = (uint32_t)min(tid, n_tok - 1);   // the value slot this lane's metadata was loaded for
    const uint32_t kslot = (uint32_t)min(ktid, n_tok - 1); // ... the key slot
    const QaqKRegions rK = qaq_k_regions(cK, D);
    const QaqVRegions rV = qaq_v_regions(cV, D);
    // (scalar base + 32-bit lane offset for what is fetched inside the loop: no 64-bit lane addresses)
    const gbytes_t baseK = uniform_ptr(qaq_tile_codes(v, 0, b, h, tile));
    const gbytes_t baseV = uniform_ptr(qaq_tile_codes(v, 1, b, h, tile));
    const int n32K = cK.n32(), n32V = cV.n32();
    const int first8V = n32V + cV.n4;
    const int first1K = H1 ? cK.first1() : n_tok, first1V = H1 ? cV.first1() : n_tok;

    // ---- keys: logits ----------------------------------------------------------------------------
    // Every lane owns key slot `ktid`; the wavefront runs one contraction chain per width class that
    // occurs among its 64 slots (one, except where a class boundary falls inside them) and
    // every lane keeps the result of its own class.
    float vmax = -INFINITY;
    if (on) {
      const int w0 = kwave * 64, w1 = w0 + 64;
      const int first8K = n32K + cK.n4;
      float dotq = 0.0f;
      if (w0 < n32K) {
        dotq = real_of(k_contract<D, 2>(kr.ka, abase0));
        if (w0 < cK.n3) {
          uint32_t k1[KRec<D, 1>::RDW];
#pragma unroll
          for (int i = 0; i < KRec<D, 1>::RDW; ++i) k1[i] = kr.kb[i];
          const float low = real_of(k_contract<D, 1>(k1, abase1));
          dotq = ktid < cK.n3 ? 2.0f * dotq + low : dotq;
        }
      }
      if (w1 > n32K && w0 < first8K) {
        uint32_t k4[KRec<D, 4>::RDW];
#pragma unroll
        for (int i = 0; i < KeyRegs<D, NO2>::HALF; ++i) { k4[i] = kr.ka[i]; k4[KeyRegs<D, NO2>::HALF + i] = kr.kb[i]; }
        const float d4 = real_of(k_contract<D, 4>(k4, abase2));
        if (ktid >= n32K) dotq = d4;
      }
      const int s8_0 = max(first8K, w0);                 // first 8-bit slot among this wavefront's
      const int n8w = min(first1K, w1) - s8_0;           // and how many there are
      if (n8w > 0 && n8w <= 4) {
        // a few 8-bit keys: every group of 16 lanes takes one, a lane 8 of its bytes (fetched
        // with the rest of the tile), fp32 products with the query in a fixed order
        const int j = 8 * (lane & 15) < D ? lane & 15 : 0, sl = j >> 1;   // a record has D bytes: D/8 lanes of the group carry it
        const int ch0 = 64 * (sl % KS) + 16 * (sl / KS) + 8 * (j & 1);   // channel of the lane's first byte
        const float4 q0 = *(const float4*)&S.qf[ch0], q1 = *(const float4*)&S.qf[ch0 + 4];
        const uint32_t c0 = kr.k8[0] ^ 0x80808080u, c1 = kr.k8[1] ^ 0x80808080u;   // stored as code - 128
        float d = (float)(c0 & 255u) * q0.x;
        d += (float)((c0 >> 8) & 255u) * q0.y;
        d += (float)((c0 >> 16) & 255u) * q0.z;
        d += (float)(c0 >> 24) * q0.w;
        d += (float)(c1 & 255u) * q1.x;
        d += (float)((c1 >> 8) & 255u) * q1.y;
        d += (float)((c1 >> 16) & 255u) * q1.z;
        d += (float)(c1 >> 24) * q1.w;
        if (8 * (lane & 15) >= D) d = 0.0f;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) d += __shfl_xor(d, o);
        const int own = ktid - s8_0;                       // the lane that owns the slot
        const float dd = __shfl(d, 16 * (own & 3));
        if (own >= 0 && own < n8w) dotq = dd;
      } else if (__builtin_expect(n8w > 4, 0)) {
        // 8-bit key bytes are stored as code - 128: the dot product gets 128 * (sum of the
        // unscaled query integers) back, rebuilt here from their digits (this class is rare)
        int sq = 0;
        for (int d = lane; d < D; d += 64) sq += (int)S.ql[2][0][d] + 256 * (int)S.ql[2][1][d] + 65536 * (int)S.ql[2][2][d];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) sq += __shfl_xor(sq, o);
        // The first half of a lane's record came with the tile (where a narrower token has its code
        // words); the second half is fetched here in pieces of two slices, the first piece before the
        // arithmetic on the first half, the next into registers that arithmetic has freed: the whole
        // record in registers would make every tile of every call pay for this path with spills.
        // (Lanes of other classes feed what they hold; their results are not used.)
        const uint32_t rec = rK.r8 + (uint32_t)min(max(ktid - first8K, 0), cK.n8 - 1) * (uint32_t)D;
        v4i cc = zero4;
        uint32_t w[8];
        gload_dwords<8>(baseK + (rec + (uint32_t)(D / 2)), w);
        if constexpr (D == 128) {
          cc = mma(*(const v4i*)(abase2), spread<8>(&kr.ka[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 16), spread<8>(&kr.ka[4], 0), cc);
          asm volatile("" ::: "memory");      // (not earlier: four pieces in flight at once do not fit the registers)
          gload_dwords<8>(baseK + (rec + 96u), kr.ka);
          cc = mma(*(const v4i*)(abase2 + 32), spread<8>(&kr.kb[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 48), spread<8>(&kr.kb[4], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 64), spread<8>(&w[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 80), spread<8>(&w[4], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 96), spread<8>(&kr.ka[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 112), spread<8>(&kr.ka[4], 0), cc);
        } else {
          static_assert(D == 64, "head_dim");
          cc = mma(*(const v4i*)(abase2), spread<8>(&kr.ka[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 16), spread<8>(&kr.kb[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 32), spread<8>(&w[0], 0), cc);
          cc = mma(*(const v4i*)(abase2 + 48), spread<8>(&w[4], 0), cc);
        }
        if (ktid >= first8K) dotq = ((((float)cc[2] * 65536.0f + (float)cc[1] * 256.0f) + (float)cc[0]) + 128.0f * (float)sq) * qscale;
      }
      if (H1 && cK.n1 > 0 && w1 > first1K) {
        // 1-bit keys (only with a width set that has 1): the record came with the tile, where
        // a 3-bit token has its low bits
        uint32_t k1[KRec<D, 1>::RDW];
#pragma unroll
        for (int i = 0; i < KRec<D, 1>::RDW; ++i) k1[i] = kr.kb[i];
        const float d1 = real_of(k_contract<D, 1>(k1, abase1));
        if (ktid >= first1K) dotq = d1;
      }
      if (ktid < n_tok) {
        if constexpr (NO2 > 2)
          if (v.csr) kr.o.load_csr(v, 0, qaq_slot_index(v, b, h, tile, 0), (kr.pos >> (8u * (kslot & 3u))) & 0xffu, no2);
        const float lg = key_logit(kr.mm, kr.o, kslot, H1 ? cK.bits_of_slot(ktid) : cK.bits_of_slot4(ktid), dotq);
        S.logit[(kr.pos >> (8u * (kslot & 3u))) & 0xffu] = lg;
        vmax = lg;
      }
    }
    // the key registers are free: request the next tile's keys
    if (tile + 1 < tile_end) kr.template load<H1>(v, len, b, h, tile + 1, counts_of(tile + 1, 0), ktid);

    vmax = wave_max(vmax);
    if (lane == 0) S.red[8 + wave] = vmax;
    lds_barrier();
    const float m_tile = vmaxf(vmaxf(S.red[8], S.red[9]), vmaxf(S.red[10], S.red[11]));
    const float smax = on ? S.vb[tile - tile_begin] : 0.0f;     // bound on w/p and on the outlier corrections over the tile
    const float M = vmaxf(m_run, m_tile);
    const float keep = on ? __expf(m_run - M) : 1.0f;          // 0 on the first tile
    m_run = M;
    int wexp = 0;
    if (smax > 0.0f) (void)frexpf(smax, &wexp);
    const float wscale = smax > 0.0f ? ldexpf(1.0f, wexp - 28) : 0.0f;

    // ---- values: weight of slot `tid`, as digits -------------------------------------------------
    if (a.scores && on && tid < n_tok) {
      // fused form: in LDS if a head's logits fit, else in the score buffer, where the same thread finds
      // them again at the end (through the L2: volatile); two-kernel form: for the merge kernel
      if (P && LDS_LOGITS) lg_all[((chunk * a.ntc + it) << 8) + tid] = S.logit[tid];
      else if (P) ((volatile float*)a.scores)[(size_t)bq * a.score_stride + tile * QAQ_TT + tid] = S.logit[tid];
      else a.scores[(size_t)bq * a.score_stride + tile * QAQ_TT + tid] = S.logit[tid];
    }
    if (on) {
      const int s = tid;
      const bool live = s < n_tok;
      float pt = 0.0f, bias_l = 0.0f, w = 0.0f;
      if (live) {
        if constexpr (NO2 > 2)
          if (v.csr) vr.o.load_csr(v, 1, qaq_slot_index(v, b, h, tile, 0), (vr.pos >> (8u * (slot & 3u))) & 0xffu, no2);
        pt = __expf(S.logit[(vr.pos >> (8u * (slot & 3u))) & 0xffu] - M);
        const float mn = h2f((uint16_t)(vr.mm & 0xffffu)), mx = h2f((uint16_t)(vr.mm >> 16));
        const float range = mx - mn;
        const int bits = H1 ? cV.bits_of_slot(s) : cV.bits_of_slot4(s);
        const float scale = ldexpf(range, -bits);
        w = pt * scale;
        bias_l = pt * mn + 0.5f * w;
        const float hs = 0.5f * scale;
#pragma unroll
        for (int j = 0; j < Outl<NO2>::CAP; ++j) {
          if (j < NO2 && j < no2 && vr.o.used(j)) {
            const float ov = vr.o.val(j);
            const bool top = ov >= mx;
            // |correction| < 2^wexp, at most 32 arrive per copy: units of 2^(wexp-25) cannot overflow
            const float cval = pt * ((ov - (top ? mx : mn)) + (top ? hs : -hs));
            const int och = vr.o.idx(j, slot);
            atomicAdd(&S.xc[och][(lane + 4 * (och >> 1)) & 15], (int)rintf(ldexpf(cval, 25 - wexp)));
          }
        }
        if (s >= first8V && (!H1 || s < first1V)) S.w8[s - first8V] = w;
      }
      l_run = l_run * keep + pt;
      bias_run = bias_run * keep + bias_l;
      // Fixed point in units of 2^(e-28), e = exponent of the bound: W = round(w * 2^(28-e-sh)),
      // sh = what the spreading mask of the slot's place in its unit leaves on the code.
      // Weights are not negative, so W is split into four base-128 digits (0..127, valid
      // signed bytes).  A 3-bit code is 2*top + low, so its top plane weighs 2w (at most the
      // bound) and its low plane w.  Every entry of a digit table in use is written exactly
      // once (zero where the slot is not in that region), so partial units multiply padding
      // by zero.
      const bool fx = live && smax > 0.0f;
      const int vg = (s & 15) >> 2;
      const uint32_t W2 = (fx && s < n32V) ? (uint32_t)rintf(ldexpf(w, 28 - wexp - shift2(vg) + (s < cV.n3 ? 1 : 0))) : 0u;
      S.wl2[0][s] = (int8_t)(W2 & 127u); S.wl2[1][s] = (int8_t)((W2 >> 7) & 127u);
      S.wl2[2][s] = (int8_t)((W2 >> 14) & 127u); S.wl2[3][s] = (int8_t)(W2 >> 21);
      // (the value phase reads these two tables in blocks of 64 slots, as far as the class reaches:
      // slots of later blocks need no digits, not even zeros)
      if (s < ((cV.n3 + 63) & ~63)) {
        const uint32_t W1 = (fx && s < cV.n3) ? (uint32_t)rintf(ldexpf(w, 28 - wexp - shift1(vg))) : 0u;
        S.wl1[0][s] = (int8_t)(W1 & 127u); S.wl1[1][s] = (int8_t)((W1 >> 7) & 127u);
        S.wl1[2][s] = (int8_t)((W1 >> 14) & 127u); S.wl1[3][s] = (int8_t)(W1 >> 21);
      }
      if (((s - n32V) & (QAQ_TT - 1)) < ((cV.n4 + 63) & ~63)) {
        const int i4 = (s - n32V) & (QAQ_TT - 1);
        const uint32_t W4 = (fx && s >= n32V && s < first8V) ? (uint32_t)rintf(ldexpf(w, 28 - wexp)) : 0u;
        S.wl4[0][i4] = (int8_t)(W4 & 127u); S.wl4[1][i4] = (int8_t)((W4 >> 7) & 127u);
        S.wl4[2][i4] = (int8_t)((W4 >> 14) & 127u); S.wl4[3][i4] = (int8_t)(W4 >> 21);
      }
      if (H1 && cV.n1 > 0) {
        const int i1 = (s - first1V) & (QAQ_TT - 1);
        const uint32_t W1 = (fx && s >= first1V) ? (uint32_t)rintf(ldexpf(w, 28 - wexp - shift1((i1 & 15) >> 2))) : 0u;
        S.wl1b[0][i1] = (int8_t)(W1 & 127u); S.wl1b[1][i1] = (int8_t)((W1 >> 7) & 127u);
        S.wl1b[2][i1] = (int8_t)((W1 >> 14) & 127u); S.wl1b[3][i1] = (int8_t)(W1 >> 21);
      }
    }
    lds_barrier();
    if (!on) continue;
    // outlier corrections of this tile: channel tid sums its 16 copies in a fixed order,
    // carries the result like the output, and clears the copies for the next tile
    if (kwave < KS) {
      int4* c4 = (int4*)&S.xc[ktid][0];
      const int r0 = (ktid >> 1) & 3, r1 = (r0 + 1) & 3, r2 = (r0 + 2) & 3, r3 = (r0 + 3) & 3;   // bank-staggered order
      const int4 x0 = c4[r0], x1 = c4[r1], x2 = c4[r2], x3 = c4[r3];
      const int4 z = {0, 0, 0, 0};
      c4[r0] = z; c4[r1] = z; c4[r2] = z; c4[r3] = z;
      // each copy is below 2^30 in magnitude: pairs are summed exactly as integers, then in fp32
      const float sum = (((float)(x0.x + x0.y) + (float)(x0.z + x0.w)) + ((float)(x1.x + x1.y) + (float)(x1.z + x1.w))) +
                        (((float)(x2.x + x2.y) + (float)(x2.z + x2.w)) + ((float)(x3.x + x3.y) + (float)(x3.z + x3.w)));
      c_run = c_run * keep + sum * ldexpf(wscale, 3);     // wscale = 2^(wexp-28)
    }

    // ---- values: integer contractions, rows 0..3 of the tile = the four digits of w -----------
    v4i cv[CGW];
#pragma unroll
    for (int j = 0; j < CGW; ++j) cv[j] = zero4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      if (blk * 64 < n32V) {
        const v4i wa = *(const v4i*)(wb2 + 64 * blk);
#pragma unroll
        for (int j = 0; j < CGW; ++j) cv[j] = mma(wa, spread<2>(&vr.vw2[blk][j], 0), cv[j]);
      }
      if (blk * 64 < cV.n3) {
        const v4i wa = *(const v4i*)(wb1 + 64 * blk);
#pragma unroll
        for (int j = 0; j < CGW; ++j) cv[j] = mma(wa, spread<1>(&vr.vw1[blk], (CGW * wave + j) & 1), cv[j]);
      }
    }
    for (int blk = 0; blk * 64 < cV.n4; ++blk) {
      const int u = blk * 4 + g;                 // 16 slots = half-units 2u, 2u+1
      const int nhu = (cV.n4 + 7) >> 3;
      uint32_t w0[CGW], w1d[CGW];
      // a half-unit past the end repeats the last one; its slots carry zero digits
      gload_dwords<CGW>(baseV + (rV.r4 + (uint32_t)min(2 * u, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave), w0);
      gload_dwords<CGW>(baseV + (rV.r4 + (uint32_t)min(2 * u + 1, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave), w1d);
      const v4i wa = *(const v4i*)(wb4 + 64 * blk);
#pragma unroll
      for (int j = 0; j < CGW; ++j) {
        const uint32_t pr[2] = {w0[j], w1d[j]};
        cv[j] = mma(wa, spread<4>(pr, 0), cv[j]);
      }
    }
    if (H1) {                                              // 1-bit tokens: units in the format of the 1-bit fields
      const int nu = (cV.n1 + 15) >> 4, nb3 = (((cV.n3 + 15) >> 4) + 3) >> 2;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        if (blk * 64 < cV.n1) {
          uint32_t w1b = vr.vw1[3 - blk];                  // came with the tile if the entry was free, else fetched here
          if (3 - blk < nb3)
            w1b = gload32(baseV, rV.r1b + (uint32_t)min(blk * 4 + g, nu - 1) * (2u * D) +
                                 (uint32_t)nn * (NCG * 2) + 4u * ((CGW * wave) >> 1));
          const v4i wa = *(const v4i*)(wb1b + 64 * blk);
#pragma unroll
          for (int j = 0; j < CGW; ++j) cv[j] = mma(wa, spread<1>(&w1b, (CGW * wave + j) & 1), cv[j]);
        }
      }
    }
    // 8-bit codes: token-major bytes, plain fp32 multiply-add; this wavefront's D/4 channels,
    // lane = (token sub-index, 4 channels)
    if (cV.n8 > 0) {
      constexpr int LPT8 = D / 16;         // lanes per token (4 channels each)
      constexpr int TPW = 64 / LPT8;       // tokens per pass
      float a8[4] = {0.f, 0.f, 0.f, 0.f};
      const int sub = lane / LPT8, ch4 = lane % LPT8;
      // rows sub, sub + TPW, ...: the first one and a batch of four are requested at once, and every further
      // batch while the one before it is summed (a row past the end repeats the last one and gets weight 0);
      // a tile of a cache the rules shaped rarely has more rows than the first covers
      constexpr int UB = 4;
      const uint32_t lane8 = (D / 4) * wave + 4 * ch4;
      auto row8 = [&](int i8) { return gload32(baseV, rV.r8 + (uint32_t)min(i8, cV.n8 - 1) * D + lane8); };
      const uint32_t dw0 = row8(sub);
      uint32_t cur[UB];
#pragma unroll
      for (int u = 0; u < UB; ++u) cur[u] = row8(sub + (1 + u) * TPW);
      {
        const float w8 = sub < cV.n8 ? S.w8[sub] : 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) a8[j] += w8 * (float)((dw0 >> (8 * j)) & 255u);
      }
#pragma unroll 1
      for (int i0 = sub + TPW; i0 < cV.n8; i0 += UB * TPW) {
        uint32_t nxt[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) nxt[u] = row8(i0 + (UB + u) * TPW);
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int i8 = i0 + u * TPW;
          const float w8 = i8 < cV.n8 ? S.w8[min(i8, QAQ_TT - 1)] : 0.0f;
#pragma unroll
          for (int j = 0; j < 4; ++j) a8[j] += w8 * (float)((cur[u] >> (8 * j)) & 255u);
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) cur[u] = nxt[u];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float t = a8[j];
#pragma unroll
        for (int o = LPT8; o < 64; o <<= 1) t += __shfl_xor(t, o);
        if (sub == 0) S.xw[wave][4 * ch4 + j] = t;
      }
    }
    // lanes of group 0 hold rows 0..3 = digit sums of channel 16*(CGW*wave + j) + n
    if (g == 0) {
#pragma unroll
      for (int j = 0; j < CGW; ++j) {
        const float hi = (float)cv[j][3] * 2097152.0f + (float)cv[j][2] * 16384.0f;   // base-128 digits
        const float lo = (float)cv[j][1] * 128.0f + (float)cv[j][0];
        const int chl = 16 * j + nn;                   // channel inside this wavefront's share
        float xt = (hi + lo) * wscale;
        if (cV.n8 > 0) xt += S.xw[wave][chl];
        xrun[j] = xrun[j] * keep + xt;
      }
    }
    // the value registers are free: request the next tile's values
    if (tile + 1 < tile_end) vr.template load<H1>(v, len, b, h, tile + 1, counts_of(tile + 1, 1), tid, wave, nn, g);
  }

  // ---- one partial per workgroup -----------------------------------------------------------------
  {
    const float ls = wave_sum(l_run);
    const float bs = wave_sum(bias_run);
    if (lane == 0) { S.red[wave] = ls; S.red[4 + wave] = bs; }
    if (kwave < KS) S.xcorr[ktid] = c_run;
  }
  lds_barrier();
  const float lsum = (S.red[0] + S.red[1]) + (S.red[2] + S.red[3]);
  const float bias = (S.red[4] + S.red[5]) + (S.red[6] + S.red[7]);
  float* part = P ? &S.part[0] : a.partial + ((size_t)bq * a.part_stride + chunk) * (D + 4);
  if (g == 0) {
#pragma unroll
    for (int j = 0; j < CGW; ++j) part[(D / 4) * wave + 16 * j + nn] = xrun[j] + bias + S.xcorr[(D / 4) * wave + 16 * j + nn];
  }
  if (tid == 0) { part[D] = m_run; part[D + 1] = lsum; }
  if (!P) return;

  // ---- fused form: merge the P parts, add the new token, normalise, write -----------------------
  lds_barrier();
  const TileLds<D>& S0 = S_all[0];
  float a_new = -INFINITY;
  if (a.k_new) a_new = ((S0.red[12] + S0.red[13]) + (S0.red[14] + S0.red[15])) / sqrtf((float)D);   // the unquantized new token's logit
  float Mx = a_new;
#pragma unroll
  for (int p = 0; p < (P ? P : 1); ++p) Mx = fmaxf(Mx, S_all[p].part[D]);
  float fac[P ? P : 1];
  float ltot = 0.0f;
#pragma unroll
  for (int p = 0; p < (P ? P : 1); ++p) { fac[p] = __expf(S_all[p].part[D] - Mx); ltot += fac[p] * S_all[p].part[D + 1]; }
  float e_new = 0.0f;
  if (a.k_new) { e_new = __expf(a_new - Mx); ltot += e_new; }
  const float inv = 1.0f / ltot;
  if (chunk == 0 && tid < D) {
    float x = 0.0f;
#pragma unroll
    for (int p = 0; p < (P ? P : 1); ++p) x += fac[p] * S_all[p].part[tid];
    if (a.k_new) x += e_new * S0.newv[tid];
    if (a.out_is_fp32) ((float*)a.out)[(size_t)bq * D + tid] = x * inv;
    else ((__half*)a.out)[(size_t)bq * D + tid] = __float2half_rn(x * inv);
  }
  if (a.scores) {
    float* sc = a.scores + (size_t)bq * a.score_stride;
    for (int it = 0; it < tile_end - tile_begin; ++it) {
      const int t = (tile_begin + it) * QAQ_TT + tid;
      if (t < len) {
        const float raw = LDS_LOGITS ? lg_all[((chunk * a.ntc + it) << 8) + tid] : ((volatile float*)sc)[t];
        sc[t] = __expf(raw - Mx) * inv;
      }
    }
    if (a.k_new && chunk == 0 && tid == 0) sc[len] = e_new * inv;
  }
}

// ---------------------------------------------------------------------------------------
// Grouped queries: one pass over a KV head's codes for four query heads at a time.
//
// k_attn_tile gives every query head its own scan, so the G heads that share a KV head unpack
// the same codes and decode the same per-token metadata G times.  Here a part (256 threads)
// serves kHG = 4 query heads of one KV head: the 16 rows of the A operand are 4 heads x
// (3 query digits + an empty row) on the key side and 4 heads x 4 weight digits on the value
// side, the B operand -- the unpacked codes -- is shared, and so are min/scale, order bytes
// and outlier entries of every token.  On the key side column n of a product is token n of a
// group of 16, lane (n, g) supplies 16 channels of it (its k-range) and receives head g's
// digit sums for it; on the value side the rows are summed over 64 slots and lane (n, g)
// receives head g's digit sums for channel n.  Parts write partials (max, sum, X) per query
// head and raw logits; k_attn_combine merges them.  Width sets without 1, the fixed-length
// side store with one outlier per end or none; G a multiple of 4 (a KV head with 8 query
// heads is scanned twice, by two workgroups that run side by side).
// ---------------------------------------------------------------------------------------
constexpr int kHG = 4;

template <int D>
struct GqaLds {
  // (rows of the two tables that the four lanes of a token address together -- one head each, the same
  // column -- are eight words longer than their payload, so that the four land in different banks)
  float qf[kHG][D + 8];
  // query digits [format][head][digit][position in record order]; "digit" 3 is a row of zeros, the fourth
  // A row of every head on the key side, so that a lane's row has the same place in all three formats
  // (one address register, the formats at constant offsets)
  alignas(16) int8_t ql[3][kHG][4][D + 16];
  alignas(16) uint16_t cnt[QAQ_MAX_NTC][8];
  float vb[QAQ_MAX_NTC];
  float logit[kHG][QAQ_TT + 8];                // raw logits by position; at the very end: outlier corrections by channel
  alignas(16) int8_t wl2[kHG][4][QAQ_TT + 16];  // weight digits [head][digit][slot of the 2-bit field region]
  alignas(16) int8_t wl1[kHG][4][QAQ_TT + 16];
  alignas(16) int8_t wl4[kHG][4][QAQ_TT + 16];
  float w8[kHG][QAQ_TT];                       // fp32 weights of the 8-bit slots
  float xw[4][kHG][D / 4];                     // per wavefront: 8-bit-class outputs of its own channels
  alignas(16) uint32_t v8[4][64];              // per wavefront: 64 / (D/16) rows of 8-bit values, its D/4 channels of each
  alignas(16) int xc[kHG][D][4];               // outlier corrections of one tile, fixed point, four copies per channel
  alignas(16) float red[4][kHG];               // per wavefront and head
  alignas(16) float red2[4][kHG];
  int sq[kHG];                                 // per head: sum of the unscaled query integers (8-bit keys are stored as code - 128)
};

template <int D, int NO2>
__global__ __launch_bounds__(kThreads, 3) void k_attn_gqa(QaqAttnArgs a) {
  constexpr int KS = D / 64;
  constexpr int NCG = D / 16;
  constexpr int CGW = NCG / 4;
  __shared__ GqaLds<D> S;
  const QaqView& v = a.v;
  const int chunk = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nn = lane & 15, g = lane >> 4;
  const int NG = a.G / kHG;
  const int unit = blockIdx.y;
  const int b = unit / (v.Hkv * NG), h = (unit / NG) % v.Hkv, hg = unit % NG;
  const int bq0 = b * v.Hq + h * a.G + kHG * hg;           // first of the four query heads
  const int len = qaq_seq_len(v, b, a.len);          // cached tokens of this sequence
  const int ntile = (len + QAQ_TT - 1) / QAQ_TT;
  const int tile_begin = (int)((long long)chunk * ntile / a.nparts);
  const int tile_end = (int)((long long)(chunk + 1) * ntile / a.nparts);
  if (tile_begin >= tile_end) {
    // a sequence shorter than the longest can leave a part without tiles: partials that the merge ignores
    for (int e = tid; e < kHG * (D + 2); e += kThreads) {
      float* part = a.partial + ((size_t)(bq0 + e / (D + 2)) * a.part_stride + chunk) * (D + 4);
      const int c = e % (D + 2);
      part[c] = c == D ? -INFINITY : 0.0f;
    }
    return;
  }
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const v4i zero4 = {0, 0, 0, 0};

  float qv[kHG];
#pragma unroll
  for (int j = 0; j < kHG; ++j) qv[j] = tid < D ? __half2float(a.q[(size_t)(bq0 + j) * D + tid]) : 0.0f;
  if (tid < tile_end - tile_begin) {
    *(uint4*)&S.cnt[tid][0] = *(const uint4*)(v.counts + ((qaq_bh(v, b, h) * v.NT + tile_begin + tid) * 2) * 4);
    S.vb[tid] = v.vbound[qaq_bh(v, b, h) * v.NT + tile_begin + tid];
  }
  if (wave < KS) {
#pragma unroll
    for (int j = 0; j < kHG; ++j) {
      const float am = wave_max(fabsf(qv[j]));
      const float sm = wave_sum(qv[j]);
      if (lane == 0) { S.red[wave][j] = am; S.red2[wave][j] = sm; }
      S.qf[j][tid] = qv[j];
    }
  }
  for (int e = tid; e < 3 * kHG * (D + 16); e += kThreads) S.ql[e / (kHG * (D + 16))][(e / (D + 16)) % kHG][3][e % (D + 16)] = 0;
  if (tid < kHG) S.sq[tid] = 0;
  for (int e = tid; e < kHG * D * 4; e += kThreads) (&S.xc[0][0][0])[e] = 0;
  lds_barrier();

  auto counts_of = [&](int t, int side) {
    const uint2 c = *(const uint2*)&S.cnt[t - tile_begin][4 * side];
    const uint32_t lo = __builtin_amdgcn_readfirstlane(c.x), hi = __builtin_amdgcn_readfirstlane(c.y);
    QaqCounts r;
    r.n3 = lo & 0xffffu; r.n2 = lo >> 16; r.n4 = hi & 0xffffu; r.n8 = hi >> 16; r.n1 = 0;
    return r;
  };

  // ---- what is loaded ahead for the key side: lane (n, g) holds, for each of its wavefront's four
  // groups of 16 slots, the slices g*KS .. g*KS+KS-1 of slot 16*tg + n; the metadata of a slot is
  // held once, by lane 16*tg + n (slot = lane index), and handed to the other three lanes that work
  // on the token (one per head) when its group is processed ----------------------------------------
  uint32_t ka[4][KS], kb[4][KS], kmm, kpos, koi, kov;
  QaqCounts cKn;
  int n_tok_n = 0;
  auto load_keys = [&](int tile) {
    cKn = counts_of(tile, 0);
    n_tok_n = min(len - tile * QAQ_TT, QAQ_TT);
    const gbytes_t ubase = uniform_ptr(qaq_tile_codes(v, 0, b, h, tile));
    const size_t gi0 = qaq_slot_index(v, b, h, tile, 0);
    const QaqKRegions rK = qaq_k_regions(cKn, D);
    const int n32 = cKn.n32();
    {
      const int so = min(64 * wave + lane, n_tok_n - 1);
      kmm = gload32(uniform_ptr(v.mm[0] + gi0), 4u * (uint32_t)so);
      kpos = gload32(uniform_ptr(v.perm[0] + gi0), (uint32_t)so & ~3u);
      if (NO2 == 2) {
        koi = gload32(uniform_ptr(v.oidx[0] + gi0 * 2), (2u * (uint32_t)so) & ~3u);
        kov = gload32(uniform_ptr(v.oval[0] + gi0 * 2), 4u * (uint32_t)so);
      }
    }
#pragma unroll
    for (int tg = 0; tg < 4; ++tg) {
      const int s = min(64 * wave + 16 * tg + nn, n_tok_n - 1);
      const bool is3 = s < cKn.n3, is23 = s < n32, is4 = !is23 && s < n32 + cKn.n4;
      const uint32_t rec4 = rK.r4 + (uint32_t)(s - n32) * (uint32_t)(D / 2) + (uint32_t)g * (8u * KS);
      const uint32_t off_a = is23 ? (uint32_t)s * (uint32_t)(D / 4) + (uint32_t)g * (4u * KS) : is4 ? rec4 : 0u;
      // the low bits of a 3-bit token: the word that holds the lane's slices (KS = 2: both halves of
      // word g; KS = 1: one half of word g / 2); a 4-bit token: the second half of its slices
      const uint32_t off_b = is3 ? rK.r1 + (uint32_t)s * (uint32_t)(D / 8) + 4u * (uint32_t)((g * KS) >> 1) : is4 ? rec4 + 4u * KS : 0u;
      gload_dwords<KS>(ubase + off_a, ka[tg]);
      gload_dwords<KS>(ubase + off_b, kb[tg]);
    }
  };
  ValRegs<D, NO2> vr;
  load_keys(tile_begin);
  vr.template load<false, true>(v, len, b, h, tile_begin, counts_of(tile_begin, 1), tid, wave, nn, g);

  // ---- query digits: 22-bit fixed point per head, three signed base-256 digits, one table per
  // spreading format ---------------------------------------------------------------------------------
  float qscale_g = 0.0f, sumq_g = 0.0f;        // of the lane's own head g
#pragma unroll
  for (int j = 0; j < kHG; ++j) {
    const float qmax = KS == 1 ? S.red[0][j] : fmaxf(S.red[0][j], S.red[1][j]);
    const float sumq = KS == 1 ? S.red2[0][j] : S.red2[0][j] + S.red2[1][j];
    int qexp = 0;
    if (qmax > 0.0f) (void)frexpf(qmax, &qexp);
    const float qscale = qmax > 0.0f ? ldexpf(1.0f, qexp - 22) : 0.0f;
    if (j == g) { qscale_g = qscale; sumq_g = sumq; }
    if (wave < KS) {
      const int i = tid & 15, vgr = i >> 2;
      const int pos = 16 * (((tid & 63) >> 4) * KS + (tid >> 6)) + i;
#pragma unroll
      for (int f = 0; f < 3; ++f) {
        const int sh = f == 0 ? shift2(vgr) : f == 1 ? shift1(vgr) : 0;
        const int x = qmax > 0.0f ? (int)rintf(ldexpf(qv[j], 22 - qexp - sh)) : 0;
        const uint32_t dg = digits_packed(x);
        S.ql[f][j][0][pos] = (int8_t)dg; S.ql[f][j][1][pos] = (int8_t)(dg >> 8); S.ql[f][j][2][pos] = (int8_t)(dg >> 16);
        if (f == 2) atomicAdd(&S.sq[j], x);        // integers: the order of the additions does not matter
      }
    }
  }
  lds_barrier();
  // A rows: row r = 4 * head + digit; the lane's k-range is slices g*KS ..
  const int arow_h = nn >> 2, arow_d = nn & 3;
  const int8_t* abase0 = &S.ql[0][arow_h][arow_d][16 * g * KS];
  const int8_t* abase1 = abase0 + sizeof(S.ql[0]);
  const int8_t* abase2 = abase0 + 2 * sizeof(S.ql[0]);
  const int8_t* wb2 = &S.wl2[arow_h][arow_d][16 * g];
  const int8_t* wb1 = wb2 + sizeof(S.wl2);       // the three tables have one shape and follow one another
  const int8_t* wb4 = wb2 + 2 * sizeof(S.wl2);
  static_assert(offsetof(GqaLds<D>, wl1) - offsetof(GqaLds<D>, wl2) == sizeof(S.wl2) &&
                offsetof(GqaLds<D>, wl4) - offsetof(GqaLds<D>, wl2) == 2 * sizeof(S.wl2), "weight digit tables are contiguous");
  auto real_of = [&](const v4i& c) { return (((float)c[2] * 65536.0f + (float)c[1] * 256.0f) + (float)c[0]) * qscale_g; };

  float m_run[kHG], l_run[kHG], bias_run[kHG];
#pragma unroll
  for (int j = 0; j < kHG; ++j) { m_run[j] = -INFINITY; l_run[j] = 0.0f; bias_run[j] = 0.0f; }
  constexpr int NCR = (kHG * D + kThreads - 1) / kThreads;      // (head, channel) pairs per thread for the outlier corrections
  float c_run[NCR];
#pragma unroll
  for (int r = 0; r < NCR; ++r) c_run[r] = 0.0f;
  float xrun[CGW];                 // head g, channel 16*(CGW*wave + j) + n
#pragma unroll
  for (int j = 0; j < CGW; ++j) xrun[j] = 0.0f;

  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const QaqCounts cK = cKn, cV = vr.c;
    const int n_tok = n_tok_n;
    const QaqKRegions rK = qaq_k_regions(cK, D);
    const QaqVRegions rV = qaq_v_regions(cV, D);
    // (scalar base + 32-bit lane offset: a 64-bit address per lane would cost the loop two registers each)
    const gbytes_t baseK = uniform_ptr(qaq_tile_codes(v, 0, b, h, tile));
    const gbytes_t baseV = uniform_ptr(qaq_tile_codes(v, 1, b, h, tile));
    const int n32K = cK.n32(), n32V = cV.n32();
    const int first8K = n32K + cK.n4, first8V = n32V + cV.n4;

    // ---- keys: logits of the lane's head for the four tokens 16*tg + n of its wavefront ---------------
    // What depends on the token only is worked out once, by the lane that holds the slot's metadata
    // (slot = lane index), not by each of the four lanes that work on the token: min, scale, the two
    // outlier corrections, and (one word) the outlier channels and the position.
    float t_mn, t_scale, t_c0 = 0.0f, t_c1 = 0.0f;
    uint32_t t_idx;
    {
      const int so = 64 * wave + lane;
      const float mx = h2f((uint16_t)(kmm >> 16));
      t_mn = h2f((uint16_t)(kmm & 0xffffu));
      t_scale = ldexpf(mx - t_mn, -cK.bits_of_slot4(min(so, n_tok - 1)));
      t_idx = ((kpos >> (8u * ((uint32_t)so & 3u))) & 0xffu) << 16;
      if (NO2 == 2) {
        const float hs = 0.5f * t_scale;
        const float o0 = h2f((uint16_t)(kov & 0xffffu)), o1 = h2f((uint16_t)(kov >> 16));
        const bool top0 = o0 >= mx, top1 = o1 >= mx;
        t_c0 = (o0 - (top0 ? mx : t_mn)) + (top0 ? hs : -hs);
        t_c1 = (o1 - (top1 ? mx : t_mn)) + (top1 ? hs : -hs);
        t_idx |= (koi >> (16 * (so & 1))) & 0xffffu;
      }
    }
    float vmax = -INFINITY;
#pragma unroll
    for (int tg = 0; tg < 4; ++tg) {
      const int s0 = 64 * wave + 16 * tg;           // uniform
      if (s0 >= n_tok) continue;
      const int s = s0 + nn;
      float dotq = 0.0f;
      if (s0 < n32K) {
        v4i c = zero4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) c = mma(*(const v4i*)(abase0 + 16 * ks), spread<2>(&ka[tg][ks], 0), c);
        dotq = real_of(c);
        if (s0 < cK.n3) {
          v4i c1 = zero4;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) c1 = mma(*(const v4i*)(abase1 + 16 * ks), spread<1>(&kb[tg][0], (g * KS + ks) & 1), c1);
          const float low = real_of(c1);
          dotq = s < cK.n3 ? 2.0f * dotq + low : dotq;
        }
      }
      if (s0 + 16 > n32K && s0 < first8K) {
        uint32_t k4[2 * KS];
#pragma unroll
        for (int i = 0; i < KS; ++i) { k4[i] = ka[tg][i]; k4[KS + i] = kb[tg][i]; }
        v4i c = zero4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) c = mma(*(const v4i*)(abase2 + 16 * ks), spread<4>(&k4[2 * ks], 0), c);
        const float d4 = real_of(c);
        if (s >= n32K) dotq = d4;
      }
      if (cK.n8 > 0 && s0 + 16 > first8K) {
        // 8-bit keys (rare): fetched here; stored as code - 128, so the product gets 128 * (sum of the
        // head's query integers) back, rebuilt from the digits
        const int i8 = min(max(s - first8K, 0), max(cK.n8 - 1, 0));
        uint32_t w8r[4 * KS];
        gload_dwords<4 * KS>(baseK + (rK.r8 + (uint32_t)i8 * D + (uint32_t)g * (16u * KS)), w8r);
        const int sq = S.sq[g];
        v4i c = zero4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) c = mma(*(const v4i*)(abase2 + 16 * ks), spread<8>(&w8r[4 * ks], 0), c);
        if (s >= first8K) dotq = ((((float)c[2] * 65536.0f + (float)c[1] * 256.0f) + (float)c[0]) + 128.0f * (float)sq) * qscale_g;
      }
      // metadata of slot s from the lane that holds it (every lane takes part in the exchange)
      const int src = 4 * (16 * tg + nn);
      const float mn = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(t_mn)));
      const float scale = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(t_scale)));
      const uint32_t idx = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)t_idx);
      float c0 = 0.0f, c1 = 0.0f;
      if (NO2 == 2) {
        c0 = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(t_c0)));
        c1 = __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(t_c1)));
      }
      if (s < n_tok) {
        float val = mn * sumq_g + scale * (dotq + 0.5f * sumq_g);
        if (NO2 == 2) {
          val += S.qf[g][idx & 0xffu] * c0;
          val += S.qf[g][(idx >> 8) & 0xffu] * c1;
        }
        const float lg = val * inv_sqrt_d;
        S.logit[g][idx >> 16] = lg;
        vmax = vmaxf(vmax, lg);
      }
    }
    if (tile + 1 < tile_end) load_keys(tile + 1);

    // maximum of the lane's head over its row of 16 lanes, then over the wavefronts
    asm volatile(QAQ_DPP_STEP("v_max_f32_dpp", "quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
                 QAQ_DPP_STEP("v_max_f32_dpp", "quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
                 QAQ_DPP_STEP("v_max_f32_dpp", "row_half_mirror row_mask:0xf bank_mask:0xf")
                 QAQ_DPP_STEP("v_max_f32_dpp", "row_mirror row_mask:0xf bank_mask:0xf")
                 "s_nop 1"
                 : "+v"(vmax));
    if (nn == 0) S.red[wave][g] = vmax;
    lds_barrier();
    float M[kHG], keep[kHG];
    {
      const float4 r0 = *(const float4*)&S.red[0][0], r1 = *(const float4*)&S.red[1][0];
      const float4 r2 = *(const float4*)&S.red[2][0], r3 = *(const float4*)&S.red[3][0];
      const float mt[kHG] = {vmaxf(vmaxf(r0.x, r1.x), vmaxf(r2.x, r3.x)), vmaxf(vmaxf(r0.y, r1.y), vmaxf(r2.y, r3.y)),
                             vmaxf(vmaxf(r0.z, r1.z), vmaxf(r2.z, r3.z)), vmaxf(vmaxf(r0.w, r1.w), vmaxf(r2.w, r3.w))};
#pragma unroll
      for (int j = 0; j < kHG; ++j) {
        M[j] = vmaxf(m_run[j], mt[j]);
        keep[j] = __expf(m_run[j] - M[j]);
        m_run[j] = M[j];
      }
    }
    const float smax = S.vb[tile - tile_begin];
    int wexp = 0;
    if (smax > 0.0f) (void)frexpf(smax, &wexp);
    const float wscale = smax > 0.0f ? ldexpf(1.0f, wexp - 28) : 0.0f;
    if (a.scores && tid < n_tok) {
#pragma unroll
      for (int j = 0; j < kHG; ++j) a.scores[(size_t)(bq0 + j) * a.score_stride + tile * QAQ_TT + tid] = S.logit[j][tid];
    }

    // ---- values: the four heads' weights of slot `tid`, as digits ---------------------------------------
    {
      const int s = tid;
      const bool live = s < n_tok;
      const uint32_t slot = (uint32_t)min(tid, n_tok - 1);
      const int posv = (int)((vr.pos >> (8u * (slot & 3u))) & 0xffu);
      const float mn = h2f((uint16_t)(vr.mm & 0xffffu)), mx = h2f((uint16_t)(vr.mm >> 16));
      const float range = mx - mn;
      const float scale = ldexpf(range, -cV.bits_of_slot4(s));
      const float hs = 0.5f * scale;
      float corr[2] = {0.0f, 0.0f};
      int och[2] = {0, 0};
      if (NO2 == 2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const float ovf = vr.o.val(j);
          const bool top = ovf >= mx;
          corr[j] = (ovf - (top ? mx : mn)) + (top ? hs : -hs);
          och[j] = vr.o.idx(j, slot);
        }
      }
      const bool fx = live && smax > 0.0f;
      const int vg = (s & 15) >> 2;
      const int i4 = (s - n32V) & (QAQ_TT - 1);
#pragma unroll
      for (int j = 0; j < kHG; ++j) {
        float pt = 0.0f, w = 0.0f;
        if (live) {
          pt = __expf(S.logit[j][posv] - M[j]);
          w = pt * scale;
          if (NO2 == 2) {
#pragma unroll
            for (int k = 0; k < 2; ++k)
              atomicAdd(&S.xc[j][och[k]][lane & 3], (int)rintf(ldexpf(pt * corr[k], 25 - wexp)));
          }
          if (s >= first8V) S.w8[j][s - first8V] = w;
        }
        l_run[j] = l_run[j] * keep[j] + pt;
        bias_run[j] = bias_run[j] * keep[j] + (pt * mn + 0.5f * w);
        const uint32_t W2 = (fx && s < n32V) ? (uint32_t)rintf(ldexpf(w, 28 - wexp - shift2(vg) + (s < cV.n3 ? 1 : 0))) : 0u;
        S.wl2[j][0][s] = (int8_t)(W2 & 127u); S.wl2[j][1][s] = (int8_t)((W2 >> 7) & 127u);
        S.wl2[j][2][s] = (int8_t)((W2 >> 14) & 127u); S.wl2[j][3][s] = (int8_t)(W2 >> 21);
        // (the value phase reads these two tables in blocks of 64 slots, as far as the class reaches:
        // slots of later blocks need no digits, not even zeros)
        if (s < ((cV.n3 + 63) & ~63)) {
          const uint32_t W1 = (fx && s < cV.n3) ? (uint32_t)rintf(ldexpf(w, 28 - wexp - shift1(vg))) : 0u;
          S.wl1[j][0][s] = (int8_t)(W1 & 127u); S.wl1[j][1][s] = (int8_t)((W1 >> 7) & 127u);
          S.wl1[j][2][s] = (int8_t)((W1 >> 14) & 127u); S.wl1[j][3][s] = (int8_t)(W1 >> 21);
        }
        if (i4 < ((cV.n4 + 63) & ~63)) {
          const uint32_t W4 = (fx && s >= n32V && s < first8V) ? (uint32_t)rintf(ldexpf(w, 28 - wexp)) : 0u;
          S.wl4[j][0][i4] = (int8_t)(W4 & 127u); S.wl4[j][1][i4] = (int8_t)((W4 >> 7) & 127u);
          S.wl4[j][2][i4] = (int8_t)((W4 >> 14) & 127u); S.wl4[j][3][i4] = (int8_t)(W4 >> 21);
        }
      }
    }
    lds_barrier();
    // outlier corrections of this tile: (head, channel) pairs sum their copies and clear them
    if (NO2 == 2) {
#pragma unroll
      for (int r = 0; r < NCR; ++r) {
        const int item = tid + kThreads * r;
        if (item < kHG * D) {
          const int j = item / D;
          int4* c4 = (int4*)&S.xc[0][0][0] + item;
          const int4 x = *c4;
          *c4 = make_int4(0, 0, 0, 0);
          const float kp = j == 0 ? keep[0] : j == 1 ? keep[1] : j == 2 ? keep[2] : keep[3];
          c_run[r] = c_run[r] * kp + ((float)(x.x + x.y) + (float)(x.z + x.w)) * ldexpf(wscale, 3);
        }
      }
    }

    // ---- values: integer contractions, rows = 4 heads x 4 weight digits ----------------------------------
    v4i cv[CGW];
#pragma unroll
    for (int j = 0; j < CGW; ++j) cv[j] = zero4;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      if (blk * 64 < n32V) {
        const v4i wa = *(const v4i*)(wb2 + 64 * blk);
#pragma unroll
        for (int j = 0; j < CGW; ++j) cv[j] = mma(wa, spread<2>(&vr.vw2[blk][j], 0), cv[j]);
      }
      if (blk * 64 < cV.n3) {
        const v4i wa = *(const v4i*)(wb1 + 64 * blk);
#pragma unroll
        for (int j = 0; j < CGW; ++j) cv[j] = mma(wa, spread<1>(&vr.vw1[blk], (CGW * wave + j) & 1), cv[j]);
      }
    }
    // 4-bit values.  Up to 16 of them in a tile (the usual case where the rules chose the widths):
    // their two half-units came with the tile, one word per lane; the lanes of group 0, whose 16
    // slots these are, collect the four words (the other groups' slots carry zero digits, so what
    // they pass as codes does not matter).  More: fetched here.
    const bool few4 = CGW == 2 && cV.n4 <= 16;
    if (few4 && cV.n4 > 0) {
      if constexpr (CGW == 2) {
        const uint32_t d00 = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * nn, (int)vr.v4p);
        const uint32_t d10 = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (nn + 16), (int)vr.v4p);
        const uint32_t d01 = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (nn + 32), (int)vr.v4p);
        const uint32_t d11 = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (nn + 48), (int)vr.v4p);
        const v4i wa = *(const v4i*)wb4;
        const uint32_t p0[2] = {d00, d01}, p1[2] = {d10, d11};
        cv[0] = mma(wa, spread<4>(p0, 0), cv[0]);
        cv[1] = mma(wa, spread<4>(p1, 0), cv[1]);
      }
    }
    for (int blk = 0; !few4 && blk * 64 < cV.n4; ++blk) {
      const int u = blk * 4 + g;
      const int nhu = (cV.n4 + 7) >> 3;
      uint32_t w0[CGW], w1d[CGW];
      gload_dwords<CGW>(baseV + (rV.r4 + (uint32_t)min(2 * u, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave), w0);
      gload_dwords<CGW>(baseV + (rV.r4 + (uint32_t)min(2 * u + 1, nhu - 1) * (4u * D) + (uint32_t)nn * (NCG * 4) + 4u * CGW * wave), w1d);
      const v4i wa = *(const v4i*)(wb4 + 64 * blk);
#pragma unroll
      for (int j = 0; j < CGW; ++j) {
        const uint32_t pr[2] = {w0[j], w1d[j]};
        cv[j] = mma(wa, spread<4>(pr, 0), cv[j]);
      }
    }
    if (cV.n8 > 0) {
      // 8-bit values: token-major bytes, fp32 multiply-add; this wavefront's D/4 channels.  Rows go
      // through the wavefront's own LDS block, 64 / (D/16) at a time (the first batch came with the
      // tile, further ones -- rare -- are fetched here), so that a lane can own a channel and sum
      // over the rows by itself: lane (c, half) = channel c of heads 2*half and 2*half + 1.  (No
      // reduction across lanes: a chain of cross-lane exchanges per head cost more than all the
      // arithmetic of this class.)  Needs D/4 <= 32 channels per wavefront, i.e. D <= 128.
      constexpr int LPT8 = D / 16;
      constexpr int TPW = 64 / LPT8;
      static_assert(D / 4 <= 32, "a wavefront's channels must fit half its lanes");
      const int c8 = lane & 31, h0 = 2 * (lane >> 5);
      const uint8_t* rows = (const uint8_t*)&S.v8[wave][0];
      float acc0 = 0.0f, acc1 = 0.0f;
      for (int r0 = 0; r0 < cV.n8; r0 += TPW) {
        uint32_t dw = vr.v8;
        if (r0 > 0) dw = gload32(baseV, rV.r8 + (uint32_t)min(r0 + lane / LPT8, cV.n8 - 1) * D + (D / 4) * wave + 4 * (lane % LPT8));
        S.v8[wave][lane] = dw;        // row lane / LPT8, bytes 4 * (lane % LPT8) .. +3: a row is D/4 consecutive bytes
        // (LDS operations of one wavefront complete in order: no barrier between the write and the reads)
        const int nr = min(cV.n8 - r0, TPW);
#pragma unroll
        for (int r = 0; r < TPW; ++r) {
          if (r < nr && c8 < D / 4) {
            const float x = (float)rows[r * (D / 4) + c8];
            acc0 += S.w8[h0][r0 + r] * x;
            acc1 += S.w8[h0 + 1][r0 + r] * x;
          }
        }
      }
      if (c8 < D / 4) { S.xw[wave][h0][c8] = acc0; S.xw[wave][h0 + 1][c8] = acc1; }
    }
    {
      const float kp = g == 0 ? keep[0] : g == 1 ? keep[1] : g == 2 ? keep[2] : keep[3];
#pragma unroll
      for (int j = 0; j < CGW; ++j) {
        const float hi = (float)cv[j][3] * 2097152.0f + (float)cv[j][2] * 16384.0f;
        const float lo = (float)cv[j][1] * 128.0f + (float)cv[j][0];
        float xt = (hi + lo) * wscale;
        if (cV.n8 > 0) xt += S.xw[wave][g][16 * j + nn];
        xrun[j] = xrun[j] * kp + xt;
      }
    }
    if (tile + 1 < tile_end) vr.template load<false, true>(v, len, b, h, tile + 1, counts_of(tile + 1, 1), tid, wave, nn, g);
  }

  // ---- one partial per query head -------------------------------------------------------------------------
  lds_barrier();          // the last tile's logits and digits are done with
#pragma unroll
  for (int j = 0; j < kHG; ++j) {
    const float ls = wave_sum(l_run[j]);
    const float bs = wave_sum(bias_run[j]);
    if (lane == 0) { S.red[wave][j] = ls; S.red2[wave][j] = bs; }
  }
#pragma unroll
  for (int r = 0; r < NCR; ++r) {
    const int item = tid + kThreads * r;
    if (item < kHG * D) S.logit[item / D][item % D] = c_run[r];
  }
  lds_barrier();
  {
    const float lsum = (S.red[0][g] + S.red[1][g]) + (S.red[2][g] + S.red[3][g]);
    const float bias = (S.red2[0][g] + S.red2[1][g]) + (S.red2[2][g] + S.red2[3][g]);
    float* part = a.partial + ((size_t)(bq0 + g) * a.part_stride + chunk) * (D + 4);
#pragma unroll
    for (int j = 0; j < CGW; ++j) {
      const int ch = (D / 4) * wave + 16 * j + nn;
      part[ch] = xrun[j] + bias + S.logit[g][ch];
    }
    const float mg = g == 0 ? m_run[0] : g == 1 ? m_run[1] : g == 2 ? m_run[2] : m_run[3];
    if (wave == 0 && nn == 0) { part[D] = mg; part[D + 1] = lsum; }
  }
}

// Merge the tiles of one (sequence, query head), add the unquantized new token and
// normalise.  Block x = 0 writes the output vector; every block normalises its share of
// the emitted scores (each recomputes the head's max and sum from the per-tile pairs).
// All global loads are issued before the first reduction.
template <int D, int EPT>      // EPT: scores per thread of a block
__global__ __launch_bounds__(kThreads) void k_attn_combine(QaqAttnArgs a) {
  constexpr int MAXP = 4;                    // per-tile pairs held per lane (256 tiles); more: loop
  __shared__ float red[8];
  const QaqView& v = a.v;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bq = blockIdx.y, b = bq / v.Hq, hq = bq % v.Hq, h = hq / a.G;
  const int nparts = a.nparts;
  const int len = qaq_seq_len(v, b, a.len);          // cached tokens of this sequence
  const float* part = a.partial + (size_t)bq * a.part_stride * (D + 4);
  float* sc = a.scores ? a.scores + (size_t)bq * a.score_stride : nullptr;
  const int t0 = blockIdx.x * (EPT * kThreads);
  float raw[EPT];
#pragma unroll
  for (int k = 0; k < EPT; ++k) raw[k] = 0.0f;
  if (sc) {
#pragma unroll
    for (int k = 0; k < EPT; ++k) {
      const int t = t0 + k * kThreads + tid;
      if (t < len) raw[k] = sc[t];
    }
  }
  float pm[MAXP], pl[MAXP];
#pragma unroll
  for (int k = 0; k < MAXP; ++k) {
    const int i = lane + 64 * k;
    pm[k] = i < nparts ? part[(size_t)i * (D + 4) + D] : -INFINITY;
    pl[k] = i < nparts ? part[(size_t)i * (D + 4) + D + 1] : 0.0f;
  }
  float qk = 0.0f;
  if (a.k_new && tid < D) qk = __half2float(a.q[(size_t)bq * D + tid]) * __half2float(a.k_new[((size_t)b * v.Hkv + h) * D + tid]);

  float a_new = -INFINITY;
  if (a.k_new) {
    qk = wave_sum(qk);
    if (lane == 0) red[wave] = qk;
    __syncthreads();
    a_new = ((red[0] + red[1]) + (red[2] + red[3])) / sqrtf((float)D);
  }
  float M = a_new;
#pragma unroll
  for (int k = 0; k < MAXP; ++k) M = fmaxf(M, pm[k]);
  for (int i = lane + 64 * MAXP; i < nparts; i += 64) M = fmaxf(M, part[(size_t)i * (D + 4) + D]);
  M = wave_max(M);
  float lsum = 0.0f;
#pragma unroll
  for (int k = 0; k < MAXP; ++k) lsum += __expf(pm[k] - M) * pl[k];
  for (int i = lane + 64 * MAXP; i < nparts; i += 64)
    lsum += __expf(part[(size_t)i * (D + 4) + D] - M) * part[(size_t)i * (D + 4) + D + 1];
  lsum = wave_sum(lsum);
  float e_new = 0.0f;
  if (a.k_new) { e_new = __expf(a_new - M); lsum += e_new; }
  const float inv = 1.0f / lsum;
  if (sc) {
#pragma unroll
    for (int k = 0; k < EPT; ++k) {
      const int t = t0 + k * kThreads + tid;
      if (t < len) sc[t] = __expf(raw[k] - M) * inv;
    }
  }
  if (blockIdx.x == 0) {
    // output vector: wavefront w takes tiles w, w+4, ..., lanes take channels; several
    // independent loads in flight per lane, then a fixed-order sum over the wavefronts
    __shared__ float fac[64 * MAXP];
    __shared__ float xacc[4][D];
    if (wave == 0) {
#pragma unroll
      for (int k = 0; k < MAXP; ++k) fac[lane + 64 * k] = __expf(pm[k] - M);
    }
    __syncthreads();
    float acc[D / 64];
#pragma unroll
    for (int c = 0; c < D / 64; ++c) acc[c] = 0.0f;
#pragma unroll 4
    for (int i = wave; i < nparts; i += 4) {
      const float f = i < 64 * MAXP ? fac[i] : __expf(part[(size_t)i * (D + 4) + D] - M);
#pragma unroll
      for (int c = 0; c < D / 64; ++c) acc[c] += f * part[(size_t)i * (D + 4) + lane + 64 * c];
    }
#pragma unroll
    for (int c = 0; c < D / 64; ++c) xacc[wave][lane + 64 * c] = acc[c];
    __syncthreads();
    if (tid < D) {
      float x = (xacc[0][tid] + xacc[1][tid]) + (xacc[2][tid] + xacc[3][tid]);
      if (a.k_new) x += e_new * __half2float(a.v_new[((size_t)b * v.Hkv + h) * D + tid]);
      if (a.out_is_fp32) ((float*)a.out)[(size_t)bq * D + tid] = x * inv;
      else ((__half*)a.out)[(size_t)bq * D + tid] = __float2half_rn(x * inv);
    }
    if (sc && a.k_new && tid == 0) sc[len] = e_new * inv;
  }
}

// P = 0: grid (nparts, B*Hq), k_attn_combine follows.  P = nparts in 1..4: grid (1, B*Hq),
// workgroups of 256*P threads, lds = bytes of the raw-logit store.
// e0, e1: NULL, or events that take the start and the end of this dispatch.
template <int D, int P>
void launch_tile_p(const QaqAttnArgs& a, dim3 grid, size_t lds, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  const dim3 block((P == 5 ? 4 : P ? P : 1) * kThreads);
  if (a.v.has1) {
    if (a.v.no2 == 2 && !a.v.csr) hipExtLaunchKernelGGL((k_attn_tile<D, 2, P, true>), grid, block, lds, s, e0, e1, 0, a);
    else if (a.v.no2 == 0) hipExtLaunchKernelGGL((k_attn_tile<D, 0, P, true>), grid, block, lds, s, e0, e1, 0, a);
    else hipExtLaunchKernelGGL((k_attn_tile<D, 8, P, true>), grid, block, lds, s, e0, e1, 0, a);
    return;
  }
  if (a.v.no2 == 2 && !a.v.csr) hipExtLaunchKernelGGL((k_attn_tile<D, 2, P, false>), grid, block, lds, s, e0, e1, 0, a);   // (the variable-length side store runs in the general form)
  else if (a.v.no2 == 0) hipExtLaunchKernelGGL((k_attn_tile<D, 0, P, false>), grid, block, lds, s, e0, e1, 0, a);
  else hipExtLaunchKernelGGL((k_attn_tile<D, 8, P, false>), grid, block, lds, s, e0, e1, 0, a);
}
template <int D>
void launch_tile(const QaqAttnArgs& a, int fused_parts, int BQ, size_t lds, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  switch (fused_parts) {
    case 1: launch_tile_p<D, 1>(a, dim3(1, BQ), lds, s, e0, e1); break;
    case 2: launch_tile_p<D, 2>(a, dim3(1, BQ), lds, s, e0, e1); break;
    case 3: launch_tile_p<D, 3>(a, dim3(1, BQ), lds, s, e0, e1); break;
    case 4: launch_tile_p<D, 4>(a, dim3(1, BQ), lds, s, e0, e1); break;
    case 5: launch_tile_p<D, 5>(a, dim3(1, BQ), 0, s, e0, e1); break;      // four parts, raw logits in the score buffer
    default: launch_tile_p<D, 0>(a, dim3(a.nparts, BQ), 0, s, e0, e1); break;
  }
}

// Scratch for callers that must not allocate (qaq_decode_attention_static): the partial results
// of the two-kernel form.  One copy per GPU the library runs on, held until the process ends;
// host code reaches it only through the address hipGetSymbolAddress returns for the current
// device (the array's name is a host-side stand-in, not a device address).
constexpr size_t kStaticScratchBytes = 1u << 20;
__attribute__((used)) static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];        // per device, filled at the first use on that device

hipError_t static_scratch_ptr(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

size_t qaq_static_scratch_bytes() { return kStaticScratchBytes; }

hipError_t qaq_launch_attention(const QaqAttnArgs& a_in, hipStream_t s, hipEvent_t* ev, int* kernels,
                                bool static_scratch, bool* too_big) {
  QaqAttnArgs a = a_in;
  a.partial = a.v.partial;
  a.part_stride = a.v.NT;
  if (too_big) *too_big = false;
  const int ntile = (a.len + QAQ_TT - 1) / QAQ_TT;
  const int BQ = a.v.B * a.v.Hq;
  // parts per (sequence, query head): as many as keep the whole grid resident at once (four
  // workgroups per compute unit), so that no second, partly filled round of workgroups trails
  // the first; every part gets floor or ceil of ntile/nparts tiles
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
    if (n_cu <= 0) n_cu = 256;
  }
  // grouped queries: four query heads of a KV head per pass (k_attn_gqa), where the cache has that form
  const bool gqa = a.G >= kHG && a.G % kHG == 0 && !a.v.has1 && !a.v.csr && (a.v.no2 == 2 || a.v.no2 == 0);
  const int units = gqa ? BQ / kHG : BQ;
  const int slots = (gqa ? 3 : 4) * n_cu;
  const int per_head = slots / units > 0 ? slots / units : 1;
  a.nparts = ntile < per_head ? ntile : per_head;
  const int least = (ntile + QAQ_MAX_NTC - 1) / QAQ_MAX_NTC;    // a part holds at most QAQ_MAX_NTC tiles
  if (a.nparts < least) a.nparts = least;
  a.ntc = a.nparts > 0 ? (ntile + a.nparts - 1) / a.nparts : 0;
  // Fused form (no second kernel) when the parts of a head fit one workgroup; their raw logits stay
  // in its LDS next to the parts' working blocks if they fit, else they wait in the score buffer.
  // (its parts run in lockstep and every one needs a tile: where the sequences differ in length, the
  // shortest must have as many tiles as a head has parts)
  const int ntile_shortest = (a.len_shortest + QAQ_TT - 1) / QAQ_TT;
  a.lds_logits = a.nparts * a.ntc <= kFusedMaxTiles || !a.scores;
  const bool fused = !gqa && ntile > 0 && a.nparts <= 4 && (!a.v.ragged || ntile_shortest >= a.nparts) &&
                     (a.lds_logits || a.nparts == 4);
  if (kernels) *kernels = ntile > 0 ? (fused ? 1 : 2) : 0;
  if (static_scratch && !fused) {
    if ((size_t)BQ * (size_t)(a.nparts > 0 ? a.nparts : 1) * (a.v.D + 4) * sizeof(float) > kStaticScratchBytes) {
      if (too_big) *too_big = true;
      return hipSuccess;
    }
    void* p = nullptr;
    const hipError_t e = static_scratch_ptr(&p);
    if (e != hipSuccess) return e;
    a.partial = (float*)p;
    a.part_stride = a.nparts > 0 ? a.nparts : 1;
  }
  if (ntile > 0 && gqa) {
    const dim3 grid(a.nparts, units), block(kThreads);
    hipEvent_t e0 = ev ? ev[0] : nullptr, e1 = ev ? ev[1] : nullptr;
    if (a.v.D == 128) {
      if (a.v.no2 == 2) hipExtLaunchKernelGGL((k_attn_gqa<128, 2>), grid, block, 0, s, e0, e1, 0, a);
      else hipExtLaunchKernelGGL((k_attn_gqa<128, 0>), grid, block, 0, s, e0, e1, 0, a);
    } else {
      if (a.v.no2 == 2) hipExtLaunchKernelGGL((k_attn_gqa<64, 2>), grid, block, 0, s, e0, e1, 0, a);
      else hipExtLaunchKernelGGL((k_attn_gqa<64, 0>), grid, block, 0, s, e0, e1, 0, a);
    }
  } else if (ntile > 0) {
    const int fp = fused ? (a.lds_logits ? a.nparts : 5) : 0;
    const size_t lds = fused && a.scores && a.lds_logits ? (size_t)a.nparts * a.ntc * QAQ_TT * sizeof(float) : 0;
    if (a.v.D == 128) launch_tile<128>(a, fp, BQ, lds, s, ev ? ev[0] : nullptr, ev ? ev[1] : nullptr);
    else launch_tile<64>(a, fp, BQ, lds, s, ev ? ev[0] : nullptr, ev ? ev[1] : nullptr);
  }
  if (fused) return hipGetLastError();
  // scores per block: every block repeats the head's merge (partial maxima and sums, the new token's
  // logit) before it normalises its share, so longer shares where there are blocks enough
  const int ept = (long long)BQ * a.len >= 16ll * kThreads * 1024 ? 16 : 4;
  const int nblk = a.scores ? (a.len + ept * kThreads - 1) / (ept * kThreads) : 1;
  dim3 grid(nblk < 1 ? 1 : nblk, BQ);
  hipEvent_t c0 = ev && ntile > 0 ? ev[2] : nullptr, c1 = ev && ntile > 0 ? ev[3] : nullptr;
  if (a.v.D == 128) {
    if (ept == 16) hipExtLaunchKernelGGL((k_attn_combine<128, 16>), grid, dim3(kThreads), 0, s, c0, c1, 0, a);
    else hipExtLaunchKernelGGL((k_attn_combine<128, 4>), grid, dim3(kThreads), 0, s, c0, c1, 0, a);
  } else {
    if (ept == 16) hipExtLaunchKernelGGL((k_attn_combine<64, 16>), grid, dim3(kThreads), 0, s, c0, c1, 0, a);
    else hipExtLaunchKernelGGL((k_attn_combine<64, 4>), grid, dim3(kThreads), 0, s, c0, c1, 0, a);
  }
  return hipGetLastError();
}

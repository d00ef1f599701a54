// Device memory layout of the quantized cache (shared by every kernel of libqaq).
//
// The sequence of one (batch, KV head) is cut into tiles of TT = 256 positions.
// Inside a tile, separately for keys and for values, tokens are ordered by code
// width: first the 3-bit tokens, then the 2-bit, 4-bit, 8-bit and 1-bit ones ("slots";
// perm[slot] = position inside the tile).  Per-token metadata (min/max, perm,
// outlier side store) is stored in slot order, so a kernel that walks the slots
// reads it coalesced.  Codes are stored per width class in operand-ready form for
// the int8 matrix/dot instructions:
//
//   R2  2-bit fields: every 2-bit token's code and the top two bits of every 3-bit
//       token's code (slots [0, n3+n2))
//   R1  1-bit fields: the low bit of every 3-bit token (slots [0, n3))
//   R4  4-bit codes, R8 8-bit codes
//   R1b 1-bit codes of the 1-bit tokens, in the format of R1 (its index starts at the
//       first 1-bit slot); the class sits last so that a cache whose width set has no 1
//       is laid out as if the class did not exist
//
// A 3-bit code c is thus 2*top + low, which makes narrowing 3 -> 2 a matter of
// dropping R1, and lets the attention kernels treat the planes as two separate
// integer dot products.
//
// Keys ("K side"): one contiguous record per token (D*bf/8 bytes), made of
// "slices" of 16 channels: slice q = g*KS + ks covers channels 64*ks + 16*g + i,
// i = 0..15 (KS = D/64).  Lane group g of a wavefront reads slices g*KS .. g*KS+KS-1.
//
// Values ("V side"): transposed in units of 16 tokens so that four bytes of a
// register are four consecutive tokens of one channel (the contraction of S.V runs
// over tokens).  8-bit values are kept token-major (one byte per channel).
//
// Element i (0..15) of a slice sits at:
//   bf=2: dword q,            bit 8*(i%4) + 2*(i/4)
//   bf=1: dword q/2, nibble h=q%2: bit 8*(i%4) + 4*h + (i/4)
//   bf=4: dword 2q + i/8,     bit 8*(i%4) + 4*((i/4)%2)
//   bf=8: dword 4q + i/4,     byte i%4   (keys store code ^ 0x80 = code-128 as int8)
// so that ((w >> k) & mask) yields four consecutive elements as four bytes.
#pragma once
#include <stdint.h>

#define QAQ_TT 256           // positions per tile
#define QAQ_MAX_NO2 8        // 2 * max outliers per side

#if defined(__HIPCC__)
#define QAQ_HD __host__ __device__ __forceinline__
#else
#define QAQ_HD inline
#endif

// class order inside a tile
enum { QC3 = 0, QC2 = 1, QC4 = 2, QC8 = 3, QC1 = 4, QAQ_NCLASS = 5 };

QAQ_HD int qaq_class_of_bits(int b) { return b == 3 ? QC3 : b == 2 ? QC2 : b == 4 ? QC4 : b == 8 ? QC8 : QC1; }
QAQ_HD int qaq_bits_of_class(int c) { return c == QC3 ? 3 : c == QC2 ? 2 : c == QC4 ? 4 : c == QC8 ? 8 : 1; }

// Tokens per class.  Only the first four are stored per tile side; n1 is what remains of
// the tile's tokens.
struct QaqCounts {
  int n3, n2, n4, n8, n1;
  QAQ_HD int n32() const { return n3 + n2; }
  QAQ_HD int first1() const { return n3 + n2 + n4 + n8; }
  QAQ_HD int total() const { return n3 + n2 + n4 + n8 + n1; }
  QAQ_HD int count(int cls) const { return cls == QC3 ? n3 : cls == QC2 ? n2 : cls == QC4 ? n4 : cls == QC8 ? n8 : n1; }
  QAQ_HD int start(int cls) const {
    return cls == QC3 ? 0 : cls == QC2 ? n3 : cls == QC4 ? n3 + n2 : cls == QC8 ? n3 + n2 + n4 : n3 + n2 + n4 + n8;
  }
  QAQ_HD int bits_of_slot(int s) const { return s < n3 ? 3 : s < n3 + n2 ? 2 : s < n3 + n2 + n4 ? 4 : s < n3 + n2 + n4 + n8 ? 8 : 1; }
  // the same where the width set is known to have no 1 (kernels specialised on that)
  QAQ_HD int bits_of_slot4(int s) const { return s < n3 ? 3 : s < n3 + n2 ? 2 : s < n3 + n2 + n4 ? 4 : 8; }
};

QAQ_HD uint32_t qaq_align16(uint32_t x) { return (x + 15u) & ~15u; }

// ---- K side region offsets (bytes from the tile-side base) -------------------
struct QaqKRegions {
  uint32_t r2, r1, r4, r8, r1b, end;
};
QAQ_HD QaqKRegions qaq_k_regions(const QaqCounts& c, int D) {
  QaqKRegions r;
  // every region is sized for a multiple of 16 records, so that appending a token or moving
  // one between width classes leaves the regions behind it where they are 15 times out of 16
  r.r2 = 0;
  r.r1 = (uint32_t)((c.n32() + 15) / 16) * 16u * (D / 4);
  r.r4 = r.r1 + (uint32_t)((c.n3 + 15) / 16) * 16u * (D / 8);
  r.r8 = r.r4 + (uint32_t)((c.n4 + 15) / 16) * 16u * (D / 2);
  r.r1b = r.r8 + (uint32_t)c.n8 * D;
  r.end = r.r1b + (uint32_t)((c.n1 + 15) / 16) * 16u * (D / 8);
  return r;
}
// worst case: 252 8-bit records and one partly filled group of 16 in each other region
QAQ_HD uint32_t qaq_k_cap(int D) { return QAQ_TT * D + 16 * D; }

// ---- V side region offsets ----------------------------------------------------
struct QaqVRegions {
  uint32_t r2, r1, r4, r8, r1b, end;
};
QAQ_HD QaqVRegions qaq_v_regions(const QaqCounts& c, int D) {
  QaqVRegions r;
  r.r2 = 0;
  r.r1 = (uint32_t)((c.n32() + 15) / 16) * (4 * D);
  r.r4 = r.r1 + (uint32_t)((c.n3 + 15) / 16) * (2 * D);
  r.r8 = r.r4 + (uint32_t)((c.n4 + 7) / 8) * (4 * D);
  r.r1b = r.r8 + (uint32_t)c.n8 * D;
  r.end = r.r1b + (uint32_t)((c.n1 + 15) / 16) * (2 * D);
  return r;
}
QAQ_HD uint32_t qaq_v_cap(int D) { return QAQ_TT * D + 16 * D; }

// ---- where one code field lives ------------------------------------------------
struct QaqFieldPos {
  uint32_t byte_off;  // byte offset of the dword, from the tile-side base
  int shift;          // bit position of the field inside the dword
};

// element i of a slice -> bit position inside its dword(s); *dw = dword index inside the slice
QAQ_HD int qaq_elem_bit(int bf, int i, int h, int* dw) {
  int j = i & 3, v = i >> 2;
  if (bf == 2) { *dw = 0; return 8 * j + 2 * v; }
  if (bf == 1) { *dw = 0; return 8 * j + 4 * h + v; }
  if (bf == 4) { *dw = v >> 1; return 8 * j + 4 * (v & 1); }
  *dw = v; return 8 * j;
}

// K side: field of width bf for the token at index `idx` of region with base `roff`,
// channel d.
QAQ_HD QaqFieldPos qaq_k_field(uint32_t roff, int bf, int idx, int d, int D) {
  const int KS = D / 64;
  int ks = d / 64, g = (d % 64) / 16, i = d % 16;
  int q = g * KS + ks;
  int dw;
  QaqFieldPos p;
  uint32_t rec = roff + (uint32_t)idx * (uint32_t)(D * bf / 8);
  if (bf == 1) {
    p.shift = qaq_elem_bit(1, i, q & 1, &dw);
    p.byte_off = rec + 4u * (uint32_t)(q >> 1);
  } else {
    p.shift = qaq_elem_bit(bf, i, 0, &dw);
    p.byte_off = rec + 4u * (uint32_t)(q * (bf / 2) + dw);
  }
  return p;
}

// V side, transposed regions (bf = 2, 1, 4): token index `idx` inside the region, channel d.
QAQ_HD QaqFieldPos qaq_v_field(uint32_t roff, int bf, int idx, int d, int D) {
  int n = d % 16, cg = d / 16;
  QaqFieldPos p;
  int dw;
  if (bf == 2) {
    int u = idx / 16, i = idx % 16;
    p.shift = qaq_elem_bit(2, i, 0, &dw);
    p.byte_off = roff + (uint32_t)u * (4u * D) + 4u * (uint32_t)(n * (D / 16) + cg);
  } else if (bf == 1) {
    int u = idx / 16, i = idx % 16;
    p.shift = qaq_elem_bit(1, i, cg & 1, &dw);
    p.byte_off = roff + (uint32_t)u * (2u * D) + 4u * (uint32_t)(n * (D / 32) + (cg >> 1));
  } else {  // bf == 4: half-units of 8 tokens
    int hu = idx / 8, i = idx % 8;
    p.shift = 8 * (i & 3) + 4 * (i >> 2);
    p.byte_off = roff + (uint32_t)hu * (4u * D) + 4u * (uint32_t)(n * (D / 16) + cg);
  }
  return p;
}

// ---- arena carving --------------------------------------------------------------
struct QaqDims {
  int B, Hq, Hkv, D, Tmax, NT, no2, window;
  int ring_half;      // the window's rows: 0 fp32, 1 fp16, 2 bf16
  int csr;            // outliers by thresholds: variable-length side store
};

struct QaqArena {
  // byte offsets from the arena base (all 256-byte aligned)
  size_t codes[2];    // [side][B][Hkv][NT][cap]
  size_t mm[2];       // u32  [B][Hkv][Tmax]   min | max<<16, slot order inside each tile
  size_t perm[2];     // u8   [B][Hkv][Tmax]
  size_t oidx[2];     // u8   [B][Hkv][Tmax][no2]
  size_t oval[2];     // u16  [B][Hkv][Tmax][no2]
  size_t tags[2];     // u8   [B][Hkv][Tmax]   width by position
  size_t counts;      // u16  [B][Hkv][NT][2][4]
  size_t vbound;      // f32  [B][Hkv][NT]   per tile: bound on (value scale, outlier correction) over its tokens
  size_t kthr;        // f32  [B][Hkv][NT][2] per tile: key-rule thresholds [lo, hi) for which no token changes width
  size_t ring;        // f32 (or fp16) [window][B][Hkv][Tmax]
  size_t partial;     // f32  [B][Hq][NT][D+4]
  size_t statbuf;     // i64  [32]
  size_t refused;     // u32  [B][Hkv][NT][2 sides][2] widenings refused / served, counted per tile side by the
                      // workgroup that owns it (plain read-modify-write: no atomics)
  size_t todo;        // u32  [B][Hkv][NT][2] tile sides a decode-step update leaves to the general build kernel
  size_t todo_count;  // u32  [2]
  // variable-length side store (outliers by thresholds) only: oidx / oval are then per-tile pools
  // of 256 * no2 entries filled in position order
  size_t ostart[2];   // u16  [B][Hkv][Tmax]  by position: first entry of the token in its tile's pool
  size_t ocnt[2];     // u8   [B][Hkv][Tmax]  by position: entries of the token
  size_t othr;        // f32  [2][Hkv][2]     thresholds (lo, hi) per side and KV head
  size_t total;
};

QAQ_HD size_t qaq_up256(size_t x) { return (x + 255) & ~(size_t)255; }

inline QaqArena qaq_carve(const QaqDims& d) {
  QaqArena a;
  size_t off = 0;
  size_t bh = (size_t)d.B * d.Hkv;
  size_t cap[2] = {qaq_k_cap(d.D), qaq_v_cap(d.D)};
  for (int s = 0; s < 2; ++s) { a.codes[s] = off; off = qaq_up256(off + bh * d.NT * cap[s]); }
  for (int s = 0; s < 2; ++s) { a.mm[s] = off; off = qaq_up256(off + bh * d.Tmax * 4); }
  for (int s = 0; s < 2; ++s) { a.perm[s] = off; off = qaq_up256(off + bh * d.Tmax); }
  for (int s = 0; s < 2; ++s) { a.oidx[s] = off; off = qaq_up256(off + bh * d.Tmax * (size_t)(d.no2 ? d.no2 : 1)); }
  for (int s = 0; s < 2; ++s) { a.oval[s] = off; off = qaq_up256(off + bh * d.Tmax * 2 * (size_t)(d.no2 ? d.no2 : 1)); }
  for (int s = 0; s < 2; ++s) { a.tags[s] = off; off = qaq_up256(off + bh * d.Tmax); }
  a.counts = off; off = qaq_up256(off + bh * d.NT * 2 * 4 * 2);
  a.vbound = off; off = qaq_up256(off + bh * d.NT * 4);
  a.kthr = off; off = qaq_up256(off + bh * d.NT * 8);
  a.ring = off; off = qaq_up256(off + (size_t)d.window * bh * d.Tmax * (d.ring_half ? 2 : 4));
  a.partial = off; off = qaq_up256(off + (size_t)d.B * d.Hq * d.NT * (d.D + 4) * 4);
  a.statbuf = off; off = qaq_up256(off + 32 * 8);
  a.refused = off; off = qaq_up256(off + bh * d.NT * 2 * 2 * 4);
  a.todo = off; off = qaq_up256(off + bh * d.NT * 2 * 4);
  a.todo_count = off; off = qaq_up256(off + 2 * 4);
  a.ostart[0] = a.ostart[1] = a.ocnt[0] = a.ocnt[1] = a.othr = 0;
  if (d.csr) {
    for (int s = 0; s < 2; ++s) { a.ostart[s] = off; off = qaq_up256(off + bh * d.Tmax * 2); }
    for (int s = 0; s < 2; ++s) { a.ocnt[s] = off; off = qaq_up256(off + bh * d.Tmax); }
    a.othr = off; off = qaq_up256(off + (size_t)2 * d.Hkv * 2 * 4);
  }
  a.total = off;
  return a;
}

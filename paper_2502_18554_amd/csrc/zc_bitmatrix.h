// In-register bit-matrix transposes: the step between 32 sign-magnitude deltas of a block and
// its sign + plane words (Section 3.3: sign bits and the fixed-length "bit-shifting" encoding).
//
// One lane owns one block.  Plane word p has bit j = bit p of value j, so the plane words are
// the transpose of the 32 x 32 bit matrix whose rows are the values.  A transpose by
// recursive block swaps costs six simple operations per pair of words and stage, for all
// planes at once, where gathering plane by plane costs one operation per value and plane.
// Blocks are narrow most of the time, so the matrix is first folded:
//   width <= 7  : four values per word (bytes), three stages on 8 words
//   width <= 15 : two values per word (halves), four stages on 16 words
//   wider       : the 16-bit form twice, for the low and the high half of the magnitudes
// The sign rides as the top bit of each value's field and comes out as the last row.
// The same swaps undo themselves, so decompression runs the identical transposes.
//
// Everything here is plain integer C++ so that the host tests can exercise it too.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define ZC_HD __host__ __device__
#else
#define ZC_HD
#endif

namespace zc {

// Exchanges, between words a and b, the bit groups selected by mask m (in b) and m << s (in a).
ZC_HD inline void swap_bits(uint32_t& a, uint32_t& b, int s, uint32_t m) {
  const uint32_t t = ((a >> s) ^ b) & m;
  b ^= t;
  a ^= t << s;
}

// Transposes the 16 x 16 bit matrix in the low halves of r[0..16) and, independently, the
// one in the high halves: afterwards bit j of half h of r[p] is what bit p of half h of r[j] was.
ZC_HD inline void transpose16x16_pairs(uint32_t (&r)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((j & 8) == 0) swap_bits(r[j], r[j + 8], 8, 0x00FF00FFu);
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((j & 4) == 0) swap_bits(r[j], r[j + 4], 4, 0x0F0F0F0Fu);
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((j & 2) == 0) swap_bits(r[j], r[j + 2], 2, 0x33333333u);
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((j & 1) == 0) swap_bits(r[j], r[j + 1], 1, 0x55555555u);
}

// Transposes the four 8 x 8 bit matrices in the bytes of r[0..8).
ZC_HD inline void transpose8x8_quads(uint32_t (&r)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if ((j & 4) == 0) swap_bits(r[j], r[j + 4], 4, 0x0F0F0F0Fu);
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if ((j & 2) == 0) swap_bits(r[j], r[j + 2], 2, 0x33333333u);
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if ((j & 1) == 0) swap_bits(r[j], r[j + 1], 1, 0x55555555u);
}

// ---- values -> planes -------------------------------------------------------------------
// d[j] = delta j in two's complement.  The planes hold its magnitude; the sign word its sign.

// Field of `bits` bits: magnitude in the low bits - 1, sign in the top bit.
template <int BITS>
ZC_HD inline uint32_t sign_magnitude_field(int32_t d) {
  const uint32_t m = uint32_t(d >> 31);
  const uint32_t mag = (uint32_t(d) ^ m) - m;
  return (mag & ((1u << (BITS - 1)) - 1u)) | (m & (1u << (BITS - 1)));
}
template <int BITS>
ZC_HD inline int32_t delta_from_field(uint32_t f) {
  const uint32_t m = 0u - ((f >> (BITS - 1)) & 1u);
  const uint32_t mag = f & ((1u << (BITS - 1)) - 1u);
  return int32_t((mag ^ m) - m);
}

// Widths up to 7: out[0..7) = planes 0..6, out[7] = sign word.
ZC_HD inline void planes_from_deltas8(const int32_t (&d)[32], uint32_t (&out)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) w |= sign_magnitude_field<8>(d[j + 8 * k]) << (8 * k);
    out[j] = w;
  }
  transpose8x8_quads(out);
}

// 16-bit fields, two per word: word j holds value j in its low half and value j + 16 in its
// high half.  This is the form the compression kernel keeps a block in once its deltas are
// known: half the registers of the deltas themselves.
ZC_HD inline uint32_t field16_pair(int32_t lo, int32_t hi) {
  return sign_magnitude_field<16>(lo) | (sign_magnitude_field<16>(hi) << 16);
}

// Widths up to 15, from the paired fields, in place: f[0..15) = planes 0..14, f[15] = sign word.
ZC_HD inline void planes16_from_fields(uint32_t (&f)[16]) { transpose16x16_pairs(f); }

// Widths up to 7, from the paired 16-bit fields: out[0..7) = planes 0..6, out[7] = sign word.
// The fields are narrowed to 8 bits (sign moved from bit 15 to bit 7), four per word.
ZC_HD inline void planes8_from_fields16(const uint32_t (&f)[16], uint32_t (&out)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t a = (f[j] & 0x007F007Fu) | ((f[j] >> 8) & 0x00800080u);          // values j, j + 16
    const uint32_t b = (f[j + 8] & 0x007F007Fu) | ((f[j + 8] >> 8) & 0x00800080u);  // values j + 8, j + 24
    out[j] = a | (b << 8);
  }
  transpose8x8_quads(out);
}

// Widths up to 15: out[0..15) = planes 0..14, out[15] = sign word.
ZC_HD inline void planes_from_deltas16(const int32_t (&d)[32], uint32_t (&out)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) out[j] = field16_pair(d[j], d[j + 16]);
  planes16_from_fields(out);
}

// Any width: lo[0..16) = planes 0..15; hi[0..15) = planes 16..30, hi[15] = sign word.
ZC_HD inline void planes_from_deltas32(const int32_t (&d)[32], uint32_t (&lo)[16], uint32_t (&hi)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const uint32_t a = sign_magnitude_field<32>(d[j]), b = sign_magnitude_field<32>(d[j + 16]);
    lo[j] = (a & 0xFFFFu) | (b << 16);
    hi[j] = (a >> 16) | (b & 0xFFFF0000u);
  }
  transpose16x16_pairs(lo);
  transpose16x16_pairs(hi);
}

// ---- planes -> values -------------------------------------------------------------------

ZC_HD inline void deltas_from_planes8(uint32_t (&in)[8], int32_t (&d)[32]) {
  transpose8x8_quads(in);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
#pragma unroll
    for (int k = 0; k < 4; ++k) d[j + 8 * k] = delta_from_field<8>((in[j] >> (8 * k)) & 0xFFu);
  }
}

ZC_HD inline void deltas_from_planes16(uint32_t (&in)[16], int32_t (&d)[32]) {
  transpose16x16_pairs(in);
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    d[j] = delta_from_field<16>(in[j] & 0xFFFFu);
    d[j + 16] = delta_from_field<16>(in[j] >> 16);
  }
}

ZC_HD inline void deltas_from_planes32(uint32_t (&lo)[16], uint32_t (&hi)[16], int32_t (&d)[32]) {
  transpose16x16_pairs(lo);
  transpose16x16_pairs(hi);
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    d[j] = delta_from_field<32>((lo[j] & 0xFFFFu) | (hi[j] << 16));
    d[j + 16] = delta_from_field<32>((lo[j] >> 16) | (hi[j] & 0xFFFF0000u));
  }
}

}  // namespace zc

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
// Narrow values enter as two's complement fields, so the sign comes out as the last row and
// the conversion between two's complement and sign + magnitude happens on the planes.
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
// The stage that exchanges whole bytes (shift 8, mask 0x00FF00FF): bytes 1 and 3 of a with bytes 0
// and 2 of b.  On the GPU that is two byte permutes instead of five bit operations.
ZC_HD inline void swap_bytes_stage(uint32_t& a, uint32_t& b) {
#if defined(__HIP_DEVICE_COMPILE__)
  const uint32_t na = __builtin_amdgcn_perm(b, a, 0x06020400u);     // a0 b0 a2 b2
  const uint32_t nb = __builtin_amdgcn_perm(b, a, 0x07030501u);     // a1 b1 a3 b3
  a = na;
  b = nb;
#else
  swap_bits(a, b, 8, 0x00FF00FFu);
#endif
}

ZC_HD inline void transpose16x16_pairs(uint32_t (&r)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if ((j & 8) == 0) swap_bytes_stage(r[j], r[j + 8]);
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

// ---- two's complement <-> sign + magnitude, on planes -------------------------------------
// r[0..N-1) = planes of N-bit two's complement values (one bit of 32 values per word), r[N-1]
// their sign plane.  Negating where the sign is set, with a ripple of carries over the planes,
// turns them into magnitude planes and back: three operations per plane for 32 values, where
// the same conversion value by value costs five operations per value.
template <int N>
ZC_HD inline void twos_planes_to_magnitude(uint32_t (&r)[N]) {
  const uint32_t s = r[N - 1];
  uint32_t carry = s;                       // (bits ^ s) + s
#pragma unroll
  for (int p = 0; p < N - 1; ++p) {
    const uint32_t t = r[p] ^ s;
    r[p] = t ^ carry;
    carry &= t;
  }
}
// The inverse is the same operation: negate the magnitudes where the sign is set.
template <int N>
ZC_HD inline void magnitude_planes_to_twos(uint32_t (&r)[N]) { twos_planes_to_magnitude<N>(r); }

// Low 16 bits of two values in one word / low 8 bits of four values in one word.
ZC_HD inline uint32_t pack16(uint32_t lo, uint32_t hi) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
#else
  return (lo & 0xFFFFu) | (hi << 16);
#endif
}
// From two words of paired 16-bit fields (values a, c and b, d): bytes a, b, c, d.
ZC_HD inline uint32_t narrow_pairs_to_bytes(uint32_t ac, uint32_t bd) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_perm(bd, ac, 0x06020400u);
#else
  return (ac & 0xFFu) | ((bd & 0xFFu) << 8) | (((ac >> 16) & 0xFFu) << 16) | (((bd >> 16) & 0xFFu) << 24);
#endif
}

// ---- values -> planes -------------------------------------------------------------------
// d[j] = delta j in two's complement.  The planes hold its magnitude; the sign word its sign.
// Narrow blocks go through two's complement fields (a plain truncation of the delta), the
// bit-matrix transpose, and the conversion to magnitudes on the planes.

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

// Paired 16-bit two's complement fields: word j holds delta j in its low half and delta
// j + 16 in its high half (exact for |delta| < 2^15).  This is the form the compression
// kernel keeps a block in once its deltas are known: half the registers of the deltas.
ZC_HD inline uint32_t field16_pair(int32_t lo, int32_t hi) { return pack16(uint32_t(lo), uint32_t(hi)); }

// Widths up to 15, from the paired fields, in place: f[0..15) = planes 0..14, f[15] = sign word.
ZC_HD inline void planes16_from_fields(uint32_t (&f)[16]) {
  transpose16x16_pairs(f);
  twos_planes_to_magnitude<16>(f);
}

// Widths up to 7, from the paired 16-bit fields: out[0..7) = planes 0..6, out[7] = sign word.
// The fields are narrowed to 8 bits, four per word (byte k of word j = delta j + 8k).
ZC_HD inline void planes8_from_fields16(const uint32_t (&f)[16], uint32_t (&out)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) out[j] = narrow_pairs_to_bytes(f[j], f[j + 8]);
  transpose8x8_quads(out);
  twos_planes_to_magnitude<8>(out);
}

// Widths up to 7: out[0..7) = planes 0..6, out[7] = sign word.
ZC_HD inline void planes_from_deltas8(const int32_t (&d)[32], uint32_t (&out)[8]) {
  uint32_t f[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) f[j] = field16_pair(d[j], d[j + 16]);
  planes8_from_fields16(f, out);
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

// in[0..7) = planes 0..6, in[7] = sign word.
ZC_HD inline void deltas_from_planes8(uint32_t (&in)[8], int32_t (&d)[32]) {
  magnitude_planes_to_twos<8>(in);
  transpose8x8_quads(in);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
#pragma unroll
    for (int k = 0; k < 4; ++k) d[j + 8 * k] = int32_t(in[j] << (24 - 8 * k)) >> 24;   // sign-extend byte k
  }
}

// in[0..15) = planes 0..14, in[15] = sign word.
ZC_HD inline void deltas_from_planes16(uint32_t (&in)[16], int32_t (&d)[32]) {
  magnitude_planes_to_twos<16>(in);
  transpose16x16_pairs(in);
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    d[j] = int32_t(in[j] << 16) >> 16;
    d[j + 16] = int32_t(in[j]) >> 16;
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

// In-lane conversion between 32 sign-magnitude values and their bit-plane words
// (Section 3.3: sign bits and the fixed-length "bit-shifting" encoding).
//
// One lane owns one block.  Value j is pre-rotated left by j, so that bit p of value j sits
// at position (p + j) mod 32.  Plane p then needs exactly one AND-OR per value with a
// one-bit mask, and one final rotate: plane_p = rotr( OR_j (c_j & bit((p + j) mod 32)), p ).
// The sign is carried as bit 31 of the sign-magnitude word, i.e. as "plane 31".
// All loops are fully unrolled so every array stays in registers.
#pragma once

#include "zc_common.h"

namespace zc {

__device__ inline u32 rotl32(u32 v, int s) { return __builtin_rotateleft32(v, u32(s)); }
__device__ inline u32 rotr32(u32 v, int s) { return __builtin_rotateright32(v, u32(s)); }

// c[j] = rotl(sign-magnitude of value j, j).  Returns plane P (P = 31: the sign word).
template <int P>
__device__ inline u32 gather_plane(const u32 (&c)[32]) {
  u32 acc = 0;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const u32 m = 1u << ((P + j) & 31);
    acc = (c[j] & m) | (acc & ~m);          // one bit-field insert per value
  }
  return rotr32(acc, P);
}

// Inverse: scatter plane word W of plane P into the rotated accumulators.
template <int P>
__device__ inline void scatter_plane(u32 (&c)[32], u32 W) {
  u32 r = rotl32(W, P);
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const u32 m = 1u << ((P + j) & 31);
    c[j] = (r & m) | (c[j] & ~m);           // one bit-field insert per value
  }
}

// Stores sign + planes 0..w-1 of one block at dst[0..w] (LDS).  wmax >= w is wave-uniform
// and bounds the unrolled plane loop.
template <int P>
__device__ inline void store_planes_from(const u32 (&c)[32], u32 w, u32 wmax, u32* dst) {
  if constexpr (P < 31) {
    if (u32(P) >= wmax) return;
    u32 word = gather_plane<P>(c);
    if (u32(P) < w) dst[1 + P] = word;
    store_planes_from<P + 1>(c, w, wmax, dst);
  }
}

__device__ inline void store_block_planes(const u32 (&c)[32], u32 w, u32 wmax, u32* dst) {
  if (wmax == 0) return;
  u32 sign = gather_plane<31>(c);
  if (w) dst[0] = sign;
  store_planes_from<0>(c, w, wmax, dst);
}

// Loads sign + planes of one block from src[0..w] (global or LDS) into rotated accumulators.
template <int P, typename Ptr>
__device__ inline void load_planes_from(u32 (&c)[32], u32 w, u32 wmax, Ptr src) {
  if constexpr (P < 31) {
    if (u32(P) >= wmax) return;
    u32 word = u32(P) < w ? src[1 + P] : 0u;
    scatter_plane<P>(c, word);
    load_planes_from<P + 1>(c, w, wmax, src);
  }
}

template <typename Ptr>
__device__ inline void load_block_planes(u32 (&c)[32], u32 w, u32 wmax, Ptr src) {
#pragma unroll
  for (int j = 0; j < 32; ++j) c[j] = 0;
  if (wmax == 0) return;
  u32 sign = w ? src[0] : 0u;
  scatter_plane<31>(c, sign);
  load_planes_from<0>(c, w, wmax, src);
}

}  // namespace zc

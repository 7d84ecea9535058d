// Fused local step of the compressed Allreduce (Section 3.1.2: per round "decompress, reduce,
// recompress"; Sum aggregation of Section 3.2), for k operands at once.
//
// All operands share the quantisation step, and both the Lorenzo delta and the sum are
// linear, so the sum of the operands' deltas is the delta of the summed codes: nothing has to
// be dequantised, and no prefix sum is needed.  More than that, the deltas never have to leave
// their bit-plane form.  One lane owns one block; a plane word holds one bit of each of the
// block's 32 deltas, so a ripple-carry adder written with bitwise operations on plane words
// adds 32 deltas at once: about four operations per plane per operand for the whole block.
// The sum is kept in two's complement planes, converted back to sign + magnitude planes at
// the end, and its highest non-zero plane gives the new code length.  Output placement is
// the same ticketed look-back scan as in compression.
#pragma once

#include "zc_common.h"
#include "zc_scan.h"

namespace zc {

constexpr int kAccPlanes = 39;   // |sum of 64 deltas| < 2^37: 38 magnitude bits + sign

struct ReduceArgs {
  StreamRef in[ZC_MAX_K];
  int k;
  StreamIndex index;
  u8* out;
  u64 out_cap;
  Control* ctl;
  u64* desc;
};

// acc (two's complement, `top` planes valid, `ext` = its sign plane) += operand given as
// sign word s and magnitude planes a[0..31) (zero above the operand's width).
// Planes [0, new_top) are valid afterwards.  top and new_top are wave-uniform.
template <int P>
__device__ inline void ripple_add(u32 (&acc)[kAccPlanes], const u32 (&a)[31], u32 s, u32 carry,
                                  u32 ext, u32 top, u32 new_top, u32& ext_out) {
  if constexpr (P < kAccPlanes) {
    if (u32(P) >= new_top) return;
    const u32 cur = u32(P) < top ? acc[P] : ext;
    u32 x = s;                                  // two's complement of the operand: (mag ^ s) + s
    if constexpr (P < 31) x ^= a[P];
    const u32 t = cur ^ x;
    const u32 sum = t ^ carry;
    const u32 cout = (t & carry) | (~t & cur);  // majority(cur, x, carry)
    acc[P] = sum;
    ext_out = sum;
    ripple_add<P + 1>(acc, a, s, cout, ext, top, new_top, ext_out);
  }
}

template <int P, typename Ptr>
__device__ inline void load_operand_planes(u32 (&a)[31], u32 w, u32 wmax, Ptr src) {
  if constexpr (P < 31) {
    if (u32(P) >= wmax) return;
    a[P] = u32(P) < w ? src[1 + P] : 0u;
    load_operand_planes<P + 1>(a, w, wmax, src);
  }
}

// Two's complement planes -> magnitude planes; returns the code length.
template <int P>
__device__ inline void magnitude_planes(u32 (&acc)[kAccPlanes], u32 s, u32 carry, u32 top, u32& width) {
  if constexpr (P < kAccPlanes) {
    if (u32(P) >= top) return;
    const u32 t = acc[P] ^ s;
    const u32 m = t ^ carry;
    acc[P] = m;
    if (m) width = P + 1;
    magnitude_planes<P + 1>(acc, s, t & carry, top, width);
  }
}

template <int P>
__device__ inline void store_sum_planes(const u32 (&acc)[kAccPlanes], u32 w, u32 wmax, u32* dst) {
  if constexpr (P < 31) {
    if (u32(P) >= wmax) return;
    if (u32(P) < w) dst[1 + P] = acc[P];
    store_sum_planes<P + 1>(acc, w, wmax, dst);
  }
}

// Exact range check of one block's summed codes, for lanes whose cheap bound did not settle
// it: rebuild every delta from the magnitude planes and walk the Lorenzo chain in 64 bits.
__device__ inline bool block_out_of_range(const u32 (&mag)[kAccPlanes], u32 sign, i64 outlier) {
  i64 q = outlier;
  bool bad = q > kMaxCode || q < -kMaxCode;
  for (int j = 1; j < 32; ++j) {
    i64 m = 0;
#pragma unroll
    for (int p = 0; p < kAccPlanes; ++p) m |= i64((mag[p] >> j) & 1u) << p;
    q += ((sign >> j) & 1u) ? -m : m;
    bad |= q > kMaxCode || q < -kMaxCode;
  }
  return bad;
}

__global__ __launch_bounds__(kTileThreads) void reduce_kernel(ReduceArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWaveLds];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  if (validation_failed(a.ctl)) return;
  const ParsedHeader h = parse_header(a.in[0]);
  if (!h.ok) return;
  const u64 tend = tables_end(h.nb);
  const u32 ntiles = u32(num_tiles(h.nb));

  // The first workgroup writes the header fields and the table padding.
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    u64 nsum = 0;
    for (int s = 0; s < a.k; ++s) nsum += parse_header(a.in[s]).nsum;
    if (nsum > 0xffffffffull) atomicOr(&a.ctl->status, status_bit(ZC_ERR_RANGE));
    if (a.out_cap >= tend) {
      u32* hw = reinterpret_cast<u32*>(a.out);
      hw[0] = kMagic;
      hw[1] = 1u | (5u << 16) | (6u << 24);
      hw[2] = u32(h.n);
      hw[3] = u32(h.n >> 32);
      hw[4] = h.eb_bits;
      hw[5] = u32(nsum);
      if (ntiles == 0) {
        hw[6] = u32(tend);
        hw[7] = u32(tend >> 32);
      }
      for (u64 i = h.nb; i < pad16(h.nb); ++i) a.out[kHeaderBytes + i] = 0;
      u8* ot = a.out + kHeaderBytes + pad16(h.nb);
      for (u64 i = 4 * h.nb; i < pad16(4 * h.nb); ++i) ot[i] = 0;
    } else {
      atomicOr(&a.ctl->status, status_bit(ZC_ERR_CAPACITY));
    }
    if (ntiles == 0) a.ctl->result = tend;
  }
  if (ntiles == 0) return;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  if (threadIdx.x == 0) sh_tile = take_tile(a.ctl, ntiles, xcc_id());
  __syncthreads();
  const u32 tile = uniform(sh_tile);
  if (tile == kNoTile) return;

  u32* wl = lds + wave * kWaveLds;
  const u64 seg = u64(tile) * kTileWaves + u64(wave);
  const bool seg_live = seg < num_segments(h.nb);
  const u64 b = seg * kWaveBlocks + u64(lane);
  const bool active = b < h.nb;

  // ---- add the k operands' blocks in plane form ----
  u32 acc[kAccPlanes];
#pragma unroll
  for (int p = 0; p < kAccPlanes; ++p) acc[p] = 0;
  u32 ext = 0, top = 0;
  u64 bound = 0;          // wave-uniform bound on |sum of deltas| so far
  i64 outlier = 0;
  for (int s = 0; s < a.k; ++s) {
    const u8* base = a.in[s].base;
    const u64 total_s = reinterpret_cast<const u64*>(base)[3];
    const u64 pw = (total_s - tend) / 4;
    u32 w = active ? u32(base[kHeaderBytes + b]) : 0u;
    const u32 words = psize_words(w);
    const u32 incl = wave_inclusive_sum(words);
    u64 off = 0;
    if (seg_live) off = segment_offset(a.index, s, seg) + (incl - words);
    if (off + words > pw) w = 0;                  // cannot happen on a validated stream
    const u32 wmax = wave_max_u32(w);
    if (active) outlier += i64(reinterpret_cast<const i32*>(base + kHeaderBytes + pad16(h.nb))[b]);
    if (wmax == 0) continue;
    const u32* src = reinterpret_cast<const u32*>(base + tend) + off;
    u32 pl[31];
#pragma unroll
    for (int p = 0; p < 31; ++p) pl[p] = 0;
    const u32 sgn = w ? src[0] : 0u;
    load_operand_planes<0>(pl, w, wmax, src);
    bound += (u64(1) << wmax) - 1;
    u32 new_top = 64u - u32(__builtin_clzll(bound)) + 1u;
    if (new_top > u32(kAccPlanes)) new_top = kAccPlanes;
    u32 ext_out = ext;
    ripple_add<0>(acc, pl, sgn, sgn, ext, top, new_top, ext_out);
    ext = ext_out;
    top = new_top;
  }

  // ---- back to sign + magnitude planes; new code length ----
  u32 w = 0;
  magnitude_planes<0>(acc, ext, ext, top, w);
  if (!active) w = 0;
  u32 err = 0;
  if (active) {
    const i64 ao = outlier < 0 ? -outlier : outlier;
    const i64 reach = ao + 31 * ((i64(1) << w) - 1);
    if (reach > kMaxCode || w > 31) {
      if (w > 31 || block_out_of_range(acc, ext, outlier)) {
        err |= status_bit(ZC_ERR_RANGE);
        w = 0;
      }
    }
  }
  const u32 words = psize_words(w);

  // ---- place, publish, pack, look back, copy out (as in compression) ----
  const u32 incl = wave_inclusive_sum(words);
  const u32 wave_total = lane_value(incl, 63);
  const u32 off_in_wave = incl - words;
  const u32 wmax = wave_max_u32(w);
  if (lane == 0) sh_wave_total[wave] = wave_total;
  if (active && a.out_cap >= tend) {
    a.out[kHeaderBytes + b] = u8(w);
    reinterpret_cast<i32*>(a.out + kHeaderBytes + pad16(h.nb))[b] = i32(outlier);
  }
  __syncthreads();
  u32 wave_off = 0, tile_total = 0;
#pragma unroll
  for (int i = 0; i < kTileWaves; ++i) {
    u32 t = sh_wave_total[i];
    if (i < wave) wave_off += t;
    tile_total += t;
  }
  if (threadIdx.x == 0) desc_store(a.desc + desc_slot(tile), (tile == 0 ? kDescPrefix : kDescAggregate) | u64(tile_total));

  if (w) wl[off_in_wave] = ext;
  store_sum_planes<0>(acc, w, wmax, wl + off_in_wave);

  if (wave == 0) {
    const u64 base = tile ? lookback_exclusive(a.desc, tile, &a.ctl->status) : 0;
    if (lane == 0) {
      if (tile) desc_store(a.desc + desc_slot(tile), kDescPrefix | (base + tile_total));
      sh_base = base;
    }
  }
  if (err) atomicOr(&a.ctl->status, err);
  __syncthreads();

  const u64 base = sh_base;
  const u64 cap_words = a.out_cap > tend ? (a.out_cap - tend) / 4 : 0;
  u32* payload = reinterpret_cast<u32*>(a.out + tend);
  const u64 dst0 = base + wave_off;
  for (u32 i = u32(lane); i < wave_total; i += 64) {
    if (dst0 + i < cap_words) payload[dst0 + i] = wl[i];
  }
  if (tile == ntiles - 1 && threadIdx.x == 0) {
    const u64 total = tend + 4 * (base + tile_total);
    a.ctl->result = total;
    if (total > a.out_cap) atomicOr(&a.ctl->status, status_bit(ZC_ERR_CAPACITY));
    if (a.out_cap >= kHeaderBytes) reinterpret_cast<u64*>(a.out)[3] = total;
  }
}

}  // namespace zc

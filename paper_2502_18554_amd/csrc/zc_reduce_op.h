// k-way Max and Min of compressed operands (the other aggregation functions of Section 3.2, in
// the k-operand form of the local step of Section 3.1.2).  All operands share the quantisation
// step and the quantiser is monotone, so the largest code is the code of the largest value:
// the result is exact on the grid, one error bound away from the true extreme whatever k is.
// Unlike the Sum of zc_reduce.h an extreme is not linear in the deltas: every operand's block
// is decoded to its 32 codes (payload through LDS, bit-matrix transpose, walk along the Lorenzo
// chain), the running extreme is kept per value in registers, and the result is encoded like a
// compressed block (new deltas, width, planes, look-back placement).
//
// reduce_op_kernel serves operands without blocks wider than 15 bits; the deltas of an extreme
// are bounded by the largest delta among the operands at the same place, so its output has
// none either.  reduce_op_wide_kernel takes any widths with per-lane loads; both are launched
// and each returns at once when the operands are not its.
#pragma once

#include "zc_bitmatrix.h"
#include "zc_common.h"
#include "zc_decompress.h"
#include "zc_place.h"
#include "zc_reduce.h"
#include "zc_scan.h"

namespace zc {

template <int OP>
__device__ inline i32 extreme(i32 a, i32 b) {
  return OP == ZC_OP_MAX ? max(a, b) : min(a, b);
}

// The extremes of a block (q[j], one lane per block) -> its place in the output stream.
// WIDE: blocks wider than 15 bits may come out (only if some operand had one).
template <bool IX, bool WIDE>
__device__ inline void place_codes(const ReduceArgs& a, const ReduceCall& c, i32 (&q)[32], bool active, u32 b, u32 tile,
                                   u32 ntiles, u32* wl, u32* sh_wave_total, u64* sh_base, int wave, int lane, u32 err) {
  const ParsedHeader& h = c.h;
  const u64 tend = tables_end(h.nb, IX);
  // range of the codes (operands of a valid stream are inside it, so is their extreme)
  i32 hi = q[0], lo = q[0];
#pragma unroll
  for (int j = 1; j < 32; ++j) {
    hi = max(hi, q[j]);
    lo = min(lo, q[j]);
  }
  const bool out_of_range = active && (i64(hi) > kMaxCode || i64(lo) < -kMaxCode);
  if (out_of_range) err |= status_bit(ZC_ERR_RANGE);
  const i32 outlier = q[0];
  // codes -> Lorenzo deltas, in place, last first
  i32 top = 0, bottom = 0;
#pragma unroll
  for (int j = 31; j >= 1; --j) {
    q[j] = i32(u32(q[j]) - u32(q[j - 1]));
    top = max(top, q[j]);
    bottom = min(bottom, q[j]);
  }
  q[0] = 0;
  const u32 any = max(u32(top), u32(-bottom));
  Placement pl;
  pl.w = (active && any && !out_of_range) ? 32u - u32(__builtin_clz(any)) : 0u;
  if (!WIDE && __any(pl.w > 15)) {          // cannot happen: |delta of an extreme| <= the operands' largest |delta|
    err |= status_bit(ZC_ERR_HIP);
    pl.w = 0;
  }
  pl.wmax = wave_max_u32(pl.w);
  const u32 words = psize_words(pl.w);
  const u32 incl = wave_inclusive_sum(words);
  pl.wave_total = lane_value(incl, 63);
  pl.half0_total = lane_value(incl, 31);
  pl.off_in_wave = incl - words;
  if (lane == 0) sh_wave_total[wave] = pl.wave_total | (IX && pl.wmax > 15 ? kWaveWideMark : 0u);
  lds_barrier();
  sum_wave_totals(sh_wave_total, wave, IX, pl);
  const PayloadSink sink{a.out, a.out_cap, h.nb, a.ctl, a.desc, IX, a.coherent != 0, 0u, c.tag};
  if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total, pl.tile_wide);
  if (err) raise_status(a.ctl, c.tag, err);
  const bool narrow = !WIDE || pl.wmax <= 15;
  const TileBase tb = resolve_tile_base(sink, pl, tile, sh_base, wave, lane, [&] {
    if (!narrow) return;
    u32 pw[16];
    planes_from_deltas16(q, pw);
    stage_wave_words<16>([&](auto i) {
      constexpr int I = decltype(i)::value;          // 0: sign, 1 + p: plane p
      if constexpr (I == 0) return pw[15];
      else return pw[I - 1];
    }, pl, wl);
  });
  if (lane == 0) write_index_entry(sink, tile * kTileWaves + u32(wave), tb.words + pl.wave_off);
  if (narrow) {
    copy_staged_wave<16>(sink, pl, tb.words, wl, lane);
  } else {
    u32 plo[16], phi[16];
    planes_from_deltas32(q, plo, phi);
    copy_wave_out<32>(sink, [&](auto i) {
      constexpr int I = decltype(i)::value;
      if constexpr (I == 0) return phi[15];
      else if constexpr (I <= 16) return plo[I - 1];
      else return phi[I - 17];
    }, pl, tb.words, wl, lane);
  }
  if (active && a.out_cap >= tend) {     // (at the very end: see place_sum_staged)
    __builtin_nontemporal_store(u8(pl.w), a.out + widths_begin(h.nb, IX) + b);
    __builtin_nontemporal_store(outlier, reinterpret_cast<i32*>(a.out + outliers_begin(h.nb, IX)) + b);
  }
  finish_stream(sink, pl, tile, ntiles, tb);
}

template <bool IX, int OP>
__global__ __launch_bounds__(kTileThreads, 3) void reduce_op_kernel(ReduceArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWholeStage];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  ReduceCall c;
  bool wide = false;
  OperandMeta meta{};
  u32 tile = 0, ntiles = 0;
  if (!open_reduce<IX>(a, false, true, c, wide, meta, false, tile, ntiles, &sh_tile)) return;
  const ParsedHeader& h = c.h;
  const int wave = wave_id();
  const int lane = lane_id();
  const u64 tend = tables_end(h.nb, IX);
  u32* const wl = lds + wave * kWholeStage;
  const u32 seg = tile * kTileWaves + u32(wave);
  const bool seg_live = seg < num_segments(h.nb);
  const u32 b = seg * kWaveBlocks + u32(lane);
  const bool active = b < h.nb;
  u32 err = 0;
  if (IX && seg_live && !index_ends_consistent(a.in, a.k, h, seg)) err |= status_bit(ZC_ERR_FORMAT);

  // operand s + 1 is on its way while operand s is decoded (as in reduce_narrow_tile)
  meta = load_operand_meta(a, 0, h, seg, b, active, seg_live, IX);
  OperandPlace next = place_operand(meta, h, IX, err);
  if (a.k > 1) meta = load_operand_meta(a, 1, h, seg, b, active, seg_live, IX);
  OperandStage stage = load_operand_payload(reinterpret_cast<const u32*>(a.in[0].base + tend), next, lane);
  i32 outlier_next = load_operand_outlier(a, 0, h, b, active, IX);

  i32 acc[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) acc[j] = OP == ZC_OP_MAX ? i32(0x80000000u) : i32(0x7fffffff);
  for (int s = 0; s < a.k; ++s) {
    const OperandPlace cur = next;
    stage_to_lds(stage, cur, reinterpret_cast<const u32*>(a.in[s].base + tend), wl, lane);
    wave_lds_sync();
    u32 code = u32(outlier_next);
    if (s + 1 < a.k) {
      next = place_operand(meta, h, IX, err);
      if (s + 2 < a.k) meta = load_operand_meta(a, s + 2, h, seg, b, active, seg_live, IX);
      stage = load_operand_payload(reinterpret_cast<const u32*>(a.in[s + 1].base + tend), next, lane);
      outlier_next = load_operand_outlier(a, s + 1, h, b, active, IX);
    }
    // the lane's sign and plane words out of the staged payload, then deltas by the bit-matrix transposes
    // (all reads at once and without conditions, what is not the block's own is dropped: see pick_block_words)
    u32 lo[16];
    {
      const u32* mine = wl + (cur.w ? cur.pick : 0u);
      u32 t[16];
#pragma unroll
      for (int p = 0; p < 16; ++p) t[p] = mine[p];
      const u32 keep = cur.w ? (1u << cur.w) - 1u : 0u;      // bit p: the block has plane p
      lo[15] = cur.w ? t[0] : 0u;
#pragma unroll
      for (int p = 0; p < 15; ++p) lo[p] = t[1 + p] & u32(__builtin_amdgcn_sbfe(i32(keep), u32(p), 1u));
    }
    wave_lds_sync();
    if (cur.wcap == 0) {                       // nothing but constant blocks: every code is the block's first
#pragma unroll
      for (int j = 0; j < 32; ++j) acc[j] = extreme<OP>(acc[j], i32(code));
    } else if (cur.wcap <= 4) {                // every block of the wave at most 4 bits wide: byte fields
      u32 r[8];
#pragma unroll
      for (int p = 0; p < 7; ++p) r[p] = lo[p];
      r[7] = lo[15];
      magnitude_planes_to_twos<8>(r);
      transpose8x8_quads(r);
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        code += u32(__builtin_amdgcn_sbfe(i32(r[j & 7]), u32(8 * (j >> 3)), 8u));
        acc[j] = extreme<OP>(acc[j], i32(code));
      }
    } else {
      magnitude_planes_to_twos<16>(lo);
      transpose16x16_pairs(lo);
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        code += u32(__builtin_amdgcn_sbfe(i32(lo[j & 15]), u32(16 * (j >> 4)), 16u));
        acc[j] = extreme<OP>(acc[j], i32(code));
      }
    }
  }
  place_codes<IX, false>(a, c, acc, active, b, tile, ntiles, wl, sh_wave_total, &sh_base, wave, lane, err);
}

template <bool IX, int OP>
__global__ __launch_bounds__(kTileThreads) void reduce_op_wide_kernel(ReduceArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWholeStage];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  ReduceCall c;
  bool wide = false;
  OperandMeta meta{};
  u32 tile = 0, ntiles = 0;
  if (!open_reduce<IX>(a, true, true, c, wide, meta, false, tile, ntiles, &sh_tile)) return;
  const ParsedHeader& h = c.h;
  const int wave = wave_id();
  const int lane = lane_id();
  const u64 tend = tables_end(h.nb, IX);
  u32* const wl = lds + wave * kWholeStage;
  const u32 seg = tile * kTileWaves + u32(wave);
  const bool seg_live = seg < num_segments(h.nb);
  const u32 b = seg * kWaveBlocks + u32(lane);
  const bool active = b < h.nb;
  u32 err = 0;
  if (IX && seg_live && !index_ends_consistent(a.in, a.k, h, seg)) err |= status_bit(ZC_ERR_FORMAT);

  i32 acc[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) acc[j] = OP == ZC_OP_MAX ? i32(0x80000000u) : i32(0x7fffffff);
#pragma nounroll
  for (int s = 0; s < a.k; ++s) {
    const u8* base = a.in[s].base;
    const u64 total_s = reinterpret_cast<const u64*>(base)[3];
    const u64 pw64 = total_s >= tend ? (total_s - tend) / 4 : 0;
    const u32 pw = pw64 > 0xffffffffull ? 0xffffffffu : u32(pw64);
    u32 w = active ? u32(*at_bytes(base, u32(widths_begin(h.nb, IX)) + b)) : 0u;
    const bool bad_w = w > 31;                    // plain streams: cannot happen on a validated stream
    if (bad_w) w = 0;
    const u32 words = psize_words(w);
    const u32 incl = wave_inclusive_sum(words);
    u32 seg_off = 0;
    bool fits = seg_live;
    if (IX) {
      const u32* index = reinterpret_cast<const u32*>(base + kHeaderBytes);
      const u32 seg_end = seg_live ? index[seg + 1] : 0u;
      seg_off = seg_live ? index[seg] : 0u;
      const bool narrow_promised = (reinterpret_cast<const u32*>(base)[1] & 1u) == 0;
      if (seg_end - seg_off != lane_value(incl, 63) || __any(bad_w) || (narrow_promised && __any(w > 15))) {
        err |= status_bit(ZC_ERR_FORMAT);
        fits = false;
      }
    } else if (seg_live) {
      const u64 so = segment_offset(a.index, s, seg);
      fits = so <= pw;
      seg_off = u32(so);
    }
    if (!fits || seg_off > pw || lane_value(incl, 63) > pw - seg_off) w = 0;
    u32 code = active ? u32(*reinterpret_cast<const i32*>(at_bytes(base, u32(outliers_begin(h.nb, IX)) + 4u * b))) : 0u;
    u32 lo[16], hi[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) lo[p] = hi[p] = 0;
    if (w) {
      const u32* mine = reinterpret_cast<const u32*>(base + tend) + seg_off + (incl - words);
      hi[15] = mine[0];
#pragma unroll
      for (int p = 0; p < 16; ++p)
        if (u32(p) < w) lo[p] = mine[1 + p];
#pragma unroll
      for (int p = 0; p < 15; ++p)
        if (u32(16 + p) < w) hi[p] = mine[17 + p];
    }
    i32 d[32];
    deltas_from_planes32(lo, hi, d);
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      code += u32(d[j]);
      acc[j] = extreme<OP>(acc[j], i32(code));
    }
  }
  place_codes<IX, true>(a, c, acc, active, b, tile, ntiles, wl, sh_wave_total, &sh_base, wave, lane, err);
}

}  // namespace zc

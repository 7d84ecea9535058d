// One round of the ring reduce-scatter in a single kernel (Section 3.1.2: per round the
// received compressed chunk is decompressed, reduced with the local chunk and compressed again;
// Section 3.2: the Sum chain adds one bounded error per round).
//
// The local chunk is uncompressed binary32, so unlike the k-way reduce of zc_reduce.h this
// step has to leave the integer domain: decode the received codes, dequantise, add the local
// values in binary32, quantise the sums on the stream's own grid, and encode again.  It is
// the decompression kernel's front half (stream index -> payload through LDS -> deltas) and
// the compression kernel's back half (deltas -> width -> planes -> look-back placement) around
// one addition, with nothing written to memory in between: 4 bytes per value of local input
// plus the two streams, instead of the 12 more that separate decompress, add and compress
// calls would move.  The other aggregation functions of Section 3.2 (Max, Min) take the
// same round with a comparison in place of the addition (combine<OP>).
//
// Geometry: tiles of 256 blocks, one wave per 64 blocks, one lane per block.  The local
// values arrive as coalesced 16-byte loads (lane = 4 consecutive values), asked for before
// anything else, and are transposed through the wave's LDS area (64 rows of one block) so
// that a lane finds its block's 32 values in its own row.
#pragma once

#include "zc_bitmatrix.h"
#include "zc_common.h"
#include "zc_compress.h"
#include "zc_decompress.h"
#include "zc_place.h"
#include "zc_scan.h"

namespace zc {

struct StepArgs {
  StreamRef in;
  const float* local;
  u64 n_local;
  StreamIndex index;
  u8* out;
  u64 out_cap;
  Control* ctl;
  u64* desc;
  u32 ticketed;      // tiles handed out by tickets instead of by workgroup id
  u64 nonce;         // drawn by the host per call, goes into the call's tag (see launch_tag)
};

constexpr int kStepStage = kWaveBlocks * kStageRow;     // 64 rows of 36 words = 9 KiB per wave
static_assert(kStepStage >= kWaveStage, "the payload staging of the decoder must fit too");

// Header fields and table padding of the output stream; one thread.
__device__ inline void write_step_header(const StepArgs& a, const ParsedHeader& h, u64 tag, u32 ntiles, bool ix) {
  const u64 tend = tables_end(h.nb, ix);
  const u64 nsum = u64(h.nsum) + 1;
  if (nsum > 0xffffffffull) raise_status(a.ctl, tag, status_bit(ZC_ERR_RANGE));
  if (a.out_cap >= tend) write_stream_header(a.out, h.n, h.nb, h.eb_bits, u32(nsum), ix, ntiles == 0);
  else raise_status(a.ctl, tag, status_bit(ZC_ERR_CAPACITY));
  if (ntiles == 0) a.ctl->result = tend;
}

// OP: what a round does with a decoded value a and the local value b (the aggregation functions
// of Section 3.2): their binary32 sum, or the larger or the smaller of the two.  A NaN or an
// infinity in the local buffer is an error whatever a comparison would make of it, so it is passed on.
template <int OP>
__device__ inline float combine(float a, float b) {
  if constexpr (OP == ZC_OP_SUM) {
    return a + b;
  } else {
    const float m = OP == ZC_OP_MAX ? (a > b ? a : b) : (a < b ? a : b);
    return (__float_as_uint(b) & 0x7fffffffu) >= 0x7f800000u ? b : m;
  }
}

template <bool IX, int OP>
__global__ __launch_bounds__(kTileThreads, 4) void step_kernel(StepArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kStepStage];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  const int lane = lane_id();
  const int wave = wave_id();
  u32* const wl = lds + wave * kStepStage;

  // Everything that can be asked for before the header is known goes out at once.  A workgroup
  // that takes the tile of its own number also asks for its local values, its segment's
  // position and its width bytes (fenced in by sizes the host passed).
  const bool early = !a.ticketed;
  const u32 zero = opaque_zero();
  uint4 gate_raw = make_uint4(0, 0, 0, 0);
  if (!IX) gate_raw = load_gate(a.ctl, zero);
  const HeaderWords hw = load_header_words(a.in.base, zero);
  float4 x[8];
  SegmentOffsetParts seg_parts{0, 0, 0};
  u32 w = 0, seg_end = 0;
  if (early) {
    const u32 seg = blockIdx.x * kTileWaves + u32(wave);
    const u32 b = seg * kWaveBlocks + u32(lane);
    const u64 v0 = u64(seg) * kWaveBlocks * kBlockValues;
    const bool whole = v0 + u64(kWaveBlocks) * kBlockValues <= a.n_local;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u64 idx = v0 + u64(256 * i + 4 * lane);
      if (whole) {
        x[i] = load_once(reinterpret_cast<const float4*>(a.local + idx));
      } else {
        x[i].x = idx + 0 < a.n_local ? a.local[idx + 0] : 0.0f;
        x[i].y = idx + 1 < a.n_local ? a.local[idx + 1] : 0.0f;
        x[i].z = idx + 2 < a.n_local ? a.local[idx + 2] : 0.0f;
        x[i].w = idx + 3 < a.n_local ? a.local[idx + 3] : 0.0f;
      }
    }
    if (IX) {                 // the width bytes sit behind the index, whose size follows from n (= n_local, or the call fails)
      if (u64(kHeaderBytes) + 4 * u64(seg) + 8 <= a.in.bytes) {
        seg_parts = load_segment_offset(a.index, 0, seg, zero, a.in.base);
        seg_end = load_segment_end(a.in.base, seg, zero);
      }
      const u64 w_at = widths_begin(num_blocks(a.n_local), true) + b;
      if (w_at < a.in.bytes) w = u32(*at_bytes(a.in.base, u32(w_at)));
    } else {
      if (seg < 4 * a.index.tiles_cap) seg_parts = load_segment_offset(a.index, 0, seg, zero);
      if (u64(kHeaderBytes) + b < a.in.bytes) w = u32(*at_bytes(a.in.base, kHeaderBytes + b));
    }
  }

  // Plain streams: validated and indexed by the kernels of zc_scan.h, whose verdict and tag are in
  // the control block.  Indexed streams: judged here, by every workgroup alike.
  const ParsedHeader h = parse_header(hw, a.in.bytes, IX);
  const u64 ltag = launch_tag(a.nonce, a.ctl);
  u64 tag;
  if (IX) {
    tag = call_tag(a.ctl, ltag, false);
    if (!h.ok) {
      if (blockIdx.x == 0 && threadIdx.x == 0) {
        a.ctl->result = 0;
        raise_status(a.ctl, tag, status_bit(ZC_ERR_FORMAT));
      }
      return;
    }
  } else {
    const Gate gate = parse_gate(gate_raw);
    tag = gate.tag;
    if (gate_failed(gate) || !h.ok) return;
  }
  if (a.n_local != h.n) {
    if (blockIdx.x == 0 && threadIdx.x == 0) raise_status(a.ctl, tag, status_bit(ZC_ERR_MISMATCH));
    return;
  }
  const u64 tend = tables_end(h.nb, IX);
  const u32 ntiles = u32(num_tiles(h.nb));
  if (blockIdx.x == 0 && threadIdx.x == 0) write_step_header(a, h, tag, ntiles, IX);
  if (ntiles == 0) {                         // a stream without blocks: its one index entry must say so
    if (IX && blockIdx.x == 0 && wave == 0 && !index_ends_consistent(&a.in, 1, h, 0) && lane == 0)
      raise_status(a.ctl, tag, status_bit(ZC_ERR_FORMAT));
    return;
  }

  u32 tile = blockIdx.x;                     // tiles in the order in which workgroups start
  if (a.ticketed) {                          // ... or handed out by tickets, see take_tile
    if (threadIdx.x == 0) sh_tile = take_tile(a.ctl, ltag, ntiles, xcc_id());
    __syncthreads();
    tile = uniform(sh_tile);
  }
  if (tile >= ntiles) return;

  const u32 seg = tile * kTileWaves + u32(wave);
  const bool seg_live = seg < num_segments(h.nb);
  const u32 b = seg * kWaveBlocks + u32(lane);
  const bool active = b < h.nb;
  const u64 v0 = u64(seg) * kWaveBlocks * kBlockValues;
  if (!early) {
    const bool whole = v0 + u64(kWaveBlocks) * kBlockValues <= h.n;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u64 idx = v0 + u64(256 * i + 4 * lane);
      if (whole) {
        x[i] = load_once(reinterpret_cast<const float4*>(a.local + idx));
      } else {
        x[i].x = idx + 0 < h.n ? a.local[idx + 0] : 0.0f;
        x[i].y = idx + 1 < h.n ? a.local[idx + 1] : 0.0f;
        x[i].z = idx + 2 < h.n ? a.local[idx + 2] : 0.0f;
        x[i].w = idx + 3 < h.n ? a.local[idx + 3] : 0.0f;
      }
    }
    if (IX) {
      if (seg_live) {
        seg_parts = load_segment_offset(a.index, 0, seg, 0, a.in.base);
        seg_end = load_segment_end(a.in.base, seg);
      }
    } else {
      if (seg_live) seg_parts = load_segment_offset(a.index, 0, seg);
      w = active ? u32(*at_bytes(a.in.base, kHeaderBytes + b)) : 0u;
    }
  }
  if (IX && !early && active) w = u32(*at_bytes(a.in.base, u32(widths_begin(h.nb, true)) + b));
  if (!active) w = 0;
  if (!seg_live) {
    seg_parts = SegmentOffsetParts{0, 0, 0};
    seg_end = 0;
  }
  u32 cur = active ? u32(reinterpret_cast<const i32*>(a.in.base + outliers_begin(h.nb, IX))[b]) : 0u;

  // ---- the received block's sign and plane words; then the local values, one block per row
  //      of the same LDS area; then the received block's deltas ----
  u32 lo[16], hi[16];
  u32 err = 0;
  const u64 seg_off = IX ? u64(uniform(seg_parts.seg)) : segment_offset(seg_parts);
  const u32 wmax_in = wave_block_words(reinterpret_cast<const u32*>(a.in.base + tend), (h.total - tend) / 4, w, seg_off,
                                       wl, lane, lo, hi, IX, uniform(seg_end) - u32(seg_off), h.wide, err);
  if (IX && seg_live && !index_ends_ok(h, seg, u32(seg_off), uniform(seg_end))) err |= status_bit(ZC_ERR_FORMAT);
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<float4*>(wl + (8 * i + (lane >> 3)) * kStageRow + 4 * (lane & 7)) = x[i];
  wave_lds_sync();
  i32 d[32];
  deltas_from_block_words(wmax_in, lo, hi, d);

  // ---- codes in, sums, codes out, new deltas (in place) ----
  CompressArgs qa;               // the quantiser's constants, from the stream's own bound
  const float eb = __uint_as_float(h.eb_bits);
  qa.step = double(eb) * 63.0 / 32.0;
  qa.inv = 1.0 / qa.step;
  qa.eb = double(eb);
  qa.screen = eb * 131072.0f;
  const u64 cnt64 = active ? h.n - u64(b) * kBlockValues : 0;      // values of this block that exist
  const u32 cnt = cnt64 < 32 ? u32(cnt64) : 32u;
  // first the sums (in place of the deltas) and their largest magnitude: a NaN or an infinity
  // has the largest bit pattern of all, so one unsigned maximum screens the whole block
  u32 amax = 0;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const float4 l4 = *reinterpret_cast<const float4*>(wl + lane * kStageRow + 4 * t);
    const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = 4 * t + u;
      cur += u32(d[j]);
      const float y = combine<OP>(float(__dmul_rn(double(i32(cur)), qa.step)), lv[u]);
      amax = max(amax, __float_as_uint(y) & 0x7fffffffu);
      d[j] = i32(__float_as_uint(y));
    }
  }
  // (values past the end of the last block are sums of a repeated code and zero: harmless here)
  const bool checked = __any(active && needs_checks(__uint_as_float(amax), qa));
  const bool ragged = __any(active && cnt < 32);      // only the wave that holds the stream's last block
  i32 outlier = 0, prev = 0, top = 0, bottom = 0;
  if (__builtin_expect(!checked && !ragged, 1)) {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const i32 q = quantize_fast(__uint_as_float(u32(d[j])), qa);
      if (j == 0) outlier = q;
      const i32 nd = j ? q - prev : 0;
      top = max(top, nd);
      bottom = min(bottom, nd);
      d[j] = nd;
      prev = q;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      i32 q = prev;                                   // the last block repeats its last code
      if (u32(j) < cnt) q = quantize_value(__uint_as_float(u32(d[j])), qa, err);
      if (j == 0) outlier = q;
      const i32 nd = j ? q - prev : 0;
      top = max(top, nd);
      bottom = min(bottom, nd);
      d[j] = nd;
      prev = q;
    }
  }
  wave_lds_sync();

  // ---- width, tables, placement ----
  const u32 any = max(u32(top), u32(-bottom));
  Placement pl;
  pl.w = (active && any) ? 32u - u32(__builtin_clz(any)) : 0u;
  pl.wmax = wave_max_u32(pl.w);
  if (active && a.out_cap >= tend) {
    a.out[widths_begin(h.nb, IX) + b] = u8(pl.w);
    reinterpret_cast<i32*>(a.out + outliers_begin(h.nb, IX))[b] = outlier;
  }
  const u32 words = psize_words(pl.w);
  const u32 incl = wave_inclusive_sum(words);
  pl.wave_total = lane_value(incl, 63);
  pl.half0_total = lane_value(incl, 31);
  pl.off_in_wave = incl - words;
  if (lane == 0) sh_wave_total[wave] = pl.wave_total | (IX && pl.wmax > 15 ? kWaveWideMark : 0u);
  lds_barrier();                // the wave totals; the stores above stay in flight
  sum_wave_totals(sh_wave_total, wave, IX, pl);
  const PayloadSink sink{a.out, a.out_cap, h.nb, a.ctl, a.desc, IX, 0u, tag};
  if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total, pl.tile_wide);
  if (err) raise_status(a.ctl, tag, err);
  const TileBase tb = resolve_tile_base(sink, pl, tile, &sh_base, wave, lane);
  const u64 base = tb.words;
  if (lane == 0) write_index_entry(sink, seg, base + pl.wave_off);

  // ---- deltas -> sign + plane words, out through LDS ----
  if (pl.wmax <= 15) {           // per wave: each wave copies its own words
    u32 pw[16];
    planes_from_deltas16(d, pw);
    copy_wave_out<16>(sink, [&](auto i) {
      constexpr int I = decltype(i)::value;          // 0: sign, 1 + p: plane p
      if constexpr (I == 0) return pw[15];
      else return pw[I - 1];
    }, pl, base, wl, lane);
  } else {
    u32 lo[16], hi[16];
    planes_from_deltas32(d, lo, hi);
    copy_wave_out<32>(sink, [&](auto i) {
      constexpr int I = decltype(i)::value;
      if constexpr (I == 0) return hi[15];
      else if constexpr (I <= 16) return lo[I - 1];
      else return hi[I - 17];
    }, pl, base, wl, lane);
  }
  finish_stream(sink, pl, tile, ntiles, tb);
}

}  // namespace zc

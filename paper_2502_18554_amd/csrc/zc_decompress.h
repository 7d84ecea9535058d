// fZ-light decompression kernel: the inverse of the stages of Section 3.3.
//
// Same geometry as compression: a tile is 256 blocks, one lane owns one block, and there is no
// dependency between workgroups: a wave's payload offset comes from the stream index
// (computed by zc_scan.h for a plain stream, carried by an indexed one), and a scan of the
// block sizes places each lane inside the wave.  The wave's
// payload is contiguous, so it is copied into LDS with coalesced loads (each byte leaves the
// L2 once) and every lane then picks its sign and plane words there.  A bit-matrix transpose
// turns them back into deltas; the Lorenzo chain from the block's outlier and the
// dequantisation follow in registers; the floats go back through LDS, in two halves of 32
// blocks, so that they leave as 16-byte coalesced stores.
#pragma once

#include "zc_bitmatrix.h"
#include "zc_common.h"
#include "zc_scan.h"

namespace zc {

struct DecompressArgs {
  StreamRef in;
  float* out;
  u64 out_cap_elems;
  StreamIndex index;
  Control* ctl;
  u64 first_value;   // decompress_range_kernel only: the part [first_value, first_value + count) of the
  u64 count;         // stream, first_value a multiple of the values of a segment
  u64 nonce;         // drawn by the host per call, goes into the call's tag (see launch_tag)
};

// The sign and plane words of the lane's block (width w, 0 for a block that does not exist) out
// of a stream's payload.  seg_off = payload word offset of the wave's segment.  The wave's
// payload goes through its LDS staging area `wl` (kWaveStage words); a wave with a block wider
// than 15 bits fetches per lane instead.  Returns the widest block of the wave.  Widths up to
// 15: lo[0..15) = planes 0..14, lo[15] = sign word.  Wider: lo[0..16) = planes 0..15,
// hi[0..15) = planes 16..30, hi[15] = sign word.  `wl` is free again on return.
// Indexed stream (ix): seg_words = the segment's size by the stream's own index.  The staged
// copy is asked for on that figure, before the widths are looked at, so it travels together
// with the loads of the tables; a segment whose widths add up to another figure, a width above
// 31, or one above 15 in a stream that promised none (!may_be_wide) make the stream malformed
// (`err`), and nothing of the segment's payload is used.
constexpr int kWaveStageLoads = 4;
struct WaveStage {
  uint4 v[kWaveStageLoads];
};

// The copy starts at the 16-byte boundary at or below the segment (the payload area itself is
// 16-byte aligned) and keeps that misalignment in LDS, so it moves 16 bytes per lane and
// instruction, all loads in flight together.  span = words to bring in, <= 1027.
// Four loads cover 1024 words; only whole 16-byte pieces are asked for here: the up to three
// words beyond (a wave whose 64 blocks are all 15 bits wide, off the 16-byte grid) and the
// last words of a stream that do not fill a piece are fetched by store_wave_stage.  The loads
// are written without any branch: a lane with nothing to fetch reads the 16 bytes at `safe`
// (the stream's header) instead.  (With a branch around a load and a zero on its other side,
// or with the stream's last words fetched into single components of the same registers, the
// compiler copied a component after every 16-byte load and waited for the load to do so: the
// loads went out one round trip after the other.)
__device__ inline WaveStage load_wave_stage(const u32* payload, u64 payload_words, u64 src0, u32 span, int lane,
                                            const uint4* safe) {
  WaveStage st;
#pragma unroll
  for (int i = 0; i < kWaveStageLoads; ++i) {
    const u32 idx = 4u * u32(lane) + 256u * u32(i);
    const bool piece = idx < span && src0 + idx + 4 <= payload_words;
    st.v[i] = *(piece ? reinterpret_cast<const uint4*>(payload + src0 + idx) : safe);
  }
  return st;
}

__device__ inline void store_wave_stage(const WaveStage& st, const u32* payload, u64 payload_words, u64 src0, u32 span,
                                        u32* wl, int lane) {
#pragma unroll
  for (int i = 0; i < kWaveStageLoads; ++i) {
    const u32 idx = 4u * u32(lane) + 256u * u32(i);
    if (idx < span) *reinterpret_cast<uint4*>(wl + idx) = st.v[i];
  }
  const u32 staged = span < 256u * kWaveStageLoads ? span : 256u * kWaveStageLoads;
  if (src0 + ((u64(staged) + 3) & ~u64(3)) > payload_words) {    // uniform: the wave that holds the end of the stream
#pragma unroll
    for (int i = 0; i < kWaveStageLoads; ++i) {
      const u32 idx = 4u * u32(lane) + 256u * u32(i);
      if (idx < span && src0 + idx + 4 > payload_words) {
        for (u32 j = 0; j < 3; ++j)
          if (src0 + idx + j < payload_words) wl[idx + j] = payload[src0 + idx + j];
      }
    }
  }
  if (span > 256u * kWaveStageLoads) {                           // uniform, and rare: words 1024 .. 1026
    const u32 idx = 256u * kWaveStageLoads + u32(lane);
    if (idx < span && src0 + idx < payload_words) wl[idx] = payload[src0 + idx];
  }
}

// What a wave knows about its segment's payload once the widths are scanned.
struct WavePayload {
  u32 w;            // this lane's block width (0 if the block must be skipped)
  u32 off_in_wave;  // payload word offset of this lane's block inside the segment
  u32 wmax;         // the widest block of the wave (uniform)
  bool inside;      // the segment lies inside the payload and agrees with the index (uniform)
};

// First half of wave_block_words: scan of the widths, the checks, and the staged copy of the
// segment's payload into `wl` when no block is wider than 15 bits.
__device__ inline WavePayload stage_wave_payload(const u32* payload, u64 payload_words, u32 w, u64 seg_off, u32* wl, int lane,
                                                 bool ix, u32 seg_words, bool may_be_wide, u32& err, const uint4* safe) {
  const u32 mis = u32(seg_off) & 3u;
  const u64 src0 = seg_off - mis;                      // in words, multiple of 4
  WaveStage st;
  u32 span = 0;
  if (ix) {
    // at most 64 * 16 words when no block is wider than 15 bits
    if (seg_words <= 64u * 16u && seg_off + seg_words <= payload_words) span = mis + seg_words;
    st = load_wave_stage(payload, payload_words, src0, span, lane, safe);
    store_wave_stage(st, payload, payload_words, src0, span, wl, lane);   // at once: the registers are free for what follows
  }
  bool unfit = false;
  if (ix) {
    unfit = __any(w > (may_be_wide ? 31u : 15u));
    if (unfit) w = 0;
  }
  WavePayload wp;
  const u32 words = psize_words(w);
  const u32 incl = wave_inclusive_sum(words);
  wp.off_in_wave = incl - words;
  const u32 wave_total = lane_value(incl, 63);
  wp.wmax = wave_max_u32(w);
  wp.w = w;
  // a validated stream keeps every segment inside the payload; refuse to read outside anyway
  wp.inside = seg_off + wave_total <= payload_words;
  if (ix && (unfit || wave_total != seg_words)) {
    err |= status_bit(ZC_ERR_FORMAT);
    wp.inside = false;
  }
  if (wp.wmax <= 15 && !ix) {
    span = wp.inside ? mis + wave_total : 0u;
    st = load_wave_stage(payload, payload_words, src0, span, lane, safe);
    store_wave_stage(st, payload, payload_words, src0, span, wl, lane);
  }
  return wp;
}

// Second half, widths up to 15: every lane picks its block's words out of the staged copy.
// lo[0..15) = planes 0..14, lo[15] = sign word.  `wl` is free again on return.
// All sixteen reads are issued at once and without conditions (the words behind a block's own
// belong to the next blocks, or are whatever the staging area held: they are dropped
// afterwards; the area is large enough for 15 words behind any staged word).  A loop that
// stops at the wave's widest block costs far more than the reads it saves: it is compiled as
// a loop, with a wait after every read.
__device__ inline void pick_block_words(const WavePayload& wp, u64 seg_off, const u32* wl, u32 (&lo)[16]) {
  static_assert(kWaveStage >= 1027 + 16, "reads behind the last staged word stay inside the staging area");
  wave_lds_sync();
  const bool have = wp.w && wp.inside;
  const u32* mine = wl + (have ? (u32(seg_off) & 3u) + wp.off_in_wave : 0u);
  u32 t[16];
#pragma unroll
  for (int p = 0; p < 16; ++p) t[p] = mine[p];
  const u32 keep = have ? (1u << wp.w) - 1u : 0u;      // bit p: the block has plane p
  lo[15] = have ? t[0] : 0u;
#pragma unroll
  for (int p = 0; p < 15; ++p) lo[p] = t[1 + p] & u32(__builtin_amdgcn_sbfe(i32(keep), u32(p), 1u));
  wave_lds_sync();
}

__device__ inline u32 wave_block_words(const u32* payload, u64 payload_words, u32 w, u64 seg_off, u32* wl, int lane,
                                       u32 (&lo)[16], u32 (&hi)[16], bool ix, u32 seg_words, bool may_be_wide,
                                       u32& err, const uint4* safe) {
  const WavePayload wp = stage_wave_payload(payload, payload_words, w, seg_off, wl, lane, ix, seg_words, may_be_wide, err, safe);
  if (wp.wmax <= 15) {
    pick_block_words(wp, seg_off, wl, lo);
  } else {
    // a block wider than 15 bits (stream of an input outside the guaranteed domain): each lane
    // fetches its words straight from global memory
#pragma unroll
    for (int p = 0; p < 16; ++p) lo[p] = 0;
#pragma unroll
    for (int p = 0; p < 16; ++p) hi[p] = 0;
    if (wp.w && wp.inside) {
      const u32* mine = payload + seg_off + wp.off_in_wave;
      hi[15] = mine[0];
#pragma unroll
      for (int p = 0; p < 16; ++p)
        if (u32(p) < wp.w) lo[p] = mine[1 + p];
#pragma unroll
      for (int p = 0; p < 15; ++p)
        if (u32(16 + p) < wp.w) hi[p] = mine[17 + p];
    }
  }
  return wp.wmax;
}

// ... and from those words the block's Lorenzo deltas (bit-matrix transposes back).
__device__ inline void deltas_from_block_words(u32 wmax, u32 (&lo)[16], u32 (&hi)[16], i32 (&d)[32]) {
  if (wmax <= 7) {
    u32 r[8];
#pragma unroll
    for (int p = 0; p < 7; ++p) r[p] = lo[p];
    r[7] = lo[15];
    deltas_from_planes8(r, d);
  } else if (wmax <= 15) {
    deltas_from_planes16(lo, d);
  } else {
    deltas_from_planes32(lo, hi, d);
  }
}

// One tile (blockIdx.x) of stream `s` of the index, into `out`.  `many`: one of several streams
// of a call (blockIdx.y); `others_ok`: the headers of the other streams are in order.
// `ix`: the stream is indexed: no kernel has run ahead of this one, the header and the index
// are judged here (see judge_indexed_streams, index_ends_ok), and the call's tag is this
// launch's; its width bytes sit behind the index, whose size only the header tells, so they
// are asked for together with the outlier and the payload.  A plain stream has been validated
// and indexed by the kernels of zc_scan.h, whose verdict and tag are in the control block.
// `average`: the values are divided by the stream's nsum (the Average aggregation of Section
// 3.2 on a stream of sums): x' = float((double(q) * s) * r), r = 1.0 / nsum.
// first_value, count: only the values [first_value, first_value + count) of the stream, cut off
// at its end, are produced, into out_values[0 ...] (a chunk handled on its own, Section 3.5.2);
// first_value is a multiple of the 2048 values of a segment.  The whole stream: 0 and ~0.
__device__ inline void decompress_tile(const StreamRef& in, float* out_values, u64 out_cap_elems, const StreamIndex& index,
                                       int s, Control* ctl, u64 nonce, bool many, bool others_ok, u64 sum_n, u32* lds,
                                       bool ix, bool average = false, u64 first_value = 0, u64 count = ~u64(0)) {
  const DecompressArgs a{in, out_values, out_cap_elems, index, ctl, first_value, count, nonce};

  // Everything that can be asked for before the header is known goes out at once: the control
  // block, the header, the segment's position and the width bytes.  The loads are fenced in
  // by sizes the host passed; what the header then rules out is dropped.
  const int lane = lane_id();
  const int wave = wave_id();
  const u32 seg = u32(first_value / (kWaveBlocks * kBlockValues)) + blockIdx.x * kTileWaves + u32(wave);   // < 2^22: the host launches at most 2^20 tiles
  const u32 wblock0 = seg * kWaveBlocks;
  const u32 b = wblock0 + u32(lane);                   // a stream has at most 2^26 blocks
  const u32 zero = opaque_zero();
  const bool first_group = blockIdx.x == 0 && blockIdx.y == 0;
  uint4 gate_raw = make_uint4(0, 0, 0, 0);
  if (!ix) gate_raw = load_gate(a.ctl, zero);
  const HeaderWords hw = load_header_words(a.in.base, zero);
  SegmentOffsetParts seg_parts{0, 0, 0};
  u32 seg_end = 0, w = 0;
  if (ix) {
    if (u64(kHeaderBytes) + 4 * u64(seg) + 8 <= a.in.bytes) {
      seg_parts = load_segment_offset(a.index, s, seg, zero, a.in.base);
      seg_end = load_segment_end(a.in.base, seg, zero);
    }
  } else {
    if (seg < 4 * a.index.tiles_cap) seg_parts = load_segment_offset(a.index, s, seg, zero);
    if (u64(kHeaderBytes) + b < a.in.bytes) w = u32(*at_bytes(a.in.base, kHeaderBytes + b));
  }

  const ParsedHeader h = parse_header(hw, a.in.bytes, ix);
  u64 tag;
  if (ix) {
    tag = call_tag(a.ctl, launch_tag(a.nonce, a.ctl), false);
    if (!h.ok || !others_ok) {
      if (first_group && threadIdx.x == 0) {
        a.ctl->result = 0;
        raise_status(a.ctl, tag, status_bit(ZC_ERR_FORMAT));
      }
      return;
    }
    // a stream without blocks: nobody looks at its index, which is one closing entry of 0
    if (h.nb == 0 && blockIdx.x == 0 && threadIdx.x == 0 &&
        (h.total != tables_end(0, true) || *reinterpret_cast<const u32*>(a.in.base + kHeaderBytes) != 0))
      raise_status(a.ctl, tag, status_bit(ZC_ERR_FORMAT));
  } else {
    const Gate gate = parse_gate(gate_raw);
    tag = gate.tag;
    if (gate_failed(gate) || !h.ok) return;
  }
  if (first_value > h.n) {                            // the part lies beyond the stream
    if (blockIdx.x == 0 && threadIdx.x == 0) raise_status(a.ctl, tag, status_bit(ZC_ERR_ARG));
    return;
  }
  const u64 end_value = count < h.n - first_value ? first_value + count : h.n;     // one past the last value wanted
  const u64 wanted = end_value - first_value;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (!many) a.ctl->result = wanted;
    else if (ix) { if (blockIdx.y == 0) a.ctl->result = sum_n; }
    else atomicAdd(reinterpret_cast<unsigned long long*>(&a.ctl->result), static_cast<unsigned long long>(wanted));
  }
  if (wanted > a.out_cap_elems) {
    if (blockIdx.x == 0 && threadIdx.x == 0) raise_status(a.ctl, tag, status_bit(ZC_ERR_CAPACITY));
    return;
  }
  if (!ix && u64(seg) >= 4 * a.index.tiles_cap) return;

  u32* const wl = lds + wave * kWaveStage;
  if (seg >= num_segments(h.nb) || u64(seg) * kWaveBlocks * kBlockValues >= end_value) return;   // no barrier below: waves are independent
  const bool active = b < h.nb;
  if (ix && active) w = u32(*at_bytes(a.in.base, u32(widths_begin(h.nb, true)) + b));
  if (!active) w = 0;

  const i32* outliers = reinterpret_cast<const i32*>(a.in.base + outliers_begin(h.nb, ix));
  const u32* payload = reinterpret_cast<const u32*>(a.in.base + tables_end(h.nb, ix));
  const u64 payload_words = (h.total - tables_end(h.nb, ix)) / 4;

  u32 cur = active ? u32(outliers[b]) : 0u;
  const u64 seg_off = ix ? u64(uniform(seg_parts.seg)) : segment_offset(seg_parts);
  i32 d[32];
  {
    u32 lo[16], hi[16];
    u32 err = 0;
    const u32 wmax = wave_block_words(payload, payload_words, w, seg_off, wl, lane, lo, hi, ix,
                                      uniform(seg_end) - u32(seg_off), h.wide, err, reinterpret_cast<const uint4*>(a.in.base));
    if (ix && !index_ends_ok(h, seg, u32(seg_off), uniform(seg_end))) err |= status_bit(ZC_ERR_FORMAT);
    if (err && lane == 0) raise_status(a.ctl, tag, err);
    deltas_from_block_words(wmax, lo, hi, d);
  }

  // ---- Lorenzo chain from the outlier, dequantise ----
  const double step = double(__uint_as_float(h.eb_bits)) * 63.0 / 32.0;
  const double r = average ? __ddiv_rn(1.0, double(h.nsum)) : 1.0;
  float x[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    cur += u32(d[j]);
    const double v = __dmul_rn(double(i32(cur)), step);
    x[j] = float(average ? __dmul_rn(v, r) : v);
  }

  // ---- transpose through LDS (two halves of 32 blocks), 16-byte coalesced stores ----
  const u64 v0 = u64(wblock0) * kBlockValues;
  const bool full = v0 + u64(kWaveBlocks) * kBlockValues <= end_value;
  float* const out = a.out - first_value;           // indexed by the value's number in the stream
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    if ((lane >> 5) == hh) {
#pragma unroll
      for (int t = 0; t < 8; ++t)
        *reinterpret_cast<float4*>(wl + (lane & 31) * kStageRow + 4 * t) =
            make_float4(x[4 * t], x[4 * t + 1], x[4 * t + 2], x[4 * t + 3]);
    }
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u64 idx = v0 + u64(1024 * hh + 256 * i + 4 * lane);
      const float4 v = *reinterpret_cast<const float4*>(wl + (8 * i + (lane >> 3)) * kStageRow + 4 * (lane & 7));
      if (full) {
        store_once(reinterpret_cast<float4*>(out + idx), v);
      } else {
        if (idx + 0 < end_value) out[idx + 0] = v.x;
        if (idx + 1 < end_value) out[idx + 1] = v.y;
        if (idx + 2 < end_value) out[idx + 2] = v.z;
        if (idx + 3 < end_value) out[idx + 3] = v.w;
      }
    }
    wave_lds_sync();
  }
}

template <bool IX, bool AVERAGE>
__global__ __launch_bounds__(kTileThreads, 5) void decompress_kernel(DecompressArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWaveStage];
  decompress_tile(a.in, a.out, a.out_cap_elems, a.index, 0, a.ctl, a.nonce, false, true, 0, lds, IX, AVERAGE);
}

// A part of a stream (see decompress_tile).
template <bool IX>
__global__ __launch_bounds__(kTileThreads, 5) void decompress_range_kernel(DecompressArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWaveStage];
  decompress_tile(a.in, a.out, a.out_cap_elems, a.index, 0, a.ctl, a.nonce, false, true, 0, lds, IX, false, a.first_value,
                  a.count);
}

// k streams in one launch (the tail of the compressed Allgather, Section 3.5.1: every rank
// decompresses all the chunks it has received): blockIdx.y = stream, blockIdx.x = tile.
struct DecompressManyArgs {
  StreamRef in[ZC_MAX_K];
  float* out[ZC_MAX_K];
  u64 out_cap_elems[ZC_MAX_K];
  int k;
  StreamIndex index;
  Control* ctl;
  u64 nonce;
};

template <bool IX>
__global__ __launch_bounds__(kTileThreads, 5) void decompress_many_kernel(DecompressManyArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWaveStage];
  const int s = blockIdx.y;
  bool all_ok = true;
  u64 sum_n = 0;
  if (IX) {                      // any malformed header stops the whole call
    const StreamsVerdict v = judge_indexed_streams(a.in, a.k, false);
    all_ok = v.err == 0;
    sum_n = v.sum_n;
  }
  decompress_tile(a.in[s], a.out[s], a.out_cap_elems[s], a.index, s, a.ctl, a.nonce, true, all_ok, sum_n, lds, IX);
}

}  // namespace zc

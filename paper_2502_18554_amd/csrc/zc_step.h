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
// Geometry: tiles of 256 blocks, one wave per 64 blocks.  A wave takes one of two paths.
// The common one (one lane per block) serves waves whose received and produced blocks are at
// most 15 bits wide, whose blocks are complete and whose sums lie inside the screened domain
// of the quantiser: the received deltas stay packed as the bit-matrix transpose leaves them
// (two 16-bit or four 8-bit fields per word), a single walk along the Lorenzo chain takes each
// delta out of its field, forms the sum and the new code, and packs the new delta at once, so
// that a block never occupies more than 16 + 16 registers; the local values arrive as coalesced
// 16-byte loads, asked for before anything else, and pass through the wave's LDS area in two
// halves (values 0..15 and 16..31 of every block) so that a lane finds its block's values in its
// own row.  Whatever that path cannot take (a block wider than 15 bits on either side, the
// ragged end of the buffer, a sum outside the screened domain, which is also where NaN and
// infinity end up) is found out before anything is written and sends the whole wave through
// the other path: 32 lanes per block, two blocks per step, the defining arithmetic with all
// its checks, first to learn the new widths, and again, once the tile's place in the output
// is known, to emit the plane words as ballots.  It is slow, rare, and needs next to no
// registers, so it does not limit how many waves fit a SIMD.
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
  u32 coherent;      // the look-back reads the tile's own chain with device-coherent loads too
  u64 nonce;         // drawn by the host per call, goes into the call's tag (see launch_tag)
  // A round done in parts (zc_reduce_step_part): this launch takes the tiles [first_tile, end_tile)
  // of the output, end_tile = 0 meaning all of them; a later part (adopt) belongs to the call whose
  // tag the first part left in the control block.
  u32 first_tile, end_tile, adopt;
};

// LDS of one wave: 64 rows (blocks) of 16 local values + 4 words of padding (an odd number of
// 16-byte units per row keeps the 128-bit row reads of neighbouring lanes on distinct banks).
// The received payload (at most 1027 words) and the produced one (at most 64 x 16 words) pass
// through the same area.
constexpr int kStepRow = 20;
constexpr int kStepStage = kWaveBlocks * kStepRow;     // 1280 words = 5 KiB per wave
static_assert(kStepStage >= 1027 + 16 && kStepStage >= 64 * 16, "payload staging, and the reads behind its last word, must fit the wave's area");

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

// ---------------------------------------------------------------------------------------
// The common path: one lane per block.
// ---------------------------------------------------------------------------------------

// What the walk along a block's Lorenzo chain carries from value to value.
struct ChainState {
  u32 cur;          // the received code of the value before
  i32 prev;         // the new code of the value before
  i32 top, bottom;  // largest and smallest new delta so far (d0 = 0 is one of them)
  u32 upos, uneg;   // largest bit pattern of a sum as a signed and as an unsigned number: the
                    // largest positive and the largest negative magnitude, NaN and infinity on top
  i32 outlier;      // the new code of value 0
};

// Bytes 1 and 2 of a plane word change places: bits 8..15 (values 8..15) and 16..23 (values
// 16..23).  On plane words swapped like this the 16 x 16 transposes pair value j with value
// j + 8 instead of j + 16: word j & 7 holds values j and j + 8 of the block's first half, word
// 8 + (j & 7) those of its second half, so the walk below is done with eight words when it has
// done half the block, and has filled eight words of new deltas.
__device__ inline u32 swap_middle_bytes(u32 v) { return __builtin_amdgcn_perm(v, v, 0x03010200u); }

// Values 16 HALF .. 16 HALF + 15 of the lane's block.  BITS: width of the fields the received
// deltas are packed in (16: word (j & 7) + 8 HALF holds values j and j + 8, see above; 8: word
// j & 7 holds values j, j + 8, j + 16, j + 24).  `row`: the lane's 16 local values of this half.
// The new deltas go into nf as 16-bit fields paired the same way.
template <int OP, int BITS, int HALF, int NF>
__device__ inline void walk_half(const u32 (&fields)[NF], const u32* row, const CompressArgs& qa, ChainState& cs, u32 (&nf)[16]) {
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const float4 l4 = *reinterpret_cast<const float4*>(row + 4 * t);
    const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
    i32 nd[4];
    u32 yb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = 16 * HALF + 4 * t + u;
      const u32 f = BITS == 16 ? fields[(j & 7) + 8 * HALF] : fields[j & 7];
      const int at = BITS == 16 ? 16 * ((j >> 3) & 1) : 8 * (j >> 3);
      cs.cur += u32(__builtin_amdgcn_sbfe(i32(f), u32(at), u32(BITS)));
      const float y = combine<OP>(float(__dmul_rn(double(i32(cs.cur)), qa.step)), lv[u]);
      yb[u] = __float_as_uint(y);
      const i32 q = quantize_fast(y, qa);
      if (j == 0) cs.outlier = q;
      nd[u] = j ? q - cs.prev : 0;
      cs.prev = q;
      if (((j >> 3) & 1) == 0) nf[(j & 7) + 8 * HALF] = u32(nd[u]);
      else nf[(j & 7) + 8 * HALF] = pack16(nf[(j & 7) + 8 * HALF], u32(nd[u]));
    }
    cs.top = max(cs.top, max(max(nd[0], nd[1]), max(nd[2], nd[3])));
    cs.bottom = min(cs.bottom, min(min(nd[0], nd[1]), min(nd[2], nd[3])));
    cs.upos = u32(max(i32(cs.upos), max(max(i32(yb[0]), i32(yb[1])), max(i32(yb[2]), i32(yb[3])))));
    cs.uneg = max(cs.uneg, max(max(yb[0], yb[1]), max(yb[2], yb[3])));
  }
}

// Local values 16..31 of every block into the wave's rows, once values 0..15 have been used (see
// step_kernel: `later` holds them spread over all lanes).
__device__ inline void stage_second_half(u32* wl, int lane, bool first_kind, const float4 (&later)[4]) {
  wave_lds_sync();
  // first kind: loads 4..7 of the partner (same rows, the partner's columns); second kind: its own loads 0..3
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<float4*>(wl + (8 * (first_kind ? 4 + i : i) + (lane >> 3)) * kStepRow + 4 * (lane & 3)) = later[i];
  wave_lds_sync();
}

// ---------------------------------------------------------------------------------------
// The other path: 32 lanes per block.
// ---------------------------------------------------------------------------------------

// Inclusive sum (modulo 2^32) over the 32 lanes of each half of the wave.
__device__ inline u32 half_inclusive_sum(u32 v) {
  v += dpp_row_shr_or_zero<1>(v);
  v += dpp_row_shr_or_zero<2>(v);
  v += dpp_row_shr_or_zero<4>(v);
  v += dpp_row_shr_or_zero<8>(v);
  const u32 t0 = lane_value(v, 15), t2 = lane_value(v, 47);
  const int row = lane_id() >> 4;
  return v + (row == 1 ? t0 : row == 3 ? t2 : 0u);
}

// Maximum over the 32 lanes of each half of the wave, in every lane of the half.
__device__ inline u32 half_max(u32 v) {
  u32 o;
  o = dpp_mov<kDppQuadSwap1>(v); v = o > v ? o : v;
  o = dpp_mov<kDppQuadSwap2>(v); v = o > v ? o : v;
  o = dpp_mov<kDppRowHalfMirror>(v); v = o > v ? o : v;
  o = dpp_mov<kDppRowMirror>(v); v = o > v ? o : v;
  const u32 a = lane_value(v, 0), b = lane_value(v, 16), c = lane_value(v, 32), d = lane_value(v, 48);
  return lane_id() < 32 ? (a > b ? a : b) : (c > d ? c : d);
}

// The value of `v` in lane `src` (any lane, chosen per lane).
__device__ inline u32 from_lane(u32 v, u32 src) { return u32(__builtin_amdgcn_ds_bpermute(int((src & 63u) << 2), int(v))); }

// What the other path needs to know about the received segment, one lane per block.
struct SlowInput {
  const u32* payload;   // the received stream's payload
  u32 w;                // width of the lane's block (0: no payload to read)
  u32 off;              // payload word offset of the lane's block
  u32 outlier;          // its first code
};

// One pass over the wave's 64 blocks, two per step.  EMIT false: computes the new width and
// first code of every block (returned one lane per block) and raises the errors of the
// quantiser.  EMIT true: computes the same values again and stores the sign and plane words
// of every block at its place: w_out, off_out (one lane per block) = its new width and its
// word offset inside the wave's payload, which starts at payload word `dst_wave`.
template <int OP, bool EMIT>
__device__ inline void step_wave_slow(const StepArgs& a, const ParsedHeader& h, const CompressArgs& qa, u32 seg,
                                      const SlowInput& in, u32& w_out, i32& outlier_out, u32 off_out, u64 dst_wave,
                                      u64 cap_words, u32* payload_out, u32& err) {
  const int lane = lane_id();
  const u32 half = u32(lane) >> 5, j = u32(lane) & 31u;
  u32 w_res = 0;
  i32 outlier_res = 0;
#pragma nounroll
  for (u32 bp = 0; bp < 32; ++bp) {
    const u32 blk_a = 2 * bp, blk_b = 2 * bp + 1;
    // ---- the received deltas of the two blocks, one per lane ----
    const u32 wa = lane_value(in.w, int(blk_a)), wb = lane_value(in.w, int(blk_b));
    const u32 w_mine = half ? wb : wa;
    const u32 off_mine = half ? lane_value(in.off, int(blk_b)) : lane_value(in.off, int(blk_a));
    const u32 outl = half ? lane_value(in.outlier, int(blk_b)) : lane_value(in.outlier, int(blk_a));
    const u32 w_top = wa > wb ? wa : wb;
    u32 mag = 0, neg = 0;
    if (w_mine) neg = (in.payload[off_mine] >> j) & 1u;
#pragma nounroll
    for (u32 p = 0; p < w_top; ++p)
      if (p < w_mine) mag |= ((in.payload[off_mine + 1 + p] >> j) & 1u) << p;
    const u32 d = neg ? 0u - mag : mag;
    const u32 code = outl + half_inclusive_sum(d);
    // ---- the sum and its code ----
    const u64 b = u64(seg) * kWaveBlocks + (half ? blk_b : blk_a);
    const u64 left = b < h.nb ? h.n - b * kBlockValues : 0;
    const u32 cnt = left < 32 ? u32(left) : 32u;        // values of this block that exist
    const float local = j < cnt ? a.local[b * kBlockValues + j] : 0.0f;
    const float y = combine<OP>(float(__dmul_rn(double(i32(code)), qa.step)), local);
    u32 ignored = 0;
    i32 q = 0;
    if (j < cnt) q = quantize_value(y, qa, EMIT ? ignored : err);
    const i32 last = i32(from_lane(u32(q), 32u * half + (cnt ? cnt - 1u : 0u)));
    if (j >= cnt) q = cnt ? last : 0;                   // the last block repeats its last code
    const i32 before = i32(from_lane(u32(q), u32(lane) + 63u));                 // lane - 1 (lane 0 gets lane 63: unused)
    const i32 nd = j ? q - before : 0;
    const u32 nmag = u32(nd < 0 ? -nd : nd);
    if (!EMIT) {
      const u32 m = half_max(nmag);
      const u32 wn = m ? 32u - u32(__builtin_clz(m)) : 0u;
      const u32 wn_a = lane_value(wn, 0), wn_b = lane_value(wn, 32);
      const u32 q0_a = lane_value(u32(q), 0), q0_b = lane_value(u32(q), 32);
      if (u32(lane) == blk_a) { w_res = wn_a; outlier_res = i32(q0_a); }
      if (u32(lane) == blk_b) { w_res = wn_b; outlier_res = i32(q0_b); }
    } else {
      const u32 wo_a = lane_value(w_out, int(blk_a)), wo_b = lane_value(w_out, int(blk_b));
      const u32 wo_mine = half ? wo_b : wo_a;
      const u64 dst = dst_wave + (half ? lane_value(off_out, int(blk_b)) : lane_value(off_out, int(blk_a)));
      const u64 sign = __ballot(nd < 0);
      if (j == 0 && wo_mine && dst < cap_words) payload_out[dst] = half ? u32(sign >> 32) : u32(sign);
      const u32 wo_top = wo_a > wo_b ? wo_a : wo_b;
#pragma nounroll
      for (u32 p = 0; p < wo_top; ++p) {
        const u64 plane = __ballot(((nmag >> p) & 1u) != 0);
        if (j == 0 && p < wo_mine && dst + 1 + p < cap_words) payload_out[dst + 1 + p] = half ? u32(plane >> 32) : u32(plane);
      }
    }
  }
  if (!EMIT) {
    w_out = w_res;
    outlier_out = outlier_res;
  }
}

// TICKETS: tiles are handed out by tickets (take_tile) instead of by workgroup id.  A template parameter,
// not an argument: a workgroup that knows its tile from its id asks for everything at once, and the waits
// for those loads can only be counted exactly when no other path joins them.
template <bool IX, int OP, bool TICKETS>
__global__ __launch_bounds__(kTileThreads, 5) void step_kernel(StepArgs a) {
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
  constexpr bool early = !TICKETS;
  const u32 zero = opaque_zero();
  // (with tickets the ticket is asked for first of all: its round trip runs beside the header's)
  u64 asked = 0;
  if (TICKETS && threadIdx.x == 0) asked = ask_ticket(ticket_counter(a.ctl, ticket_shard()));
  uint4 gate_raw = make_uint4(0, 0, 0, 0);
  if (!IX) gate_raw = load_gate(a.ctl, zero);
  const HeaderWords hw = load_header_words(a.in.base, zero);
  float4 x[8];
  SegmentOffsetParts seg_parts{0, 0, 0};
  u32 w = 0, seg_end = 0;
  if (early) {
    const u32 seg = (a.first_tile + blockIdx.x) * kTileWaves + u32(wave);
    const u32 b = seg * kWaveBlocks + u32(lane);
    const u64 v0 = u64(seg) * kWaveBlocks * kBlockValues;
    const bool whole = v0 + u64(kWaveBlocks) * kBlockValues <= a.n_local;
    // The segment's position and the width bytes first: loads return in the order in which they were asked
    // for, and the payload can be asked for as soon as these are there, while the local values still arrive.
    // None of these loads sits behind a branch (what must not be read is replaced by the stream's first
    // bytes and dropped afterwards): where paths with different numbers of loads under way meet, the
    // compiler has to wait for all of them at the first use of any.
    if (IX) {                 // the width bytes sit behind the index, whose size follows from n (= n_local, or the call fails)
      const bool have = u64(kHeaderBytes) + 4 * u64(seg) + 8 <= a.in.bytes;
      const u32 at = have ? kHeaderBytes + 4u * seg : 0u;
      const u32 e0 = *reinterpret_cast<const u32*>(at_bytes(a.in.base, at + zero));
      const u32 e1 = *reinterpret_cast<const u32*>(at_bytes(a.in.base, at + 4u + zero));
      const u64 w_at = widths_begin(num_blocks(a.n_local), true) + b;
      const u32 wb = u32(*at_bytes(a.in.base, w_at < a.in.bytes ? u32(w_at) : 0u));
      seg_parts.seg = have ? e0 : 0u;
      seg_end = have ? e1 : 0u;
      w = w_at < a.in.bytes ? wb : 0u;
    } else {
      if (seg < 4 * a.index.tiles_cap) seg_parts = load_segment_offset(a.index, 0, seg, zero);
      if (u64(kHeaderBytes) + b < a.in.bytes) w = u32(*at_bytes(a.in.base, kHeaderBytes + b));
    }
    const float4* const nothing = reinterpret_cast<const float4*>(a.in.base);      // (a ragged wave fetches its values later)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u64 idx = v0 + u64(256 * i + 4 * lane);
      x[i] = load_once(whole ? reinterpret_cast<const float4*>(a.local + idx) : nothing);
    }
    // Nothing moves across this line: left to itself the compiler puts the wait for the header in front of
    // the last of these loads, which then goes out a round trip late.
    __builtin_amdgcn_sched_barrier(0);
  }

  // Plain streams: validated and indexed by the kernels of zc_scan.h, whose verdict and tag are in
  // the control block.  Indexed streams: judged here, by every workgroup alike.
  const ParsedHeader h = parse_header(hw, a.in.bytes, IX);
  const u64 ltag = launch_tag(a.nonce, a.ctl);
  u64 tag;
  if (IX) {
    tag = call_tag(a.ctl, ltag, a.adopt != 0);
    if (!h.ok) {
      if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (!a.adopt) a.ctl->result = 0;
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
  if (blockIdx.x == 0 && threadIdx.x == 0 && a.first_tile == 0) write_step_header(a, h, tag, ntiles, IX);
  if (ntiles == 0) {                         // a stream without blocks: its one index entry must say so
    if (IX && blockIdx.x == 0 && wave == 0 && !index_ends_consistent(&a.in, 1, h, 0) && lane == 0)
      raise_status(a.ctl, tag, status_bit(ZC_ERR_FORMAT));
    return;
  }
  const u32 end_tile = a.end_tile && a.end_tile < ntiles ? a.end_tile : ntiles;
  if (a.first_tile >= end_tile) return;

  u32 tile = a.first_tile + blockIdx.x;      // tiles in the order in which workgroups start
  if (TICKETS) {                             // ... or handed out by tickets, see take_tile
    if (threadIdx.x == 0) {
      const u32 t = take_tile(a.ctl, ltag, end_tile - a.first_tile, ticket_shard(), asked);
      sh_tile = t == kNoTile ? kNoTile : a.first_tile + t;
    }
    __syncthreads();
    tile = uniform(sh_tile);
  }
  if (tile >= end_tile) return;

  const u32 seg = tile * kTileWaves + u32(wave);
  const bool seg_live = seg < num_segments(h.nb);
  const u32 b = seg * kWaveBlocks + u32(lane);
  const bool active = b < h.nb;
  const u64 v0 = u64(seg) * kWaveBlocks * kBlockValues;
  const bool whole = v0 + u64(kWaveBlocks) * kBlockValues <= h.n;     // every block of the wave exists, and is complete
  if (!early) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u64 idx = v0 + u64(256 * i + 4 * lane);
      x[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (whole) x[i] = load_once(reinterpret_cast<const float4*>(a.local + idx));
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
  const u32 outlier_in = active ? u32(reinterpret_cast<const i32*>(a.in.base + outliers_begin(h.nb, IX))[b]) : 0u;

  // ---- the received segment: scan of the widths, checks, payload into LDS ----
  const u32* const payload_in = reinterpret_cast<const u32*>(a.in.base + tend);
  u32 err = 0;
  const u64 seg_off = IX ? u64(uniform(seg_parts.seg)) : segment_offset(seg_parts);
  const WavePayload wp = stage_wave_payload(payload_in, (h.total - tend) / 4, w, seg_off, wl, lane, IX,
                                            uniform(seg_end) - u32(seg_off), h.wide, err, reinterpret_cast<const uint4*>(a.in.base));
  if (IX && seg_live && !index_ends_ok(h, seg, u32(seg_off), uniform(seg_end))) err |= status_bit(ZC_ERR_FORMAT);

  CompressArgs qa;               // the quantiser's constants, from the stream's own bound
  const float eb = __uint_as_float(h.eb_bits);
  qa.step = double(eb) * 63.0 / 32.0;
  qa.inv = 1.0 / qa.step;
  qa.eb = double(eb);
  qa.screen = fminf(eb * 131072.0f, 3.4028234663852886e38f);    // kept finite: an infinite sum must fail the screen

  // ---- the common path, if the wave can take it ----
  Placement pl;
  pl.w = 0;
  i32 outlier = 0;
  u32 nf[16];
#pragma unroll
  for (int p = 0; p < 16; ++p) nf[p] = 0;
  bool slow = wp.wmax > 15 || !whole;
  if (!slow) {
    u32 lo[16];
    pick_block_words(wp, seg_off, wl, lo);
    // Local values 0..15 of every block go to LDS first: each 16-byte load holds four values of one
    // block, and the lanes with (lane & 7) < 4 hold those of the first halves.  The other lanes'
    // registers hold the second halves, 8 KiB per wave in all, which wait for the first half of the
    // walk: spread over all 64 lanes (each lane of the first kind takes over loads 4..7 of its
    // partner, four lanes up) they occupy four registers of 16 bytes per lane instead of eight.
    const bool first_kind = (lane & 7) < 4;
    float4 later[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (first_kind) {
        *reinterpret_cast<float4*>(wl + (8 * i + (lane >> 3)) * kStepRow + 4 * (lane & 7)) = x[i];
        *reinterpret_cast<float4*>(wl + (8 * (4 + i) + (lane >> 3)) * kStepRow + 4 * (lane & 7)) = x[4 + i];
      }
      // row_shl:4 hands every lane the value of the lane four up in its row of 16 (all lanes take part:
      // a lane that is switched off cannot be read from)
      const float ux = __uint_as_float(dpp_mov<0x104>(__float_as_uint(x[4 + i].x)));
      const float uy = __uint_as_float(dpp_mov<0x104>(__float_as_uint(x[4 + i].y)));
      const float uz = __uint_as_float(dpp_mov<0x104>(__float_as_uint(x[4 + i].z)));
      const float uw = __uint_as_float(dpp_mov<0x104>(__float_as_uint(x[4 + i].w)));
      later[i].x = first_kind ? ux : x[i].x;
      later[i].y = first_kind ? uy : x[i].y;
      later[i].z = first_kind ? uz : x[i].z;
      later[i].w = first_kind ? uw : x[i].w;
    }
    wave_lds_sync();
    ChainState cs{outlier_in, 0, 0, 0, 0u, 0u, 0};
    const u32* const row = wl + lane * kStepRow;
    if (wp.wmax <= 7) {
      u32 r[8];
#pragma unroll
      for (int p = 0; p < 7; ++p) r[p] = lo[p];
      r[7] = lo[15];
      magnitude_planes_to_twos<8>(r);
      transpose8x8_quads(r);
      walk_half<OP, 8, 0>(r, row, qa, cs, nf);
      stage_second_half(wl, lane, first_kind, later);
      walk_half<OP, 8, 1>(r, row, qa, cs, nf);
    } else {
#pragma unroll
      for (int p = 0; p < 16; ++p) lo[p] = swap_middle_bytes(lo[p]);
      magnitude_planes_to_twos<16>(lo);
      transpose16x16_pairs(lo);
      walk_half<OP, 16, 0>(lo, row, qa, cs, nf);
      stage_second_half(wl, lane, first_kind, later);
      walk_half<OP, 16, 1>(lo, row, qa, cs, nf);
    }
    wave_lds_sync();
    const u32 any = max(u32(cs.top), u32(-cs.bottom));
    pl.w = (active && any) ? 32u - u32(__builtin_clz(any)) : 0u;
    outlier = cs.outlier;
    // the largest magnitude among the sums: a NaN or an infinity has the largest bit pattern of all
    const u32 amax = max(i32(cs.upos) < 0 ? 0u : cs.upos, cs.uneg & 0x7fffffffu);
    slow = __any(active && (needs_checks(__uint_as_float(amax), qa) || pl.w > 15));
  }
  SlowInput si{payload_in, 0u, 0u, outlier_in};
  if (slow) {
    // (the segment is inside the payload, or its blocks count as empty)
    si.w = wp.inside ? wp.w : 0u;
    si.off = u32(seg_off) + wp.off_in_wave;
    step_wave_slow<OP, false>(a, h, qa, seg, si, pl.w, outlier, 0u, 0, 0, nullptr, err);
    if (!active) pl.w = 0;
  }

  // ---- width, tables, placement ----
  pl.wmax = wave_max_u32(pl.w);
  // (width and outlier go to their tables at the very end: a store that is under way is waited for by
  // every poll of the look-back)
  const u32 words = psize_words(pl.w);
  const u32 incl = wave_inclusive_sum(words);
  pl.wave_total = lane_value(incl, 63);
  pl.half0_total = lane_value(incl, 31);
  pl.off_in_wave = incl - words;
  if (lane == 0) sh_wave_total[wave] = pl.wave_total | (IX && pl.wmax > 15 ? kWaveWideMark : 0u);
  lds_barrier();                // the wave totals; the stores above stay in flight
  sum_wave_totals(sh_wave_total, wave, IX, pl);
  const PayloadSink sink{a.out, a.out_cap, h.nb, a.ctl, a.desc, IX, a.coherent != 0, a.end_tile ? end_tile : 0u, tag};
  if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total, pl.tile_wide);
  if (err) raise_status(a.ctl, tag, err);
  // ---- the new deltas as sign + plane words into the staging area, while the look-back is under way ----
  const TileBase tb = resolve_tile_base(sink, pl, tile, &sh_base, wave, lane, [&] {
    if (slow) return;
    u32 pw[16];          // pw[0] = sign, pw[1 + p] = plane p
    if (pl.wmax <= 7) {
      // four 8-bit fields per word: word j = values j, j + 8 (word j of nf), j + 16, j + 24 (word j + 8)
      u32 r[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) r[j] = __builtin_amdgcn_perm(nf[j + 8], nf[j], 0x06040200u);
      transpose8x8_quads(r);
      twos_planes_to_magnitude<8>(r);
      pw[0] = r[7];
#pragma unroll
      for (int p = 0; p < 7; ++p) pw[1 + p] = r[p];
#pragma unroll
      for (int p = 8; p < 16; ++p) pw[p] = 0;
    } else {
      planes16_from_fields(nf);
      pw[0] = swap_middle_bytes(nf[15]);
#pragma unroll
      for (int p = 0; p < 15; ++p) pw[1 + p] = swap_middle_bytes(nf[p]);
    }
    stage_wave_words<16>([&](auto i) { return pw[decltype(i)::value]; }, pl, wl);
  });
  const u64 base = tb.words;
  if (lane == 0) write_index_entry(sink, seg, base + pl.wave_off);

  // ---- out ----
  if (!slow) {
    copy_staged_wave<16>(sink, pl, base, wl, lane);
  } else {
    const u64 cap_words = a.out_cap > tend ? (a.out_cap - tend) / 4 : 0;
    u32 ignored = 0;
    step_wave_slow<OP, true>(a, h, qa, seg, si, pl.w, outlier, pl.off_in_wave, base + pl.wave_off, cap_words,
                             reinterpret_cast<u32*>(a.out + tend), ignored);
  }
  if (active && a.out_cap >= tend) {
    a.out[widths_begin(h.nb, IX) + b] = u8(pl.w);
    reinterpret_cast<i32*>(a.out + outliers_begin(h.nb, IX))[b] = outlier;
  }
  finish_stream(sink, pl, tile, ntiles, tb);
}

}  // namespace zc

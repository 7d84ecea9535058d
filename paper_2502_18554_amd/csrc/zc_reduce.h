// Fused local step of the compressed Allreduce (Section 3.1.2: per round "decompress, reduce,
// recompress"; Sum aggregation of Section 3.2), for k operands at once.
//
// All operands share the quantisation step, and both the Lorenzo delta and the sum are
// linear, so the sum of the operands' deltas is the delta of the summed codes: nothing has to
// be dequantised, and no prefix sum is needed.  More than that, the deltas never have to leave
// their bit-plane form.  One lane owns one block; a plane word holds one bit of each of the
// block's 32 deltas, so a ripple-carry adder written with bitwise operations on plane words
// adds 32 deltas at once: a handful of operations per plane per operand for the whole block.
// The sum is kept in two's complement planes, converted back to sign + magnitude planes at
// the end, and its highest non-zero plane gives the new code length.  Output placement is
// the same ticketed look-back scan as in compression.
//
// Two kernels share this scheme.  reduce_kernel serves streams whose blocks are all at most
// 15 bits wide (every stream of an input inside the guaranteed domain of a sensible bound):
// a wave's payload of one operand is then at most 1024 words, is brought into LDS with
// 16-byte loads, and the loads of the next operand fly while the current one is added; the
// summed planes go to LDS in one pass and leave as coalesced stores.  Operand payloads are
// read, and the output stream is written, with the non-temporal hint (see load_once).
// The other path of the same kernel (reduce_wide_tile) takes any widths with per-lane loads,
// a few planes at a time so that it needs no more registers than the common path.  Whether any
// operand has a wider block is known when a workgroup starts (from the stream index of plain
// streams, from the version words of indexed ones), so the whole call takes one path.
// IX = the streams are indexed (see index_bytes): operands bring the positions of their
// segments along, which every wave checks against the widths it reads, and the output gets
// its own index as it is placed.
#pragma once

#include "zc_common.h"
#include "zc_place.h"
#include "zc_scan.h"

namespace zc {

struct ReduceArgs {
  StreamRef in[ZC_MAX_K];
  int k;
  StreamIndex index;
  u8* out;
  u64 out_cap;
  Control* ctl;
  u64* desc;
  u32 ticketed;      // tiles handed out by tickets instead of by workgroup id
  u32 coherent;      // the look-back reads the tile's own chain with device-coherent loads too
  u64 nonce;         // drawn by the host per call, goes into the call's tag (see launch_tag)
  // A reduce done in parts (zc_reduce_compressed_part): this launch takes the tiles
  // [first_tile, end_tile) of the output, end_tile = 0 meaning all of them; a later part
  // (adopt) belongs to the call whose tag the first part left in the control block.
  u32 first_tile, end_tile, adopt;
  u64 n_part;        // a reduce done in parts: the n the caller laid the parts out for (the streams must have it); else 0
};

// What a workgroup knows about the call once the headers are judged.
struct ReduceCall {
  ParsedHeader h;    // header of operand 0 (all operands have its n and bound)
  u64 tag;           // the call's tag
  u64 ltag;          // this launch's tag (tile tickets)
  u64 nsum;          // sum of the operands' nsum
  u32 part_end;      // a reduce done in parts: one past the last tile of this part; else 0
};

// Header fields and table padding of the output stream; one thread.
__device__ inline void write_reduce_header(const ReduceArgs& a, const ReduceCall& c, u32 ntiles, bool ix) {
  const ParsedHeader& h = c.h;
  const u64 tend = tables_end(h.nb, ix);
  if (c.nsum > 0xffffffffull) raise_status(a.ctl, c.tag, status_bit(ZC_ERR_RANGE));
  if (a.out_cap >= tend) write_stream_header(a.out, h.n, h.nb, h.eb_bits, u32(c.nsum), ix, ntiles == 0);
  else raise_status(a.ctl, c.tag, status_bit(ZC_ERR_CAPACITY));
  if (ntiles == 0) a.ctl->result = tend;
}

// Exact range check of one block's summed codes, for lanes whose cheap bound did not settle
// it: rebuild every delta from the magnitude planes and walk the Lorenzo chain in 64 bits.
template <int NP>
__device__ inline bool block_out_of_range(const u32 (&mag)[NP], u32 sign, i64 outlier) {
  i64 q = outlier;
  bool bad = q > kMaxCode || q < -kMaxCode;
  for (int j = 1; j < 32; ++j) {
    i64 m = 0;
#pragma unroll
    for (int p = 0; p < NP; ++p) m |= i64((mag[p] >> j) & 1u) << p;
    q += ((sign >> j) & 1u) ? -m : m;
    bad |= q > kMaxCode || q < -kMaxCode;
  }
  return bad;
}

// Range screen and placement of a summed block inside its wave and tile, then the shared
// back half.  mag[0..NP) = magnitude planes, sign = sign word, w = highest non-zero plane + 1;
// `word(i)` hands out the sign word (i = 0) and plane i - 1, for at most NW words.
template <int NW, int NP, typename WordFn>
__device__ inline void place_sum(const ReduceArgs& a, const ReduceCall& c, const u32 (&mag)[NP], u32 sign, u32 w,
                                 i64 outlier, bool active, u32 b, u32 tile, u32 ntiles, WordFn word, u32* wl,
                                 u32* sh_wave_total, u64* sh_base, int wave, int lane, bool ix) {
  const ParsedHeader& h = c.h;
  const u64 tend = tables_end(h.nb, ix);
  if (!active) w = 0;
  u32 err = 0;
  if (active) {
    const i64 ao = outlier < 0 ? -outlier : outlier;
    const i64 reach = ao + 31 * ((i64(1) << w) - 1);
    if (reach > kMaxCode || w > 31) {
      if (w > 31 || block_out_of_range(mag, sign, outlier)) {
        err |= status_bit(ZC_ERR_RANGE);
        w = 0;
      }
    }
  }
  Placement pl;
  pl.w = w;
  pl.wmax = wave_max_u32(w);
  const u32 words = psize_words(w);
  const u32 incl = wave_inclusive_sum(words);
  pl.wave_total = lane_value(incl, 63);
  pl.half0_total = lane_value(incl, 31);
  pl.off_in_wave = incl - words;
  if (lane == 0) sh_wave_total[wave] = pl.wave_total | (ix && pl.wmax > 15 ? kWaveWideMark : 0u);
  if (active && a.out_cap >= tend) {
    a.out[widths_begin(h.nb, ix) + b] = u8(w);
    reinterpret_cast<i32*>(a.out + outliers_begin(h.nb, ix))[b] = i32(outlier);
  }
  lds_barrier();                // the wave totals; the stores above stay in flight
  sum_wave_totals(sh_wave_total, wave, ix, pl);
  const PayloadSink sink{a.out, a.out_cap, h.nb, a.ctl, a.desc, ix, a.coherent != 0, c.part_end, c.tag};
  if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total, pl.tile_wide);
  if (err) raise_status(a.ctl, c.tag, err);
  finish_tile<NW>(sink, word, pl, tile, ntiles, wl, sh_base, wave, lane);
}

// The same for a wave whose whole payload fits its staging area (kWholeStage words per wave):
// the plane words go to LDS in one pass before the wait for the tile's base offset, so the
// registers that hold them are free from then on, and the copy-out is a plain LDS-to-memory
// copy of the wave's words.
constexpr int kWholeStage = 64 * 24;

template <int NW, int NP, typename WordFn>
__device__ inline void place_sum_staged(const ReduceArgs& a, const ReduceCall& c, const u32 (&mag)[NP], u32 sign, u32 w,
                                        i64 outlier, bool active, u32 b, u32 tile, u32 ntiles, WordFn word, u32* wl,
                                        u32* sh_wave_total, u64* sh_base, int wave, int lane, bool ix) {
  static_assert(64 * NW <= kWholeStage, "a wave of widest blocks must fit the staging area");
  const ParsedHeader& h = c.h;
  const u64 tend = tables_end(h.nb, ix);
  if (!active) w = 0;
  u32 err = 0;
  if (active) {
    const i64 ao = outlier < 0 ? -outlier : outlier;
    const i64 reach = ao + 31 * ((i64(1) << w) - 1);
    if (reach > kMaxCode || w > 31) {
      if (w > 31 || block_out_of_range(mag, sign, outlier)) {
        err |= status_bit(ZC_ERR_RANGE);
        w = 0;
      }
    }
  }
  Placement pl;
  pl.w = w;
  pl.wmax = wave_max_u32(w);
  const u32 words = psize_words(w);
  const u32 incl = wave_inclusive_sum(words);
  pl.wave_total = lane_value(incl, 63);
  pl.half0_total = lane_value(incl, 31);
  pl.off_in_wave = incl - words;
  if (lane == 0) sh_wave_total[wave] = pl.wave_total | (ix && pl.wmax > 15 ? kWaveWideMark : 0u);
  // (width and outlier go to their tables at the very end: a store that is under way is waited for by
  // every poll of the look-back)
  if (w) {
    wl[pl.off_in_wave] = word(std::integral_constant<int, 0>{});
    [&]<int... P>(std::integer_sequence<int, P...>) {
      ((u32(P) < w ? void(wl[pl.off_in_wave + 1 + P] = word(std::integral_constant<int, 1 + P>{})) : void()), ...);
    }(std::make_integer_sequence<int, NW - 1>{});
  }
  lds_barrier();                // the wave totals (and the words above); the stores stay in flight
  sum_wave_totals(sh_wave_total, wave, ix, pl);
  const PayloadSink sink{a.out, a.out_cap, h.nb, a.ctl, a.desc, ix, a.coherent != 0, c.part_end, c.tag};
  if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total, pl.tile_wide);
  if (err) raise_status(a.ctl, c.tag, err);
  const TileBase tb = resolve_tile_base(sink, pl, tile, sh_base, wave, lane);
  const u64 cap_words = a.out_cap > tend ? (a.out_cap - tend) / 4 : 0;
  const u64 d0 = tb.words + pl.wave_off;
  if (lane == 0) write_index_entry(sink, tile * kTileWaves + u32(wave), d0);
  u32* const dst = reinterpret_cast<u32*>(a.out + tend) + d0;
  const u64 room = cap_words > d0 ? cap_words - d0 : 0;
  const u32 limit = u64(pl.wave_total) < room ? pl.wave_total : u32(room);
  copy_staged_words<NW + 1>(wl, dst, limit, lane);
  wave_lds_sync();
  if (active && a.out_cap >= tend) {
    // (the whole output stream is written with the non-temporal hint, see store_once)
    __builtin_nontemporal_store(u8(w), a.out + widths_begin(h.nb, ix) + b);
    __builtin_nontemporal_store(i32(outlier), reinterpret_cast<i32*>(a.out + outliers_begin(h.nb, ix)) + b);
  }
  finish_stream(sink, pl, tile, ntiles, tb);
}

// ---------------------------------------------------------------------------------------
// Streams without blocks wider than 15 bits.
// ---------------------------------------------------------------------------------------

// The accumulator: 24 two's complement planes hold the sum of up to 64 deltas below 2^16 in
// magnitude.  Planes [0, top) are valid, top a multiple of 4 and wave-uniform; plane top - 1
// is a copy of the sign plane.
constexpr int kSumPlanes = 24;
static_assert(64 * kSumPlanes <= kWholeStage && kWholeStage >= kWaveStage, "staging area of reduce_kernel");
constexpr int kSumChunk = 4;

// What a wave needs to know about one operand's share, loaded two operands ahead: the values
// as they come from memory.  Nothing is computed from them where they are loaded, so that
// no load has to be waited for there.
struct OperandMeta {
  u32 w;            // this lane's block width
  SegmentOffsetParts seg_off;   // payload word offset of the wave's segment (uniform)
  u32 seg_end;                  // indexed streams: the payload word offset at which the segment ends (uniform)
  u32 payload_room;             // words between the start of the payload and the end of the caller's buffer (saturated)
};

// ... and after the scan of the widths: one operand ahead.
struct OperandPlace {
  u32 w;            // this lane's block width (0 if the block must be skipped)
  u32 pick;         // LDS word index of this lane's sign word
  u32 wcap;         // uniform: 0 (nothing to add), 4, 8, 12 or 16: at least the widest block of the wave
  u32 span;         // uniform: words the wave stages, from the aligned start
  u32 src0;         // uniform: payload word index of the aligned start
  u32 room;         // uniform: words from src0 to the end of the caller's buffer
};

// The tables of operand s for the wave's segment (seg: the same in every lane; b: the lane's
// block; both fit 32 bits because a stream has at most 2^26 blocks, and so do all byte offsets
// into the tables).  w_ok and seg_ok say which loads stay inside the stream and the index;
// they need not be the exact "block exists" conditions (the caller drops what it must not
// use), which lets a workgroup ask before it knows the header.
__device__ inline OperandMeta load_operand_tables(const ReduceArgs& a, int s, u32 seg, u32 b, bool w_ok, bool seg_ok,
                                                  u32 zero = 0) {
  OperandMeta m;
  const u8* base = a.in[s].base;
  m.seg_off = SegmentOffsetParts{0, 0, 0};
  if (seg_ok) m.seg_off = load_segment_offset(a.index, s, seg, zero);
  m.seg_end = 0;
  m.payload_room = 0;
  m.w = w_ok ? u32(*at_bytes(base, kHeaderBytes + b)) : 0u;
  return m;
}

__device__ inline i32 load_operand_outlier(const ReduceArgs& a, int s, const ParsedHeader& h, u32 b, bool active, bool ix) {
  const u8* base = a.in[s].base;
  return active ? *reinterpret_cast<const i32*>(at_bytes(base, u32(outliers_begin(h.nb, ix)) + 4u * b)) : 0;
}

__device__ inline u32 payload_room(const ReduceArgs& a, int s, const ParsedHeader& h, bool ix) {
  const u64 tend = tables_end(h.nb, ix);
  const u64 room = a.in[s].bytes > tend ? (a.in[s].bytes - tend) / 4 : 0;
  return room > 0xffffffffull ? 0xffffffffu : u32(room);   // a stream's payload has at most 2^31 words
}

// The payload is fenced in by the size of the caller's buffer, which a validated stream does
// not exceed (a 16-byte load may run up to 12 bytes past the stream's own end, inside the
// buffer; nothing reads those words).
// An indexed stream (ix) has the segment's position in its own index, and its width bytes
// behind that index (every stream of a validated call has the header's nb).
__device__ inline OperandMeta load_operand_meta(const ReduceArgs& a, int s, const ParsedHeader& h, u32 seg, u32 b,
                                                bool active, bool seg_live, bool ix) {
  OperandMeta m;
  if (ix) {
    const u8* base = a.in[s].base;
    m.seg_off = SegmentOffsetParts{0, 0, 0};
    m.seg_end = 0;
    if (seg_live) {
      m.seg_off = load_segment_offset(a.index, s, seg, 0, base);
      m.seg_end = load_segment_end(base, seg);
    }
    m.w = active ? u32(*at_bytes(base, u32(widths_begin(h.nb, true)) + b)) : 0u;
  } else {
    m = load_operand_tables(a, s, seg, b, active, seg_live);
  }
  m.payload_room = payload_room(a, s, h, ix);
  return m;
}

// `err`: an indexed stream is checked as it is used: the widths of the segment must add up to
// what the index says, and a stream that promised narrow blocks must have no other.
__device__ inline OperandPlace place_operand(const OperandMeta& m, const ParsedHeader& h, bool ix, u32& err) {
  OperandPlace p;
  // the same in every lane, and long since loaded: into scalar registers, 32-bit arithmetic
  const u64 seg_off64 = ix ? u64(uniform(m.seg_off.seg)) : uniform64(segment_offset(m.seg_off));
  const u32 seg_off = u32(seg_off64);
  const u32 w = m.w > 15 ? 0u : m.w;           // plain streams: cannot happen here; keeps every LDS access in range
  const u32 words = psize_words(w);
  const u32 incl = wave_inclusive_sum(words);
  const u32 wave_total = lane_value(incl, 63);
  // true on a validated stream
  bool inside = (seg_off64 >> 32) == 0 && seg_off <= m.payload_room && wave_total <= m.payload_room - seg_off;
  if (ix && (__any(m.w > 15) || uniform(m.seg_end) - seg_off != wave_total)) {
    err |= status_bit(ZC_ERR_FORMAT);
    inside = false;
  }
  const u32 mis = seg_off & 3u;
  p.src0 = seg_off - mis;
  p.room = m.payload_room - p.src0;
  p.span = inside ? mis + wave_total : 0u;     // <= 3 + 64 * 16
  p.pick = mis + (incl - words);
  p.w = inside ? w : 0u;
  p.wcap = __any(p.w > 12) ? 16u : __any(p.w > 8) ? 12u : __any(p.w > 4) ? 8u : __any(p.w != 0) ? 4u : 0u;
  return p;
}

// The operand's payload for this wave: 16 bytes per lane and load, all in flight together.
// The copy starts at the 16-byte boundary at or below the segment (the payload area itself is
// 16-byte aligned) and keeps that misalignment in LDS.  Four loads cover 1024 words; a wave
// whose 64 blocks are all 15 bits wide can need up to three more words, which stage_to_lds
// fetches on the spot.
constexpr int kStageLoads = 4;
struct OperandStage {
  uint4 v[kStageLoads];
};

__device__ inline OperandStage load_operand_payload(const u32* payload, const OperandPlace& p, int lane) {
  OperandStage st;
  const u32* src = payload + p.src0;             // uniform
#pragma unroll
  for (int i = 0; i < kStageLoads; ++i) {
    const u32 idx = 4u * u32(lane) + 256u * u32(i);
    st.v[i] = make_uint4(0, 0, 0, 0);
    // whole 16-byte pieces only: the last words of the caller's buffer are left to stage_to_lds (see load_wave_stage)
    if (idx < p.span && idx + 4 <= p.room) st.v[i] = load_once(reinterpret_cast<const uint4*>(src + idx));
  }
  return st;
}

__device__ inline void stage_to_lds(const OperandStage& st, const OperandPlace& p, const u32* payload, u32* wl, int lane) {
#pragma unroll
  for (int i = 0; i < kStageLoads; ++i) {
    const u32 idx = 4u * u32(lane) + 256u * u32(i);
    if (idx < p.span) *reinterpret_cast<uint4*>(wl + idx) = st.v[i];
  }
  const u32 staged = p.span < 256u * kStageLoads ? p.span : 256u * kStageLoads;
  if (((staged + 3u) & ~3u) > p.room) {            // uniform, and rare: the buffer ends inside a 16-byte piece
#pragma unroll
    for (int i = 0; i < kStageLoads; ++i) {
      const u32 idx = 4u * u32(lane) + 256u * u32(i);
      if (idx < p.span && idx + 4 > p.room) {
        for (u32 j = 0; j < 3; ++j)
          if (idx + j < p.room) wl[idx + j] = payload[p.src0 + idx + j];
      }
    }
  }
  if (p.span > 256u * kStageLoads) {               // uniform, and rare: words 1024 .. 1026
    const u32 idx = 256u * kStageLoads + u32(lane);
    if (idx < p.span) wl[idx] = payload[p.src0 + idx];
  }
}

// Three-input bitwise functions, one v_bitop3_b32 each.  The table is the function evaluated
// on a = 0xF0, b = 0xCC, c = 0xAA.
__device__ inline u32 xor3(u32 a, u32 b, u32 c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96); }
__device__ inline u32 majority(u32 a, u32 b, u32 c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8); }
__device__ inline u32 and_xor(u32 a, u32 b, u32 c) { return __builtin_amdgcn_bitop3_b32(a, b, c, 0x6A); }   // (a & b) ^ c

// acc += operand, planes [4C, 4C + 4).  DATA: the operand has magnitude planes here, read
// from LDS (`mine` points at the lane's sign word) and masked by the block's own width (bit P
// of `keep` is set iff the block has plane P); otherwise the operand only contributes its
// sign extension.  Four instructions per plane: mask, operand bit, sum, carry.
template <int C, bool DATA>
__device__ inline void add_chunk(u32 (&acc)[kSumPlanes], const u32* mine, u32 keep, u32 sgn, u32& carry) {
#pragma unroll
  for (int i = 0; i < kSumChunk; ++i) {
    constexpr int kFirst = C * kSumChunk;
    const int P = kFirst + i;
    u32 x = sgn;                                  // two's complement of the operand: (mag ^ s) + s
    if (DATA) {
      const u32 m = u32(__builtin_amdgcn_sbfe(i32(keep), u32(P), 1u));   // all ones iff the block has plane P
      x = and_xor(mine[1 + P], m, sgn);
    }
    const u32 cur = acc[P];                       // full adder
    acc[P] = xor3(cur, x, carry);
    carry = majority(cur, x, carry);
  }
}

template <int C>
__device__ inline void add_operand_chunks(u32 (&acc)[kSumPlanes], const u32* mine, u32 keep, u32 sgn, u32& carry,
                                          u32 wcap, u32 top) {
  if constexpr (C * kSumChunk < kSumPlanes) {
    if (u32(C * kSumChunk) >= top) return;        // uniform
    if (C * kSumChunk < 16 && u32(C * kSumChunk) < wcap) add_chunk<C, true>(acc, mine, keep, sgn, carry);
    else add_chunk<C, false>(acc, mine, keep, sgn, carry);
    add_operand_chunks<C + 1>(acc, mine, keep, sgn, carry, wcap, top);
  }
}

// Extends the valid planes from `top` to `new_top` with copies of the sign plane.
template <int C>
__device__ inline void grow_sum(u32 (&acc)[kSumPlanes], u32 top, u32 new_top) {
  if constexpr (C * kSumChunk < kSumPlanes) {
    if (u32(C * kSumChunk) >= new_top) return;    // uniform
    if (u32(C * kSumChunk) >= top) {
      u32 e = 0;
      if constexpr (C > 0) e = acc[C * kSumChunk - 1];
#pragma unroll
      for (int i = 0; i < kSumChunk; ++i) acc[C * kSumChunk + i] = e;
    }
    grow_sum<C + 1>(acc, top, new_top);
  }
}

// Two's complement planes -> magnitude planes (in place), given the sign plane; tracks the width.
template <int C>
__device__ inline void sum_to_magnitude(u32 (&acc)[kSumPlanes], u32 sgn, u32& carry, u32& width, u32 top) {
  if constexpr (C * kSumChunk < kSumPlanes) {
    if (u32(C * kSumChunk) >= top) {
#pragma unroll
      for (int i = 0; i < kSumChunk; ++i) acc[C * kSumChunk + i] = 0;
    } else {
#pragma unroll
      for (int i = 0; i < kSumChunk; ++i) {
        constexpr int kFirst = C * kSumChunk;
        const int P = kFirst + i;
        const u32 t = acc[P] ^ sgn;
        const u32 m = t ^ carry;
        carry = t & carry;
        acc[P] = m;
        width = m ? u32(P + 1) : width;
      }
    }
    sum_to_magnitude<C + 1>(acc, sgn, carry, width, top);
  }
}

template <int C>
__device__ inline u32 sign_plane(const u32 (&acc)[kSumPlanes], u32 top) {
  if constexpr ((C + 1) * kSumChunk > kSumPlanes) {
    return 0u;
  } else {
    if (top == u32((C + 1) * kSumChunk)) return acc[(C + 1) * kSumChunk - 1];
    return sign_plane<C + 1>(acc, top);
  }
}

// The lane number, in a way that keeps the compiler from recognising two calls as the same value.
// What an operand step derives from the lane number is cheap to compute and is computed on
// the spot: hoisted out of the loop over the operands it would sit in registers that the
// adder needs.
__device__ inline int fresh_lane() {
  int lane = lane_id();
  asm volatile("" : "+v"(lane));
  return lane;
}

// One tile of a call whose operands have no block wider than 15 bits.  `meta`: the tables of
// operand 0 if the workgroup asked for them early (`early`).
template <bool IX>
__device__ inline void reduce_narrow_tile(const ReduceArgs& a, const ReduceCall& c, u32 tile, u32 ntiles, OperandMeta meta,
                                          bool early, u32* lds, u32* sh_wave_total, u64* sh_base) {
  const ParsedHeader& h = c.h;
  const int wave = wave_id();
  const u64 tend = tables_end(h.nb, IX);
  u32* const wl = lds + wave * kWholeStage;
  const u32 seg = tile * kTileWaves + u32(wave);
  const bool seg_live = seg < num_segments(h.nb);
  OperandPlace next;
  OperandStage stage;
  i32 outlier_next;        // the outlier of the operand in `stage`: travels with the payload
  u32 err = 0;             // uniform
  {
    const int lane = fresh_lane();
    const u32 b = seg * kWaveBlocks + u32(lane);
    const bool active = b < h.nb;
    if (early) {
      if (!active) meta.w = 0;
      if (!seg_live) {
        meta.seg_off = SegmentOffsetParts{0, 0, 0};
        meta.seg_end = 0;
      }
      meta.payload_room = payload_room(a, 0, h, IX);
    } else {
      meta = load_operand_meta(a, 0, h, seg, b, active, seg_live, IX);
    }
    next = place_operand(meta, h, IX, err);
    if (a.k > 1) meta = load_operand_meta(a, 1, h, seg, b, active, seg_live, IX);
    stage = load_operand_payload(reinterpret_cast<const u32*>(a.in[0].base + tend), next, lane);
    outlier_next = load_operand_outlier(a, 0, h, b, active, IX);
  }
  // the ends of every operand's index, by the waves that hold them
  if (IX && seg_live && !index_ends_consistent(a.in, a.k, h, seg)) err |= status_bit(ZC_ERR_FORMAT);

  // ---- add the k operands' blocks in plane form; loads run ahead of the adds ----
  u32 acc[kSumPlanes];
#pragma unroll
  for (int p = 0; p < kSumPlanes; ++p) acc[p] = 0;
  u32 top = 0;
  u32 bound = 0;          // wave-uniform bound on |sum of deltas| so far (< 64 * 2^16)
  i64 outlier = 0;
  for (int s = 0; s < a.k; ++s) {
    const int lane = fresh_lane();
    const u32 b = seg * kWaveBlocks + u32(lane);
    const bool active = b < h.nb;
    const OperandPlace cur = next;
    stage_to_lds(stage, cur, reinterpret_cast<const u32*>(a.in[s].base + tend), wl, lane);
    wave_lds_sync();
    outlier += i64(outlier_next);
    if (s + 1 < a.k) {
      next = place_operand(meta, h, IX, err);
      if (s + 2 < a.k) meta = load_operand_meta(a, s + 2, h, seg, b, active, seg_live, IX);
      stage = load_operand_payload(reinterpret_cast<const u32*>(a.in[s + 1].base + tend), next, lane);
      outlier_next = load_operand_outlier(a, s + 1, h, b, active, IX);
    }
    if (cur.wcap) {
      bound += (1u << cur.wcap) - 1u;
      u32 new_top = (32u - u32(__builtin_clz(bound)) + 1u + 3u) & ~3u;
      if (new_top > u32(kSumPlanes)) new_top = kSumPlanes;      // cannot happen for k <= 64
      grow_sum<0>(acc, top, new_top);
      top = new_top;
      const u32* mine = wl + cur.pick;
      const u32 sgn = cur.w ? mine[0] : 0u;
      u32 carry = sgn;
      const u32 keep = (1u << cur.w) - 1u;      // bit P set iff the block has plane P
      add_operand_chunks<0>(acc, mine, keep, sgn, carry, cur.wcap, top);
    }
    wave_lds_sync();
  }

  // ---- back to sign + magnitude planes; new code length; placement and copy-out ----
  const u32 sgn = sign_plane<0>(acc, top);
  u32 carry = sgn, w = 0;
  sum_to_magnitude<0>(acc, sgn, carry, w, top);
  auto word = [&](auto i) {
    constexpr int I = decltype(i)::value;        // 0: sign, 1 + p: plane p
    if constexpr (I == 0) return sgn;
    else return acc[I - 1];
  };
  const int lane = fresh_lane();
  const u32 b = seg * kWaveBlocks + u32(lane);
  if (IX && err && lane == 0) raise_status(a.ctl, c.tag, err);
  place_sum_staged<kSumPlanes>(a, c, acc, sgn, w, outlier, b < h.nb, b, tile, ntiles, word, wl, sh_wave_total, sh_base,
                               wave, lane, IX);
}

// ---------------------------------------------------------------------------------------
// Any widths.
// ---------------------------------------------------------------------------------------
constexpr int kAccPlanes = 38;   // |sum of 64 deltas| < 2^37: 37 magnitude bits + sign
constexpr int kWideChunk = 2;    // operand planes fetched at a time

// acc (two's complement, `top` planes valid, `ext` = its sign plane) += operand given as sign
// word s and the magnitude planes at src[1 ...] (w of them; zero above), kWideChunk planes at
// a time: their loads are in flight together, then they are added.  Planes [0, new_top) are
// valid afterwards.  top and new_top are wave-uniform.
template <int P0>
__device__ inline void ripple_add(u32 (&acc)[kAccPlanes], const u32* src, u32 w, u32 s, u32 carry, u32 ext, u32 top,
                                  u32 new_top, u32& ext_out) {
  if constexpr (P0 < kAccPlanes) {
    if (u32(P0) >= new_top) return;             // uniform
    u32 x[kWideChunk];
#pragma unroll
    for (int i = 0; i < kWideChunk; ++i) {
      const int P = P0 + i;
      x[i] = (P < 31 && u32(P) < w) ? src[1 + P] : 0u;
    }
#pragma unroll
    for (int i = 0; i < kWideChunk; ++i) {
      const int P = P0 + i;
      if (P < kAccPlanes && u32(P) < new_top) {
        const u32 cur = u32(P) < top ? acc[P] : ext;
        const u32 xx = s ^ x[i];                // two's complement of the operand: (mag ^ s) + s
        const u32 t = cur ^ xx;
        const u32 sum = t ^ carry;
        carry = (t & carry) | (~t & cur);       // majority(cur, xx, carry)
        acc[P] = sum;
        ext_out = sum;
      }
    }
    ripple_add<P0 + kWideChunk>(acc, src, w, s, carry, ext, top, new_top, ext_out);
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

template <bool IX>
__device__ inline void reduce_wide_tile(const ReduceArgs& a, const ReduceCall& c, u32 tile, u32 ntiles, u32* lds,
                                        u32* sh_wave_total, u64* sh_base) {
  const ParsedHeader& h = c.h;
  const u64 tend = tables_end(h.nb, IX);
  const int lane = lane_id();
  const int wave = wave_id();
  u32* const wl = lds + wave * kWholeStage;
  const u32 seg = tile * kTileWaves + u32(wave);           // a stream has at most 2^26 blocks
  const bool seg_live = seg < num_segments(h.nb);
  const u32 b = seg * kWaveBlocks + u32(lane);
  const bool active = b < h.nb;
  if (IX && seg_live && !index_ends_consistent(a.in, a.k, h, seg) && lane == 0)
    raise_status(a.ctl, c.tag, status_bit(ZC_ERR_FORMAT));

  u32 acc[kAccPlanes];
#pragma unroll
  for (int p = 0; p < kAccPlanes; ++p) acc[p] = 0;
  u32 ext = 0, top = 0;
  u64 bound = 0;          // wave-uniform bound on |sum of deltas| so far
  i64 outlier = 0;
#pragma nounroll
  for (int s = 0; s < a.k; ++s) {
    const u8* base = a.in[s].base;
    const u64 total_s = reinterpret_cast<const u64*>(base)[3];
    const u64 pw64 = total_s >= tend ? (total_s - tend) / 4 : 0;
    const u32 pw = pw64 > 0xffffffffull ? 0xffffffffu : u32(pw64);   // payload words (a stream has at most 2^31)
    u32 w = active ? u32(*at_bytes(base, u32(widths_begin(h.nb, IX)) + b)) : 0u;
    const bool bad_w = w > 31;                    // plain streams: cannot happen on a validated stream
    if (bad_w) w = 0;
    const u32 words = psize_words(w);
    const u32 incl = wave_inclusive_sum(words);
    u32 seg_off = 0;
    bool fits = seg_live;
    if (IX) {
      // the segment's place by the stream's own index, which must agree with the widths
      const u32* index = reinterpret_cast<const u32*>(base + kHeaderBytes);
      const u32 seg_end = seg_live ? index[seg + 1] : 0u;
      seg_off = seg_live ? index[seg] : 0u;
      const bool narrow_promised = (reinterpret_cast<const u32*>(base)[1] & 1u) == 0;
      if (seg_end - seg_off != lane_value(incl, 63) || __any(bad_w) || (narrow_promised && __any(w > 15))) {
        if (lane == 0) raise_status(a.ctl, c.tag, status_bit(ZC_ERR_FORMAT));
        fits = false;
      }
    } else if (seg_live) {
      const u64 so = segment_offset(a.index, s, seg);
      fits = so <= pw;
      seg_off = u32(so);
    }
    // (cannot fail on a validated stream) the segment lies inside the payload
    if (!fits || seg_off > pw || lane_value(incl, 63) > pw - seg_off) w = 0;
    const u32 wmax = wave_max_u32(w);
    if (active) outlier += i64(*reinterpret_cast<const i32*>(at_bytes(base, u32(outliers_begin(h.nb, IX)) + 4u * b)));
    if (wmax == 0) continue;
    const u32* src = reinterpret_cast<const u32*>(base + tend) + seg_off + (incl - words);
    const u32 sgn = w ? src[0] : 0u;
    bound += (u64(1) << wmax) - 1;
    u32 new_top = 64u - u32(__builtin_clzll(bound)) + 1u;
    if (new_top > u32(kAccPlanes)) new_top = kAccPlanes;
    u32 ext_out = ext;
    ripple_add<0>(acc, src, w, sgn, sgn, ext, top, new_top, ext_out);
    ext = ext_out;
    top = new_top;
  }

  u32 w = 0;
  magnitude_planes<0>(acc, ext, ext, top, w);
  auto word = [&](auto i) {
    constexpr int I = decltype(i)::value;        // 0: sign, 1 + p: plane p
    if constexpr (I == 0) return ext;
    else return acc[I - 1];
  };
  place_sum<32>(a, c, acc, ext, w, outlier, active, b, tile, ntiles, word, wl, sh_wave_total, sh_base, wave, lane, IX);
}

// What every workgroup of a reduce kernel does first: the call's verdict, tag and header, and its tile.
// Returns false when the workgroup has nothing (more) to do.  Plain streams (IX false) have
// been validated and indexed by the kernels of zc_scan.h, whose verdict and tag are in the
// control block; indexed streams are judged here, by every workgroup alike, from their headers.
// `meta`, `early`: see reduce_narrow_tile.  `for_wide`: the caller is the kernel that serves
// streams with blocks wider than 15 bits (the narrow one returns at once on those, and
// the other way round; either writes the header of its own calls); `split`: indexed streams
// have such a pair of kernels as well (otherwise one kernel takes both kinds).
template <bool IX>
__device__ inline bool open_reduce(const ReduceArgs& a, bool for_wide, bool split, ReduceCall& c, bool& wide, OperandMeta& meta,
                                   bool early, u32& tile, u32& ntiles, u32* sh_tile) {
  c.ltag = launch_tag(a.nonce, a.ctl);
  // (with tickets the ticket is asked for first of all: its round trip runs beside the headers')
  u64 asked = 0;
  if (a.ticketed && threadIdx.x == 0) asked = ask_ticket(ticket_counter(a.ctl, ticket_shard()));
  if (IX) {
    if (early) {
      // the caller has said what n is (a reduce in parts): where the first operand's tables are follows from
      // that, and they are asked for together with the headers; a stream of another n ends the call below
      const u32 nb_said = u32(num_blocks(a.n_part));
      const u32 seg = (a.first_tile + blockIdx.x) * kTileWaves + u32(wave_id());
      const u32 b = seg * kWaveBlocks + u32(fresh_lane());
      const u8* base = a.in[0].base;
      const u32 zero = opaque_zero();
      const bool seg_ok = seg < num_segments(nb_said) && u64(kHeaderBytes) + 4ull * seg + 8 <= a.in[0].bytes;
      const bool w_ok = b < nb_said && widths_begin(nb_said, true) + b < a.in[0].bytes;
      meta.seg_off = SegmentOffsetParts{0, 0, 0};
      meta.seg_end = 0;
      if (seg_ok) {
        meta.seg_off = load_segment_offset(a.index, 0, seg, zero, base);
        meta.seg_end = load_segment_end(base, seg, zero);
      }
      meta.w = w_ok ? u32(*at_bytes(base, u32(widths_begin(nb_said, true)) + b + zero)) : 0u;
    }
    const StreamsVerdict v = judge_indexed_streams(a.in, a.k, true);
    // (of a pair of kernels the narrow one is launched first and opens the call; a later part of a
    //  reduce done in parts belongs to the call its first part opened)
    const bool adopt = a.adopt != 0 || (split && for_wide);
    c.tag = call_tag(a.ctl, c.ltag, adopt);
    c.h = v.h0;
    c.nsum = v.nsum;
    wide = v.wide;
    if (v.err) {
      if (blockIdx.x == 0 && threadIdx.x == 0 && !(split && for_wide)) {
        if (!a.adopt) a.ctl->result = 0;
        raise_status(a.ctl, c.tag, v.err);
      }
      return false;
    }
    if (a.n_part && a.n_part != c.h.n) {      // the parts were laid out for another n
      if (blockIdx.x == 0 && threadIdx.x == 0) raise_status(a.ctl, c.tag, status_bit(ZC_ERR_MISMATCH));
      return false;
    }
    if (split && wide != for_wide) return false;
  } else {
    const u32 zero = opaque_zero();
    if (early) {
      const u32 seg = blockIdx.x * kTileWaves + u32(wave_id());     // < 2^22: the host launches at most 2^18 tiles
      const u32 b = seg * kWaveBlocks + u32(fresh_lane());
      meta = load_operand_tables(a, 0, seg, b, u64(kHeaderBytes) + b < a.in[0].bytes, seg < 4 * a.index.tiles_cap, zero);
    }
    const uint4 gate_raw = load_gate(a.ctl, zero);
    const HeaderWords hw = load_header_words(a.in[0].base, zero);
    c.h = parse_header(hw, a.in[0].bytes, false);
    const Gate gate = parse_gate(gate_raw);
    c.tag = gate.tag;
    if (gate_failed(gate) || !c.h.ok) return false;
    wide = gate_wide(gate);
    if (wide != for_wide) return false;
    c.nsum = 0;
  }
  ntiles = u32(num_tiles(c.h.nb));
  const u32 end_tile = a.end_tile && a.end_tile < ntiles ? a.end_tile : ntiles;
  c.part_end = a.end_tile ? end_tile : 0u;
  if (blockIdx.x == 0 && threadIdx.x == 0 && a.first_tile == 0) {
    if (!IX) c.nsum = a.ctl->nsum;           // of all operands, summed by the validation kernel
    write_reduce_header(a, c, ntiles, IX);
  }
  if (ntiles == 0) {                         // streams without blocks: their one index entry must say so
    if (IX && blockIdx.x == 0 && wave_id() == 0 && !index_ends_consistent(a.in, a.k, c.h, 0) && lane_id() == 0)
      raise_status(a.ctl, c.tag, status_bit(ZC_ERR_FORMAT));
    return false;
  }
  if (a.first_tile >= end_tile) return false;
  tile = a.first_tile + blockIdx.x;          // tiles in the order in which workgroups start
  if (a.ticketed) {                          // ... or handed out by tickets, see take_tile
    if (threadIdx.x == 0) {
      const u32 t = take_tile(a.ctl, c.ltag, end_tile - a.first_tile, ticket_shard(), asked);
      *sh_tile = t == kNoTile ? kNoTile : a.first_tile + t;
    }
    __syncthreads();
    tile = uniform(*sh_tile);
  }
  return tile < end_tile;
}

// Indexed streams: one launch per call, whatever the widths.  Plain streams: the common case;
// reduce_wide_kernel, launched behind it, takes the calls with wider blocks.
template <bool IX>
__global__ __launch_bounds__(kTileThreads, 6) void reduce_kernel(ReduceArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWholeStage];   // also holds an operand's payload
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  ReduceCall c;
  bool wide = false;
  OperandMeta meta{};
  // A workgroup that takes the tile of its own number asks for the first operand's tables
  // together with the control block and the header, before it knows the header: one memory
  // round trip instead of two.  The loads are fenced in by sizes the host passed.  (Not for
  // indexed streams: where their width bytes are is only known with the header.)
  const bool early = !a.ticketed && (!IX || a.n_part != 0);
  u32 tile = 0, ntiles = 0;
  if (!open_reduce<IX>(a, false, false, c, wide, meta, early, tile, ntiles, &sh_tile)) return;
  if (IX && wide) reduce_wide_tile<true>(a, c, tile, ntiles, lds, sh_wave_total, &sh_base);
  else reduce_narrow_tile<IX>(a, c, tile, ntiles, meta, early, lds, sh_wave_total, &sh_base);
}

// Plain streams with blocks wider than 15 bits.
__global__ __launch_bounds__(kTileThreads) void reduce_wide_kernel(ReduceArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWholeStage];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  ReduceCall c;
  bool wide = false;
  OperandMeta meta{};
  u32 tile = 0, ntiles = 0;
  if (!open_reduce<false>(a, true, true, c, wide, meta, false, tile, ntiles, &sh_tile)) return;
  reduce_wide_tile<false>(a, c, tile, ntiles, lds, sh_wave_total, &sh_base);
}

}  // namespace zc

// Placement of a tile's variable-size payload in the output stream, shared by the kernels
// that write streams (compression and the fused reduce): the tile publishes its size, looks
// back for its base offset (the exclusive sum of the sizes of all tiles before it, in block
// order), and copies its packed words out through LDS as coalesced stores.
#pragma once

#include <type_traits>
#include <utility>

#include "zc_common.h"

namespace zc {

// The stream being written.
struct PayloadSink {
  u8* out;          // stream base
  u64 out_cap;      // bytes
  u64 nb;           // blocks of the stream
  Control* ctl;
  u64* desc;        // look-back descriptors
  bool ix;          // the stream carries a segment index (see index_bytes)
  bool coherent;    // the look-back reads the tile's own chain with device-coherent loads (ZC_CHAINS_COHERENT)
  u32 part_end;     // a stream produced in parts (zc_compress_part): one past the last tile of this part; else 0
  u64 tag;          // the call's tag (see launch_tag): descriptors and status bits carry it
};

// Per-wave view of where its payload goes.
struct Placement {
  u32 w, wmax;              // this block's width; the widest of the wave
  u32 off_in_wave;          // payload word offset of this block inside the wave
  u32 half0_total, wave_total;
  u32 wave_off, tile_total; // the wave inside the tile; payload words of the tile
  bool tile_wide;           // some block of the tile is wider than 15 bits (only indexed streams record it)
};

// Where a tile starts, as resolve_tile_base hands it out.
struct TileBase {
  u64 words;                // payload words of all tiles before this one
  bool wide_so_far;         // this tile or one before it holds a block wider than 15 bits
};

// The waves of a tile tell each other their payload sizes through LDS; a wave that writes an
// indexed stream marks its size when it holds a block wider than 15 bits.
constexpr u32 kWaveWideMark = 1u << 31;

__device__ inline void sum_wave_totals(const u32* sh_wave_total, int wave, bool ix, Placement& pl) {
  pl.wave_off = 0;
  pl.tile_total = 0;
  u32 marks = 0;
#pragma unroll
  for (int i = 0; i < kTileWaves; ++i) {
    u32 t = sh_wave_total[i];
    if (ix) {
      marks |= t;
      t &= ~kWaveWideMark;
    }
    if (i < wave) pl.wave_off += t;
    pl.tile_total += t;
  }
  pl.tile_wide = ix && (marks & kWaveWideMark) != 0;
}

// Fixed header fields and the zero padding of the tables of the stream being written; one
// thread, and out_cap >= tables_end.  The version word of an indexed stream, total_bytes and
// the closing entry of the index belong to the last tile (finish_stream), whose stores must
// not meet others to the same bytes from the same kernel: `closing` says that no tile follows
// in this kernel (an empty stream, or a kernel of its own ahead of the tiles), and has them
// written here, for an empty payload.
__device__ inline void write_stream_header(u8* out, u64 n, u64 nb, u32 eb_bits, u32 nsum, bool ix, bool closing) {
  const u64 tend = tables_end(nb, ix);
  const u64 nseg = num_segments(nb);
  u32* hw = reinterpret_cast<u32*>(out);
  hw[0] = kMagic;
  if (!ix) hw[1] = kVersionPlain;
  hw[2] = u32(n);
  hw[3] = u32(n >> 32);
  hw[4] = eb_bits;
  hw[5] = nsum;
  if (closing) {
    if (ix) hw[1] = kVersionIndexed;
    hw[6] = u32(tend);
    hw[7] = u32(tend >> 32);
    if (ix) hw[kHeaderBytes / 4 + nseg] = 0;
  }
  if (ix)
    for (u64 i = nseg + 1; i < index_bytes(nb, true) / 4; ++i) hw[kHeaderBytes / 4 + i] = 0;
  u8* wt = out + widths_begin(nb, ix);
  for (u64 i = nb; i < pad16(nb); ++i) wt[i] = 0;
  u8* ot = out + outliers_begin(nb, ix);
  for (u64 i = 4 * nb; i < pad16(4 * nb); ++i) ot[i] = 0;
}

// Copies `limit` staged words of a wave to dst with coalesced stores that each cover whole 128-byte
// lines of memory (the first and the last line of the run aside): lane 0 of every store sits on a
// line boundary, so a line is written by one instruction and not by the tail of one and the head of
// the next.  The stores bypass the caches: a stream is on its way to another device, or to a later
// call, and keeping it in cache lines would only push the write-back into the kernels that follow.
// ROUNDS * 64 >= limit + 31.
template <int ROUNDS>
__device__ inline void copy_staged_words(const u32* wl, u32* dst, u32 limit, int lane) {
  const u32 lead = uniform(u32(reinterpret_cast<uintptr_t>(dst) >> 2) & 31u);   // words of dst's line before dst
  const u32 end = uniform(limit) + lead;
  // four rounds at a time: their LDS reads are all under way before the first store needs its word
#pragma unroll
  for (int r0 = 0; r0 < ROUNDS; r0 += 4) {
    if (64u * u32(r0) >= end) break;           // uniform
    u32 i[4], v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      i[k] = u32(lane) + 64u * u32(r0 + k) - lead;   // wraps for the lanes ahead of dst: they sit out
      v[k] = wl[i[k] < limit ? i[k] : 0u];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (r0 + k < ROUNDS && i[k] < limit) store_once(dst + i[k], v[k]);
  }
}

// Writes the payload words of the lanes of one half-wave to the wave's staging area and copies
// them out with coalesced stores.  Word 0 is the sign word, word 1 + p is plane p; `word(i)`
// yields word i from registers and is only ever called with compile-time constants.
// half_total <= 32 * NW.
template <int NW, typename WordFn>
__device__ inline void stage_and_copy_half(WordFn word, u32 w, bool in_half, u32 off_in_half, u32 half_total,
                                           u32* wl, u32* dst, u64 dst_room, int lane) {
  if (in_half && w) {
    wl[off_in_half] = word(std::integral_constant<int, 0>{});
    [&]<int... P>(std::integer_sequence<int, P...>) {
      ((u32(P) < w ? void(wl[off_in_half + 1 + P] = word(std::integral_constant<int, 1 + P>{})) : void()), ...);
    }(std::make_integer_sequence<int, NW - 1>{});
  }
  wave_lds_sync();
  const u32 limit = u64(half_total) < dst_room ? half_total : u32(dst_room);
  copy_staged_words<NW / 2 + 1>(wl, dst, limit, lane);
  wave_lds_sync();
}

// Publishes the tile's payload size; called by one thread as soon as the size is known,
// because the tiles after this one wait for it.
__device__ inline void publish_tile_size(const PayloadSink& s, u32 tile, u32 tile_total, bool tile_wide) {
  // (the first tile of a chain has nothing before it in the chain: its size is its chain sum)
  desc_store(s.desc, tile,
             (tile < u32(kChains) ? kDescChain : kDescAggregate) | (tile_wide ? kDescWide : 0) | u64(tile_total), s.tag);
}

// Base offset of the tile, in payload words: wave 0 looks back (see "Look-back by chains"),
// everyone meets at one barrier.  The tile's size must have been published.  Called by every wave
// of the workgroup.  `meanwhile()` runs in every wave: in the other waves while wave 0 looks back,
// in wave 0 between the publication of its chain sum and its poll of the other chains, whose
// tiles publish their chain sums at about the same time: a poll that goes out a little later
// more often finds them and saves a second one (measured: 1 % over the whole kernel against
// the poll ahead of `meanwhile()`).
template <typename MeanwhileFn>
__device__ inline TileBase resolve_tile_base(const PayloadSink& s, const Placement& pl, u32 tile, u64* sh_base, int wave,
                                             int lane, MeanwhileFn meanwhile) {
  u32 own = 0;              // sizes of the tile's chain before it
  u64 wide = pl.tile_wide ? kDescWide : 0;
  if (wave == 0 && tile >= u32(kChains)) {
    u64 own_wide = 0;
    if (s.coherent || !own_chain_scalar(s.desc, tile, s.tag, own, own_wide)) {
      const u64 v = chains_lookback(s.desc, tile, s.ctl, s.tag, kOwnChain);
      own = u32(v);
      own_wide = v & kDescWide;
    }
    wide |= own_wide;
    if (lane == 0) desc_store(s.desc, tile, kDescChain | wide | u64(u32(own + pl.tile_total)), s.tag);
  }
  meanwhile();
  if (wave == 0) {
    // words of the tiles before this one, and kDescWide if one of them, or this one, is wide
    const u64 others = chains_lookback(s.desc, tile, s.ctl, s.tag, kOtherChains);
    if (lane == 0) *sh_base = u64(u32(own + u32(others))) | wide | (others & kDescWide);
  }
  lds_barrier();                // only sh_base passes through it
  const u64 before = *sh_base;
  return TileBase{before & kDescValueMask, (before & kDescWide) != 0};
}

__device__ inline TileBase resolve_tile_base(const PayloadSink& s, const Placement& pl, u32 tile, u64* sh_base, int wave,
                                             int lane) {
  return resolve_tile_base(s, pl, tile, sh_base, wave, lane, [] {});
}

// Index entry of a segment of the stream being written: one lane of the wave that owns it.
__device__ inline void write_index_entry(const PayloadSink& s, u32 seg, u64 seg_words_before) {
  if (s.ix && u64(seg) < num_segments(s.nb) && s.out_cap >= tables_end(s.nb, true))
    reinterpret_cast<u32*>(s.out + kHeaderBytes)[seg] = u32(seg_words_before);
}

// The last tile knows the size of the stream, and of an indexed one whether it holds wide blocks.
// The last tile of a part of a stream that is produced in parts writes the same for the stream
// so far: what has been produced is then a stream that can be read up to there.
__device__ inline void finish_stream(const PayloadSink& s, const Placement& pl, u32 tile, u32 ntiles, const TileBase& tb) {
  if ((tile == ntiles - 1 || tile + 1 == s.part_end) && threadIdx.x == 0) {
    const u64 words = tb.words + pl.tile_total;
    const u64 total = tables_end(s.nb, s.ix) + 4 * words;
    s.ctl->result = total;
    if (total > s.out_cap) raise_status(s.ctl, s.tag, status_bit(ZC_ERR_CAPACITY));
    if (s.out_cap >= kHeaderBytes) reinterpret_cast<u64*>(s.out)[3] = total;
    if (s.ix && s.out_cap >= tables_end(s.nb, true)) {
      u32* hw = reinterpret_cast<u32*>(s.out);
      hw[1] = kVersionIndexed | (tb.wide_so_far ? 1u : 0u);
      hw[kHeaderBytes / 4 + num_segments(s.nb)] = u32(words);      // the closing entry of the index
      // the end of a part is where the next part's first segment will start: its entry, ahead of time,
      // lets the last segment of this part be checked and read before the next part exists
      const u64 next_seg = u64(tile + 1) * (blockDim.x >> 6);
      if (next_seg < num_segments(s.nb)) hw[kHeaderBytes / 4 + next_seg] = u32(words);
    }
  }
}

// Moves a wave's payload out once the tile's base offset is known: through LDS, one half-wave
// of blocks at a time (the staging area `wl` of a wave holds kWaveStage words).
template <int NW, typename WordFn>
__device__ inline void copy_wave_out(const PayloadSink& s, WordFn word, const Placement& pl, u64 base, u32* wl, int lane) {
  static_assert(32 * NW <= kWaveStage, "a half-wave of widest blocks must fit the staging area");
  const u64 tend = tables_end(s.nb, s.ix);
  const u64 cap_words = s.out_cap > tend ? (s.out_cap - tend) / 4 : 0;
  u32* const payload = reinterpret_cast<u32*>(s.out + tend);
  const u64 dst0 = base + pl.wave_off;
  const u32 half_base[2] = {0u, pl.half0_total};
  const u32 half_total[2] = {pl.half0_total, pl.wave_total - pl.half0_total};
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const u64 d0 = dst0 + half_base[h];
    stage_and_copy_half<NW>(word, pl.w, (lane >> 5) == h, pl.off_in_wave - half_base[h], half_total[h], wl,
                            payload + d0, cap_words > d0 ? cap_words - d0 : 0, lane);
  }
}

// The same in one pass, for a wave whose whole payload fits its staging area (64 * NW words), in two
// steps.  First every lane writes its block's words to the staging area at the block's offset inside
// the wave: this needs no base offset, so it can be done while the look-back is under way.
template <int NW, typename WordFn>
__device__ inline void stage_wave_words(WordFn word, const Placement& pl, u32* wl) {
  if (pl.w) {
    wl[pl.off_in_wave] = word(std::integral_constant<int, 0>{});
    [&]<int... P>(std::integer_sequence<int, P...>) {
      ((u32(P) < pl.w ? void(wl[pl.off_in_wave + 1 + P] = word(std::integral_constant<int, 1 + P>{})) : void()), ...);
    }(std::make_integer_sequence<int, NW - 1>{});
  }
}

// Then the copy-out is a plain LDS-to-memory copy of the wave's words.
template <int NW>
__device__ inline void copy_staged_wave(const PayloadSink& s, const Placement& pl, u64 base, u32* wl, int lane) {
  wave_lds_sync();
  const u64 tend = tables_end(s.nb, s.ix);
  const u64 cap_words = s.out_cap > tend ? (s.out_cap - tend) / 4 : 0;
  const u64 d0 = base + pl.wave_off;
  u32* const dst = reinterpret_cast<u32*>(s.out + tend) + d0;
  const u64 room = cap_words > d0 ? cap_words - d0 : 0;
  const u32 limit = u64(pl.wave_total) < room ? pl.wave_total : u32(room);
  copy_staged_words<NW + 1>(wl, dst, limit, lane);
  wave_lds_sync();
}

// Back half of a tile whose size is published: look back for the base offset, then move the
// payload out.  Called by every wave of the workgroup; one barrier.  `make_words()` runs while the
// look-back's first poll is on its way and leaves the wave's words in its staging area (see
// stage_wave_words): whatever turns the tile's codes into plane words belongs there.
template <int NW, typename MakeWordsFn>
__device__ inline void finish_staged_tile(const PayloadSink& s, const Placement& pl, u32 tile, u32 ntiles, u32* wl,
                                          u64* sh_base, int wave, int lane, MakeWordsFn make_words) {
  static_assert(64 * NW <= kWaveStage, "a wave of widest blocks must fit the staging area");
  const TileBase tb = resolve_tile_base(s, pl, tile, sh_base, wave, lane, make_words);
  if (lane == 0) write_index_entry(s, tile * (blockDim.x >> 6) + u32(wave), tb.words + pl.wave_off);
  copy_staged_wave<NW>(s, pl, tb.words, wl, lane);
  finish_stream(s, pl, tile, ntiles, tb);
}

// The same with the plane words in registers (`word(i)`: 0 = sign, 1 + p = plane p), for waves
// whose payload need not fit the staging area at once.
template <int NW, typename WordFn, typename MeanwhileFn>
__device__ inline void finish_tile(const PayloadSink& s, WordFn word, const Placement& pl, u32 tile, u32 ntiles,
                                   u32* wl, u64* sh_base, int wave, int lane, MeanwhileFn meanwhile) {
  const TileBase tb = resolve_tile_base(s, pl, tile, sh_base, wave, lane, meanwhile);
  if (lane == 0) write_index_entry(s, tile * (blockDim.x >> 6) + u32(wave), tb.words + pl.wave_off);
  copy_wave_out<NW>(s, word, pl, tb.words, wl, lane);
  finish_stream(s, pl, tile, ntiles, tb);
}

template <int NW, typename WordFn>
__device__ inline void finish_tile(const PayloadSink& s, WordFn word, const Placement& pl, u32 tile, u32 ntiles,
                                   u32* wl, u64* sh_base, int wave, int lane) {
  finish_tile<NW>(s, word, pl, tile, ntiles, wl, sh_base, wave, lane, [] {});
}

}  // namespace zc

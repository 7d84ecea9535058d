// Block positions of an existing stream: header validation and the exclusive prefix sum of
// the block sizes implied by its width table (Section 3.3 stores one code length per block;
// a block's position is the sum of the sizes before it), kept per segment of 64 blocks, the
// share of one wave.  An indexed stream (Section 3.5.2) brings these positions along: neither
// kernel of this file runs for it; the main kernels judge the headers themselves
// (judge_indexed_streams) and every wave of a consumer checks that its own segment's entries
// agree with its width bytes and with the ends of the index, which together is the whole index.
//
// stream_index_kernel records the offset of every segment inside its scan group, of every
// group inside its index span and the size of every span, and validates header and width
// bytes on the way; index_prep_kernel then turns the span sizes into offsets, compares the
// header's total_bytes with the indexed payload and writes the control block.  No workgroup
// waits for, or counts, another, and neither kernel needs anything cleared beforehand.
#pragma once

#include "zc_common.h"

namespace zc {

struct StreamRef {
  const u8* base;
  u64 bytes;
};

struct ParsedHeader {
  u64 n, nb, total;
  u32 eb_bits, nsum;
  bool ok;
  bool wide;        // an indexed stream that may hold blocks wider than 15 bits
};

// Field checks that need nothing but the 32 header bytes and the buffer size.
__device__ inline ParsedHeader parse_header_words(const u32 (&w)[8], u64 bytes, bool ix) {
  ParsedHeader h;
  h.ok = false;
  h.wide = false;
  h.nb = 0;
  h.n = u64(w[2]) | (u64(w[3]) << 32);
  h.eb_bits = w[4];
  h.nsum = w[5];
  h.total = u64(w[6]) | (u64(w[7]) << 32);
  if (bytes < kHeaderBytes) return h;
  if (w[0] != kMagic || (ix ? (w[1] | 1u) != (kVersionIndexed | 1u) : w[1] != kVersionPlain)) return h;
  h.wide = ix && (w[1] & 1u) != 0;
  if (h.n > ZC_MAX_N) return h;
  // abs_eb must be a finite binary32 >= 2^-96: sign 0, biased exponent in [31, 254]
  const u32 e = h.eb_bits >> 23;
  if (e < 31 || e > 254) return h;
  if (h.nsum < 1) return h;
  h.nb = num_blocks(h.n);
  if (h.total > bytes || h.total < tables_end(h.nb, ix)) return h;
  h.ok = true;
  return h;
}

__device__ inline ParsedHeader parse_header(const StreamRef& s, bool ix) {
  u32 w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (s.bytes >= kHeaderBytes) {
    const u32* src = reinterpret_cast<const u32*>(s.base);
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = src[i];
  }
  return parse_header_words(w, s.bytes, ix);
}

// The same for a main kernel's first instructions: the header (and with load_gate the control
// block) is asked for with vector loads (see opaque_zero), so that it travels together with
// whatever else the kernel can ask for before it knows the header.  The stream must have
// at least kHeaderBytes bytes (the host checks that before it launches anything).
struct HeaderWords {
  uint4 lo, hi;
};

__device__ inline HeaderWords load_header_words(const u8* base, u32 zero) {
  HeaderWords hw;
  hw.lo = *reinterpret_cast<const uint4*>(at_bytes(base, zero));
  hw.hi = *reinterpret_cast<const uint4*>(at_bytes(base, zero + 16u));
  return hw;
}

__device__ inline ParsedHeader parse_header(const HeaderWords& hw, u64 bytes, bool ix) {
  const u32 w[8] = {uniform(hw.lo.x), uniform(hw.lo.y), uniform(hw.lo.z), uniform(hw.lo.w),
                    uniform(hw.hi.x), uniform(hw.hi.y), uniform(hw.hi.z), uniform(hw.hi.w)};
  return parse_header_words(w, bytes, ix);
}

// What a main kernel that reads plain streams finds in the control block: the call's tag and
// the verdict of the validation kernel that ran ahead of it (final before the main kernel starts).
struct Gate {
  u64 tag;
  u32 bits;
};

__device__ inline uint4 load_gate(const Control* ctl, u32 zero) {
  return *reinterpret_cast<const uint4*>(at_bytes(reinterpret_cast<const u8*>(ctl), zero));
}

__device__ inline Gate parse_gate(uint4 raw) {
  Gate g;
  g.tag = u64(uniform(raw.z)) | (u64(uniform(raw.w)) << 32);
  g.bits = uniform(raw.y) == u32(g.tag >> 32) ? uniform(raw.x) : 0u;
  return g;
}

__device__ inline bool gate_failed(const Gate& g) { return (g.bits & kGateBits) != 0; }
__device__ inline bool gate_wide(const Gate& g) { return (g.bits & kStatusWide) != 0; }

struct ScanArgs {
  StreamRef streams[ZC_MAX_K];
  int k;
  int check_match;   // reduce: every stream must have the n and eb_bits of stream 0
  StreamIndex index;
  Control* ctl;
  u64 nonce;         // drawn by the host per call, goes into the call's tag (see launch_tag)
};

constexpr u32 kSpanBadWidth = 1u;   // per-span flags left by stream_index_kernel: a width byte above 31
constexpr u32 kSpanWide = 2u;       //                                               a width byte above 15

// Whether the caller's workspace has room for the index of this stream.
__device__ inline bool stream_fits(const ParsedHeader& h, const StreamIndex& ix) {
  return num_tiles(h.nb) <= ix.tiles_cap && num_scan_groups(h.nb) <= ix.groups_cap && num_spans(h.nb) <= ix.spans_cap;
}

// Payload word offset of segment `seg` of stream `s`: the offset of its index span, plus its
// group's offset in the span, plus its own offset in the group: three independent loads.
// The parts are kept apart until the sum is needed.  Summing them where they are loaded makes
// the compiler wait for two of the loads before it issues the third, which puts two memory
// round trips where one will do.
struct SegmentOffsetParts {
  u32 span, grp, seg;
};

// `zero`: 0, or opaque_zero() to have vector loads whatever the compiler knows about seg.
// An indexed stream has the sum in its own index (`base`: the stream): one load.
__device__ inline SegmentOffsetParts load_segment_offset(const StreamIndex& ix, int s, u64 seg, u32 zero = 0,
                                                         const u8* base = nullptr) {
  SegmentOffsetParts p;
  if (base) {
    p.span = 0;
    p.grp = 0;
    p.seg = *reinterpret_cast<const u32*>(at_bytes(base, kHeaderBytes + 4u * u32(seg) + zero));
    return p;
  }
  p.span = ix.span_off[u64(s) * ix.spans_cap + seg / kSpanSegs + zero];
  p.grp = ix.grp_off[u64(s) * ix.groups_cap + seg / kScanGroupSegs + zero];
  p.seg = ix.seg_off[u64(s) * 4 * ix.tiles_cap + seg + zero];
  return p;
}

// The three loads above are in flight together when this is reached: nothing may use one of
// the parts before all of them have been asked for.
__device__ inline u64 segment_offset(SegmentOffsetParts p) {
  asm volatile("" : "+v"(p.span), "+v"(p.grp), "+v"(p.seg));
  return u64(p.span) + u64(p.grp) + u64(p.seg);
}

__device__ inline u64 segment_offset(const StreamIndex& ix, int s, u64 seg) {
  return segment_offset(load_segment_offset(ix, s, seg));
}

// The entry after a segment's own in the index of an indexed stream: where the segment ends.
__device__ inline u32 load_segment_end(const u8* base, u32 seg, u32 zero = 0) {
  return *reinterpret_cast<const u32*>(at_bytes(base, kHeaderBytes + 4u + 4u * seg + zero));
}

// Payload words of the four blocks whose width bytes are packed in x, and whether any byte
// exceeds 31 (bad) or 15 (wide).  Sum of (1 + w) over the non-zero bytes = byte sum + number of non-zero bytes.
__device__ inline u32 psize_words4(u32 x, bool& bad, bool& wide) {
  bad |= (x & 0xE0E0E0E0u) != 0;
  wide |= (x & 0xF0F0F0F0u) != 0;
  const u32 nonzero = (((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u;   // top bit of every non-zero byte
  return __builtin_amdgcn_sad_u8(x, 0u, u32(__builtin_popcount(nonzero)));
}

// A workgroup covers one index span: kIndexGroups scan groups of 4096 blocks (64 segments)
// of one stream.  Each thread takes 16 blocks of a group (one 16-byte load of the width
// table), four threads make a segment; a scan over the workgroup gives every segment its
// offset inside the group, every group its offset inside the span, and the span its size.
__global__ __launch_bounds__(256) void stream_index_kernel(ScanArgs a) {
  __shared__ u32 sh_wave[kIndexGroups][4];
  __shared__ u32 sh_flags;
  const int s = blockIdx.y;
  const StreamRef st = a.streams[s];
  const ParsedHeader h = parse_header(st, false);
  if (!h.ok || !stream_fits(h, a.index)) return;        // index_prep_kernel reports both
  const u64 ngroups = num_scan_groups(h.nb);
  const u64 group0 = u64(blockIdx.x) * kIndexGroups;
  if (group0 >= ngroups) return;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  if (threadIdx.x == 0) sh_flags = 0;
  const u8* widths = st.base + kHeaderBytes;
  // all loads first: the table is padded to a multiple of 16 bytes, so a 16-byte load that
  // starts below nb stays inside it; bytes of blocks that do not exist are masked off
  uint4 v[kIndexGroups];
#pragma unroll
  for (int i = 0; i < kIndexGroups; ++i) {
    const u64 b0 = (group0 + u64(i)) * kScanGroupBlocks + u64(threadIdx.x) * 16;
    v[i] = make_uint4(0, 0, 0, 0);
    if (b0 < h.nb) v[i] = *reinterpret_cast<const uint4*>(widths + b0);
  }
  u32 sum[kIndexGroups], incl[kIndexGroups];
  bool bad = false, wide = false;
#pragma unroll
  for (int i = 0; i < kIndexGroups; ++i) {
    const u64 b0 = (group0 + u64(i)) * kScanGroupBlocks + u64(threadIdx.x) * 16;
    u32 x[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    if (b0 < h.nb && b0 + 16 > h.nb) {
      const u32 live = u32(h.nb - b0);                 // 1..15 bytes exist
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32 keep = live >= 4u * j + 4 ? 0xFFFFFFFFu : (live > 4u * j ? (1u << (8 * (live - 4u * j))) - 1u : 0u);
        x[j] &= keep;
      }
    }
    sum[i] = psize_words4(x[0], bad, wide) + psize_words4(x[1], bad, wide) + psize_words4(x[2], bad, wide) +
             psize_words4(x[3], bad, wide);
    incl[i] = wave_inclusive_sum(sum[i]);
    if (lane == 63) sh_wave[i][wave] = incl[i];
  }
  __syncthreads();                                       // sh_flags cleared, wave sums visible
  if (bad || wide) atomicOr(&sh_flags, (bad ? kSpanBadWidth : 0u) | (wide ? kSpanWide : 0u));
  u32* grp = a.index.grp_off + u64(s) * a.index.groups_cap;
  u32* seg_off = a.index.seg_off + u64(s) * 4 * a.index.tiles_cap;
  const u64 nsegs = num_segments(h.nb);
  u32 span_before = 0;                                   // payload words of the span's groups so far
#pragma unroll
  for (int i = 0; i < kIndexGroups; ++i) {
    u32 before = 0, all = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32 t = sh_wave[i][j];
      if (j < wave) before += t;
      all += t;
    }
    const u64 seg = (group0 + u64(i)) * kScanGroupSegs + (threadIdx.x >> 2);
    if ((threadIdx.x & 3) == 0 && seg < nsegs) seg_off[seg] = before + incl[i] - sum[i];
    if (threadIdx.x == 0 && group0 + u64(i) < ngroups) grp[group0 + u64(i)] = span_before;
    span_before += all;
  }
  __syncthreads();                                       // every thread's flags are in
  if (threadIdx.x == 0) {
    const u64 slot = u64(s) * a.index.spans_cap + blockIdx.x;
    a.index.span_off[slot] = span_before;                // its size; index_prep_kernel makes it an offset
    a.index.span_flags[slot] = sh_flags;
  }
}

// Second step of the index of plain streams, and the first launch of the call as far as its
// tag goes; one workgroup for all streams.  Each wave takes streams (wave, wave + 4, ...):
// validates the header, turns the span sizes into exclusive offsets in place, collects the
// spans' flags and checks that the header's total_bytes equals tables + payload.  Thread 0 then
// writes the control block: the call's tag, the verdict under that tag, the operands' nsum.
__global__ __launch_bounds__(256) void index_prep_kernel(ScanArgs a) {
  __shared__ u32 sh_status[4], sh_wide[4];
  __shared__ unsigned long long sh_nsum;        // sum of the valid streams' nsum, for the kernel that writes a stream
  if (threadIdx.x == 0) sh_nsum = 0;
  __syncthreads();
  const u64 tag = launch_tag(a.nonce, a.ctl);
  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  u32 status = 0, wide = 0;
  ParsedHeader h0;
  h0.ok = false;
  if (a.check_match) h0 = parse_header(a.streams[0], false);
  for (int s = wave; s < a.k; s += 4) {
    const ParsedHeader h = parse_header(a.streams[s], false);
    if (!h.ok) {
      status |= status_bit(ZC_ERR_FORMAT);
      continue;
    }
    if (!stream_fits(h, a.index)) {
      status |= status_bit(ZC_ERR_ARG);
      continue;
    }
    if (a.check_match && h0.ok && (h0.n != h.n || h0.eb_bits != h.eb_bits)) status |= status_bit(ZC_ERR_MISMATCH);
    if (lane == 0) atomicAdd(&sh_nsum, static_cast<unsigned long long>(h.nsum));
    const u64 nspans = num_spans(h.nb);
    u32* spans = a.index.span_off + u64(s) * a.index.spans_cap;
    const u32* flags = a.index.span_flags + u64(s) * a.index.spans_cap;
    u64 carry = 0;
    u32 seen = 0;
    for (u64 start = 0; start < nspans; start += 64) {
      const u64 i = start + u64(lane);
      const u32 val = i < nspans ? spans[i] : 0u;
      seen |= i < nspans ? flags[i] : 0u;
      const u32 inc = wave_inclusive_sum(val);
      if (i < nspans) spans[i] = u32(carry) + inc - val;
      carry += lane_value(inc, 63);
    }
    if (__any((seen & kSpanBadWidth) != 0)) status |= status_bit(ZC_ERR_FORMAT);
    if (__any((seen & kSpanWide) != 0)) wide = kStatusWide;
    if (tables_end(h.nb, false) + 4 * carry != h.total) status |= status_bit(ZC_ERR_FORMAT);
  }
  if (lane == 0) {
    sh_status[wave] = status;
    sh_wide[wave] = wide;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const u32 bits = sh_status[0] | sh_status[1] | sh_status[2] | sh_status[3] | sh_wide[0] | sh_wide[1] | sh_wide[2] | sh_wide[3];
    a.ctl->status = (tag & 0xffffffff00000000ull) | bits;
    a.ctl->call_tag = tag;
    a.ctl->result = 0;
    a.ctl->nsum = sh_nsum;
  }
}

// ---------------------------------------------------------------------------------------
// Indexed streams need no launch ahead of the main kernel: every workgroup reads the headers
// of all input streams itself and comes to the same verdict, and every wave checks the part
// of the index it uses (the entries of its segment against its width bytes; the wave of the
// first segment that entry 0 is 0, the wave of the last that the closing entry accounts for
// total_bytes), which together is the whole index.
// ---------------------------------------------------------------------------------------

// Verdict on the k <= 64 input streams of a call, from their headers alone.  Lane s of the
// calling wave reads and judges the header of stream s, so that all headers are in flight at
// once; every wave of every workgroup comes to the same verdict.
struct StreamsVerdict {
  ParsedHeader h0;      // header of stream 0 (uniform)
  u32 err;              // status bits: FORMAT, MISMATCH (uniform)
  u64 nsum;             // sum of the nsum fields of the valid streams
  u64 sum_n;            // sum of their n fields
  bool wide;            // some stream may hold blocks wider than 15 bits
};

__device__ inline StreamsVerdict judge_indexed_streams(const StreamRef* streams, int k, bool check_match) {
  const int lane = lane_id();
  const bool mine = lane < k;
  u32 w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  u64 bytes = 0;
  if (mine) {
    bytes = streams[lane].bytes;                       // >= kHeaderBytes: the host has checked
    const uint4* src = reinterpret_cast<const uint4*>(streams[lane].base);
    const uint4 lo = src[0], hi = src[1];
    w[0] = lo.x; w[1] = lo.y; w[2] = lo.z; w[3] = lo.w;
    w[4] = hi.x; w[5] = hi.y; w[6] = hi.z; w[7] = hi.w;
  }
  const ParsedHeader h = parse_header_words(w, bytes, true);
  StreamsVerdict v;
  v.h0.n = u64(lane_value(u32(h.n), 0)) | (u64(lane_value(u32(h.n >> 32), 0)) << 32);
  v.h0.nb = num_blocks(v.h0.n);
  v.h0.total = u64(lane_value(u32(h.total), 0)) | (u64(lane_value(u32(h.total >> 32), 0)) << 32);
  v.h0.eb_bits = lane_value(h.eb_bits, 0);
  v.h0.nsum = lane_value(h.nsum, 0);
  v.h0.ok = lane_value(u32(h.ok), 0) != 0;
  v.h0.wide = lane_value(u32(h.wide), 0) != 0;
  if (!v.h0.ok) v.h0.nb = 0;
  v.err = 0;
  if (__any(mine && !h.ok)) v.err |= status_bit(ZC_ERR_FORMAT);
  if (check_match && v.h0.ok && __any(mine && h.ok && (h.n != v.h0.n || h.eb_bits != v.h0.eb_bits)))
    v.err |= status_bit(ZC_ERR_MISMATCH);
  v.wide = __any(mine && h.ok && h.wide);
  const u32 ns = mine && h.ok ? h.nsum : 0u;
  v.nsum = u64(wave_sum_u32(ns & 0xffffu)) + (u64(wave_sum_u32(ns >> 16)) << 16);
  const u64 nn = mine && h.ok ? h.n : 0;              // <= 2^31
  v.sum_n = u64(wave_sum_u32(u32(nn) & 0xffffu)) + (u64(wave_sum_u32(u32(nn >> 16))) << 16);
  return v;
}

// The checks on the two ends of the index that fall to the wave that holds segment `seg`:
// seg_off and seg_end are its two entries.  (A stream without blocks has a single entry, which
// nobody uses: see index_ends_consistent.)
__device__ inline bool index_ends_ok(const ParsedHeader& h, u32 seg, u32 seg_off, u32 seg_end) {
  const u64 nseg = num_segments(h.nb);
  if (seg == 0 && seg_off != 0) return false;
  if (u64(seg) + 1 == nseg && tables_end(h.nb, true) + 4 * u64(seg_end) != h.total) return false;
  return true;
}

// The same for a kernel with k <= 64 input streams of the same n (headers judged already):
// called by the wave that holds segment `seg`, it does something only for the first and the
// last segment (and for a stream without blocks, whose one entry must be 0): lane s looks at
// stream s.  Uniform result.
__device__ inline bool index_ends_consistent(const StreamRef* streams, int k, const ParsedHeader& h, u32 seg) {
  const u64 nseg = num_segments(h.nb);
  const bool first = seg == 0;
  const bool last = nseg == 0 || u64(seg) + 1 == nseg;
  if (!first && !last) return true;                    // uniform
  const int lane = lane_id();
  bool bad = false;
  if (lane < k) {
    const u8* base = streams[lane].base;
    const u32* index = reinterpret_cast<const u32*>(base + kHeaderBytes);
    if (first && index[0] != 0) bad = true;
    if (last) {
      const u64 total = reinterpret_cast<const u64*>(base)[3];
      if (tables_end(h.nb, true) + 4 * u64(index[nseg]) != total) bad = true;
    }
  }
  return !__any(bad);
}

}  // namespace zc

// Block positions of an existing stream: header validation and the exclusive prefix sum of
// the block sizes implied by its width table (Section 3.3 stores one code length per block;
// a block's position is the sum of the sizes before it), kept per segment of 64 blocks, the
// share of one wave.
//
// stream_index_kernel records the offset of every segment inside its scan group, of every
// group inside its index span and the size of every span, and validates header and width
// bytes on the way; span_scan_kernel then turns the span sizes into offsets and compares the
// header's total_bytes with the indexed payload.  No workgroup waits for, or counts, another.
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
};

// Field checks that need nothing but the 32 header bytes and the buffer size.
__device__ inline ParsedHeader parse_header(const StreamRef& s) {
  ParsedHeader h;
  h.ok = false;
  h.n = h.nb = h.total = 0;
  h.eb_bits = h.nsum = 0;
  if (s.bytes < kHeaderBytes) return h;
  const u32* w = reinterpret_cast<const u32*>(s.base);
  const u32 w0 = w[0], w1 = w[1];
  h.n = u64(w[2]) | (u64(w[3]) << 32);
  h.eb_bits = w[4];
  h.nsum = w[5];
  h.total = u64(w[6]) | (u64(w[7]) << 32);
  if (w0 != kMagic || w1 != (1u | (5u << 16) | (6u << 24))) return h;
  if (h.n > ZC_MAX_N) return h;
  // abs_eb must be a finite binary32 >= 2^-96: sign 0, biased exponent in [31, 254]
  const u32 e = h.eb_bits >> 23;
  if (e < 31 || e > 254) return h;
  if (h.nsum < 1) return h;
  h.nb = num_blocks(h.n);
  if (h.total > s.bytes || h.total < tables_end(h.nb)) return h;
  h.ok = true;
  return h;
}

struct ScanArgs {
  StreamRef streams[ZC_MAX_K];
  int k;
  int check_match;   // reduce: every stream must have the n and eb_bits of stream 0
  StreamIndex index;
  Control* ctl;
};

// Payload word offset of segment `seg` of stream `s`: the offset of its index span, plus its
// group's offset in the span, plus its own offset in the group.  Three independent loads.
__device__ inline u64 segment_offset(const StreamIndex& ix, int s, u64 seg) {
  return u64(ix.span_off[u64(s) * ix.spans_cap + seg / kSpanSegs]) +
         u64(ix.grp_off[u64(s) * ix.groups_cap + seg / kScanGroupSegs]) +
         u64(ix.seg_off[u64(s) * 4 * ix.tiles_cap + seg]);
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
  const int s = blockIdx.y;
  const StreamRef st = a.streams[s];
  const ParsedHeader h = parse_header(st);
  if (!h.ok) {
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
    return;
  }
  const u64 ngroups = num_scan_groups(h.nb);
  const bool fits = num_tiles(h.nb) <= a.index.tiles_cap && ngroups <= a.index.groups_cap &&
                    num_spans(h.nb) <= a.index.spans_cap;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (!fits) atomicOr(&a.ctl->status, status_bit(ZC_ERR_ARG));
    if (a.check_match && s > 0) {
      const ParsedHeader h0 = parse_header(a.streams[0]);
      if (h0.ok && (h0.n != h.n || h0.eb_bits != h.eb_bits)) atomicOr(&a.ctl->status, status_bit(ZC_ERR_MISMATCH));
    }
  }
  if (!fits) return;
  const u64 group0 = u64(blockIdx.x) * kIndexGroups;
  if (group0 >= ngroups) return;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
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
  if (bad) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
  if (wide) atomicOr(&a.ctl->flags, kFlagWide);
  __syncthreads();
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
  if (threadIdx.x == 0) a.index.span_off[u64(s) * a.index.spans_cap + blockIdx.x] = span_before;   // its size; span_scan_kernel makes it an offset
}

// Second step of the index: one workgroup per stream turns the span sizes into exclusive
// offsets, in place, and checks that the header's total_bytes equals tables + payload.
__global__ __launch_bounds__(256) void span_scan_kernel(ScanArgs a) {
  __shared__ u32 sh_scan[4];
  __shared__ u64 sh_carry;
  const int s = blockIdx.x;
  const ParsedHeader h = parse_header(a.streams[s]);
  if (!h.ok) return;
  const u64 nspans = num_spans(h.nb);
  if (nspans > a.index.spans_cap) return;               // already flagged by stream_index_kernel
  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  u32* spans = a.index.span_off + u64(s) * a.index.spans_cap;
  if (threadIdx.x == 0) sh_carry = 0;
  __syncthreads();
  for (u64 start = 0; start < nspans; start += 256) {
    const u64 i = start + threadIdx.x;
    const u32 val = i < nspans ? spans[i] : 0u;
    const u32 inc = wave_inclusive_sum(val);
    if (lane == 63) sh_scan[wave] = inc;
    __syncthreads();
    u32 before = 0, all = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32 t = sh_scan[j];
      if (j < wave) before += t;
      all += t;
    }
    const u64 carry = sh_carry;
    if (i < nspans) spans[i] = u32(carry) + before + inc - val;
    __syncthreads();
    if (threadIdx.x == 0) sh_carry = carry + all;
    __syncthreads();
  }
  if (threadIdx.x == 0 && tables_end(h.nb) + 4 * sh_carry != h.total) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
}

}  // namespace zc

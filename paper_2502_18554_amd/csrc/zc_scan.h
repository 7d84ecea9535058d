// Block positions of an existing stream: header validation and the exclusive prefix sum of
// the block sizes implied by its width table (Section 3.3 stores one code length per block;
// a block's position is the sum of the sizes before it), kept per segment of 64 blocks, the
// share of one wave.
//
// stream_index_kernel records the payload size of every segment and the exclusive offset of
// every scan group of 64 segments, and validates header and width bytes on the way.
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

// Payload word offset of segment `seg` of stream `s`: the offset of its scan group plus the
// sizes of the segments before it inside the group.  Called by all 64 lanes of a wave.
__device__ inline u64 segment_offset(const StreamIndex& ix, int s, u64 seg) {
  const u64 g = seg / kScanGroupSegs;
  const u32 r = u32(seg % kScanGroupSegs);
  const u32* sums = ix.seg_sum + u64(s) * 4 * ix.tiles_cap + g * kScanGroupSegs;
  const u32 mine = u32(lane_id()) < r ? sums[lane_id()] : 0u;
  return u64(ix.grp_off[u64(s) * ix.groups_cap + g]) + wave_sum_u32(mine);
}

// One workgroup per scan group of 4096 blocks (64 segments) and stream.  Each thread sums
// the payload sizes of 16 blocks (one 16-byte load of the width table) and checks the width
// bytes; four threads make a segment.  The workgroup that finishes last for a stream turns
// the group sums into exclusive offsets and checks header total_bytes = tables + payload.
__global__ __launch_bounds__(256) void stream_index_kernel(ScanArgs a) {
  __shared__ u32 sh_wave[4];
  __shared__ u32 sh_last;
  __shared__ u64 sh_carry;
  const int s = blockIdx.y;
  const StreamRef st = a.streams[s];
  const ParsedHeader h = parse_header(st);
  if (!h.ok) {
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
    return;
  }
  const u64 ngroups = num_scan_groups(h.nb);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (num_tiles(h.nb) > a.index.tiles_cap || ngroups > a.index.groups_cap)
      atomicOr(&a.ctl->status, status_bit(ZC_ERR_ARG));
    if (a.check_match && s > 0) {
      const ParsedHeader h0 = parse_header(a.streams[0]);
      if (h0.ok && (h0.n != h.n || h0.eb_bits != h.eb_bits)) atomicOr(&a.ctl->status, status_bit(ZC_ERR_MISMATCH));
    }
  }
  if (num_tiles(h.nb) > a.index.tiles_cap || ngroups > a.index.groups_cap) return;
  const u64 group = blockIdx.x;
  if (group >= ngroups) return;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  const u8* widths = st.base + kHeaderBytes;
  const u64 b0 = group * kScanGroupBlocks + u64(threadIdx.x) * 16;
  u32 bytes[4] = {0, 0, 0, 0};
  if (b0 + 16 <= h.nb) {
    const uint4 v = *reinterpret_cast<const uint4*>(widths + b0);
    bytes[0] = v.x; bytes[1] = v.y; bytes[2] = v.z; bytes[3] = v.w;
  } else {
    for (int i = 0; i < 16; ++i)
      if (b0 + i < h.nb) bytes[i >> 2] |= u32(widths[b0 + i]) << (8 * (i & 3));
  }
  u32 sum = 0;
  bool bad = false;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const u32 w = (bytes[i >> 2] >> (8 * (i & 3))) & 0xffu;
    bad |= w > 31;
    sum += psize_words(w > 31 ? 0 : w);
  }
  if (bad) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
  // four threads = one segment of 64 blocks
  u32 seg_total = sum + dpp_mov<kDppQuadSwap1>(sum);
  seg_total += dpp_mov<kDppQuadSwap2>(seg_total);
  const u64 seg = group * kScanGroupSegs + (threadIdx.x >> 2);
  if ((threadIdx.x & 3) == 0 && seg < num_segments(h.nb))
    a.index.seg_sum[u64(s) * 4 * a.index.tiles_cap + seg] = seg_total;
  const u32 wave_total = wave_sum_u32(sum);
  if (lane == 0) sh_wave[wave] = wave_total;
  __syncthreads();
  u32* grp = a.index.grp_off + u64(s) * a.index.groups_cap;
  if (threadIdx.x == 0) {
    desc32_store(grp + group, sh_wave[0] + sh_wave[1] + sh_wave[2] + sh_wave[3]);
    __threadfence();
    const u32 finished = atomicAdd(&a.index.done[s], 1u);
    sh_last = (finished + 1 == u32(ngroups));
  }
  __syncthreads();
  if (!sh_last) return;

  // ---- last workgroup of this stream: exclusive scan of the group sums, in place ----
  __threadfence();
  if (threadIdx.x == 0) sh_carry = 0;
  __syncthreads();
  for (u64 start = 0; start < ngroups; start += 256) {
    const u64 i = start + threadIdx.x;
    const u32 v = i < ngroups ? desc32_load(grp + i) : 0u;
    const u32 incl = wave_inclusive_sum(v);
    if (lane == 63) sh_wave[wave] = incl;
    __syncthreads();
    u32 before = 0, all = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32 t = sh_wave[j];
      if (j < wave) before += t;
      all += t;
    }
    const u64 carry = sh_carry;
    if (i < ngroups) grp[i] = u32(carry) + before + incl - v;
    __syncthreads();
    if (threadIdx.x == 0) sh_carry = carry + all;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const u64 payload_bytes = 4 * sh_carry;
    if (tables_end(h.nb) + payload_bytes != h.total) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
  }
}

}  // namespace zc

// Block positions of an existing stream: header validation and the exclusive prefix sum of
// the block sizes implied by its width table (Section 3.3 stores one code length per block;
// a block's position is the sum of the sizes before it), kept per segment of 64 blocks, the
// share of one wave.
//
// segment_sizes_kernel : one wave per segment sums the payload words of its 64 blocks and
//                        checks every width byte; the first thread of each stream's first
//                        workgroup validates the header (and, for a reduce, that the stream
//                        matches stream 0).
// segment_scan_kernel  : one workgroup per stream turns the segment sums into exclusive
//                        offsets and checks that header total_bytes = tables + payload.
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
  u64 tiles_cap;     // tiles the workspace has room for; row stride of seg_off is 4 * tiles_cap
  u32* seg_off;      // [k][4 * tiles_cap]
  Control* ctl;
};

__global__ __launch_bounds__(256) void segment_sizes_kernel(ScanArgs a) {
  const int s = blockIdx.y;
  const StreamRef st = a.streams[s];
  const ParsedHeader h = parse_header(st);
  if (!h.ok) {
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (num_tiles(h.nb) > a.tiles_cap) atomicOr(&a.ctl->status, status_bit(ZC_ERR_ARG));
    if (a.check_match && s > 0) {
      const ParsedHeader h0 = parse_header(a.streams[0]);
      if (h0.ok && (h0.n != h.n || h0.eb_bits != h.eb_bits)) atomicOr(&a.ctl->status, status_bit(ZC_ERR_MISMATCH));
    }
  }
  const u64 nseg = num_segments(h.nb);
  const u64 seg = u64(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (seg >= nseg || seg >= 4 * a.tiles_cap) return;
  const int lane = lane_id();
  const u64 b = seg * kWaveBlocks + u64(lane);
  u32 w = b < h.nb ? u32(st.base[kHeaderBytes + b]) : 0u;
  if (w > 31) {
    atomicOr(&a.ctl->status, status_bit(ZC_ERR_FORMAT));
    w = 0;
  }
  const u32 sum = wave_sum_u32(psize_words(w));
  if (lane == 0) a.seg_off[u64(s) * 4 * a.tiles_cap + seg] = sum;
}

constexpr int kScanPerThread = 16;

__global__ __launch_bounds__(1024) void segment_scan_kernel(ScanArgs a) {
  __shared__ u32 sh_wave[16];
  __shared__ u64 sh_carry;
  const int s = blockIdx.x;
  const StreamRef st = a.streams[s];
  const ParsedHeader h = parse_header(st);
  if (!h.ok) return;                      // already flagged by segment_sizes_kernel
  u64 nseg = num_segments(h.nb);
  if (nseg > 4 * a.tiles_cap) return;     // already flagged: workspace too small
  u32* row = a.seg_off + u64(s) * 4 * a.tiles_cap;
  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  if (threadIdx.x == 0) sh_carry = 0;
  __syncthreads();
  for (u64 start = 0; start < nseg; start += 1024 * kScanPerThread) {
    const u64 i0 = start + u64(threadIdx.x) * kScanPerThread;
    u32 v[kScanPerThread];
    u32 mine = 0;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
      v[j] = i0 + j < nseg ? row[i0 + j] : 0u;
      mine += v[j];
    }
    const u32 incl = wave_inclusive_sum(mine);
    if (lane == 63) sh_wave[wave] = incl;
    __syncthreads();
    u32 before = 0, all = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const u32 t = sh_wave[j];
      if (j < wave) before += t;
      all += t;
    }
    const u64 carry = sh_carry;
    u32 run = u32(carry) + before + incl - mine;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
      if (i0 + j < nseg) row[i0 + j] = run;
      run += v[j];
    }
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

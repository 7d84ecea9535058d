// fZ-light decompression kernel: the inverse of the stages of Section 3.3.
//
// Same geometry as compression: a tile is 256 blocks, one lane owns one block.  A wave's
// payload offset comes from the stream index (zc_scan.h); inside the wave a scan of
// the block sizes places each lane.  The lane reads its sign and plane words, rebuilds the
// deltas, runs the Lorenzo chain from the block's outlier, dequantises, and the floats are
// transposed through LDS so that they leave as 16-byte coalesced stores.
#pragma once

#include "zc_common.h"
#include "zc_planes.h"
#include "zc_scan.h"

namespace zc {

struct DecompressArgs {
  StreamRef in;
  float* out;
  u64 out_cap_elems;
  StreamIndex index;
  Control* ctl;
};

__global__ __launch_bounds__(kTileThreads) void decompress_kernel(DecompressArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWaveLds];

  if (validation_failed(a.ctl)) return;
  const ParsedHeader h = parse_header(a.in);
  if (!h.ok) return;
  if (blockIdx.x == 0 && threadIdx.x == 0) a.ctl->result = h.n;
  if (h.n > a.out_cap_elems) {
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&a.ctl->status, status_bit(ZC_ERR_CAPACITY));
    return;
  }
  const u32 tile = blockIdx.x;
  if (u64(tile) >= num_tiles(h.nb) || u64(tile) >= a.index.tiles_cap) return;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  u32* wl = lds + wave * kWaveLds;
  const u64 wblock0 = u64(tile) * kTileBlocks + u64(wave) * kWaveBlocks;
  const u64 b = wblock0 + u64(lane);
  const bool active = b < h.nb;

  const u8* widths = a.in.base + kHeaderBytes;
  const i32* outliers = reinterpret_cast<const i32*>(a.in.base + kHeaderBytes + pad16(h.nb));
  const u32* payload = reinterpret_cast<const u32*>(a.in.base + tables_end(h.nb));
  const u64 payload_words = (h.total - tables_end(h.nb)) / 4;

  u32 w = active ? u32(widths[b]) : 0u;
  const u32 words = psize_words(w);
  const u32 incl = wave_inclusive_sum(words);
  const u64 seg = u64(tile) * kTileWaves + u64(wave);
  u64 off = 0;
  if (seg < num_segments(h.nb)) off = segment_offset(a.index, 0, seg) + (incl - words);
  if (off + words > payload_words) w = 0;        // cannot happen once the scan has validated the stream
  const u32 wmax = wave_max_u32(w);

  // ---- planes -> sign-magnitude deltas -> codes ----
  u32 c[32];
  load_block_planes(c, w, wmax, payload + off);
  const double step = double(__uint_as_float(h.eb_bits)) * 63.0 / 32.0;
  u32 cur = active ? u32(outliers[b]) : 0u;
  float x[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const u32 sm = rotr32(c[j], j);
    const u32 m = u32(i32(sm) >> 31);             // all ones when the delta is negative
    cur += ((sm & 0x7fffffffu) ^ m) - m;
    x[j] = float(__dmul_rn(double(i32(cur)), step));
  }

  // ---- transpose through LDS, 16-byte coalesced stores ----
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    float4 v = make_float4(x[4 * t], x[4 * t + 1], x[4 * t + 2], x[4 * t + 3]);
    *reinterpret_cast<float4*>(wl + lane * kRow + 4 * t) = v;
  }
  __syncthreads();
  const u64 v0 = wblock0 * kBlockValues;
  const bool full = v0 + u64(kWaveBlocks) * kBlockValues <= h.n;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const u64 idx = v0 + u64(256 * i + 4 * lane);
    const float4 v = *reinterpret_cast<const float4*>(wl + (8 * i + (lane >> 3)) * kRow + 4 * (lane & 7));
    if (full) {
      *reinterpret_cast<float4*>(a.out + idx) = v;
    } else {
      if (idx + 0 < h.n) a.out[idx + 0] = v.x;
      if (idx + 1 < h.n) a.out[idx + 1] = v.y;
      if (idx + 2 < h.n) a.out[idx + 2] = v.z;
      if (idx + 3 < h.n) a.out[idx + 3] = v.w;
    }
  }
}

}  // namespace zc

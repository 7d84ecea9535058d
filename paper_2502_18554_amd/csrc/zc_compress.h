// fZ-light compression kernel (Section 3.3): quantise, per-block Lorenzo delta, code length,
// sign + plane packing, single-pass placement of the variable-size blocks.
//
// Work split.  A tile is 256 blocks (8192 values, 32 KiB of input) handled by a workgroup of
// 4 waves; tiles are handed out by atomic tickets, so that look-back
// only ever waits on tiles that are already running.  Each wave loads 2048 consecutive values with 16-byte
// loads, quantises them where they land, and transposes the integer codes through LDS so
// that one lane owns one block.  Delta, width and plane packing are then in-lane; the
// packed words go back to LDS at the wave's running offset and leave as coalesced stores
// once the tile's base offset is known from the look-back scan.
#pragma once

#include "zc_common.h"
#include "zc_planes.h"

namespace zc {

struct CompressArgs {
  const float* in;
  u64 n, nb;
  double inv;        // 1 / step, divided on the host
  double step;       // abs_eb * 63 / 32
  double eb;         // abs_eb as binary64
  float screen;      // 2^17 * abs_eb: |x| at or below it needs no per-value checks
  u32 eb_bits;
  u8* out;           // stream base
  u64 out_cap;       // bytes
  Control* ctl;
  u64* desc;
};

// Round-to-nearest-even of r for |r| < 2^31 as the low word of r + 1.5 * 2^52.
__device__ inline i32 rint_small(double r) {
  double t = __dadd_rn(r, 6755399441055744.0);
  return i32(__double2loint(t));
}

// Codes of one value that failed the cheap screen: the defining arithmetic, with its checks.
__device__ inline i32 quantize_checked(float x, const CompressArgs& a, u32& err) {
  if (!(__builtin_fabsf(x) <= 3.4028234663852886e38f)) {   // NaN or Inf
    err |= status_bit(ZC_ERR_NONFINITE);
    return 0;
  }
  double t = __builtin_rint(__dmul_rn(double(x), a.inv));
  if (__builtin_fabs(t) > double(kMaxCode)) {
    err |= status_bit(ZC_ERR_RANGE);
    return 0;
  }
  i32 q = i32(t);
  float xr = float(__dmul_rn(double(q), a.step));
  if (!(__builtin_fabs(double(x) - double(xr)) <= a.eb)) err |= status_bit(ZC_ERR_BOUND);
  return q;
}

// Inside |x| <= 2^17 eb the code is below 2^17 and the bound cannot fail (the guard of 1/64
// of eb exceeds the binary32 rounding of the reconstruction there), so the checks are skipped.
__device__ inline bool needs_checks(float x, const CompressArgs& a) { return !(__builtin_fabsf(x) <= a.screen); }

__device__ inline i32 quantize_fast(float x, const CompressArgs& a) {
  return rint_small(__dmul_rn(double(x), a.inv));
}

__device__ inline i32 quantize_value(float x, const CompressArgs& a, u32& err) {
  if (__builtin_expect(needs_checks(x, a), 0)) return quantize_checked(x, a, err);
  return quantize_fast(x, a);
}

__global__ __launch_bounds__(kTileThreads) void compress_kernel(CompressArgs a) {
  __shared__ __attribute__((aligned(16))) u32 lds[kTileWaves * kWaveLds];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kTileWaves];
  __shared__ u64 sh_base;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  const u32 ntiles = u32(num_tiles(a.nb));
  if (threadIdx.x == 0) sh_tile = take_tile(a.ctl, ntiles, xcc_id());
  __syncthreads();
  const u32 tile = uniform(sh_tile);
  if (tile == kNoTile) return;

  u32* wl = lds + wave * kWaveLds;
  const u64 wblock0 = u64(tile) * kTileBlocks + u64(wave) * kWaveBlocks;
  const u64 v0 = wblock0 * kBlockValues;
  const bool full = v0 + u64(kWaveBlocks) * kBlockValues <= a.n;
  u32 err = 0;

  // ---- load 16 B per lane (all eight loads in flight before the first use) ----
  float4 x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const u64 idx = v0 + u64(256 * i + 4 * lane);
    if (full) {
      x[i] = *reinterpret_cast<const float4*>(a.in + idx);
    } else {
      x[i].x = idx + 0 < a.n ? a.in[idx + 0] : 0.0f;
      x[i].y = idx + 1 < a.n ? a.in[idx + 1] : 0.0f;
      x[i].z = idx + 2 < a.n ? a.in[idx + 2] : 0.0f;
      x[i].w = idx + 3 < a.n ? a.in[idx + 3] : 0.0f;
    }
  }

  // ---- quantise where the values landed, park the codes in LDS row = block ----
  bool flagged = false;
#pragma unroll
  for (int i = 0; i < 8; ++i)
    flagged |= needs_checks(x[i].x, a) | needs_checks(x[i].y, a) | needs_checks(x[i].z, a) | needs_checks(x[i].w, a);
  if (__builtin_expect(__any(flagged), 0)) {
    // some value of this wave lies outside the screened domain: the checked arithmetic for all
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int4 q;
      q.x = quantize_value(x[i].x, a, err);
      q.y = quantize_value(x[i].y, a, err);
      q.z = quantize_value(x[i].z, a, err);
      q.w = quantize_value(x[i].w, a, err);
      *reinterpret_cast<int4*>(wl + (8 * i + (lane >> 3)) * kRow + 4 * (lane & 7)) = q;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int4 q;
      q.x = quantize_fast(x[i].x, a);
      q.y = quantize_fast(x[i].y, a);
      q.z = quantize_fast(x[i].z, a);
      q.w = quantize_fast(x[i].w, a);
      *reinterpret_cast<int4*>(wl + (8 * i + (lane >> 3)) * kRow + 4 * (lane & 7)) = q;
    }
  }
  __syncthreads();

  // ---- one lane = one block: fetch its 32 codes ----
  i32 q[32];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    int4 r = *reinterpret_cast<const int4*>(wl + lane * kRow + 4 * t);
    q[4 * t + 0] = r.x; q[4 * t + 1] = r.y; q[4 * t + 2] = r.z; q[4 * t + 3] = r.w;
  }
  const u64 b = wblock0 + u64(lane);
  const bool active = b < a.nb;
  if (!full) {
    // the last block repeats its last code up to 32 values
    u64 cnt = active ? a.n - b * kBlockValues : 0;
#pragma unroll
    for (int j = 1; j < 32; ++j) q[j] = u64(j) < cnt ? q[j] : q[j - 1];
  }

  // ---- Lorenzo delta, sign-magnitude, rotate by j, width ----
  u32 c[32];
  u32 any = 0;
  c[0] = 0;
#pragma unroll
  for (int j = 1; j < 32; ++j) {
    i32 d = q[j] - q[j - 1];
    u32 neg = u32(d) & 0x80000000u;
    u32 mag = u32(d < 0 ? -d : d);
    any |= mag;
    c[j] = rotl32(mag | neg, j);
  }
  const u32 w = (active && any) ? 32u - u32(__builtin_clz(any)) : 0u;
  const u32 words = psize_words(w);

  // ---- place the block inside the wave and the wave inside the tile ----
  const u32 incl = wave_inclusive_sum(words);
  const u32 wave_total = uniform(u32(__shfl(int(incl), 63)));
  const u32 off_in_wave = incl - words;
  const u32 wmax = wave_max_u32(w);
  if (lane == 0) sh_wave_total[wave] = wave_total;

  if (active && a.out_cap >= tables_end(a.nb)) {
    a.out[kHeaderBytes + b] = u8(w);
    reinterpret_cast<i32*>(a.out + kHeaderBytes + pad16(a.nb))[b] = q[0];
  }
  __syncthreads();   // all q reads of this wave's LDS rows are done; wave totals visible

  u32 wave_off = 0, tile_total = 0;
#pragma unroll
  for (int i = 0; i < kTileWaves; ++i) {
    u32 t = sh_wave_total[i];
    if (i < wave) wave_off += t;
    tile_total += t;
  }
  // publish this tile's size before the packing phase so successors never wait for it
  if (threadIdx.x == 0) desc_store(a.desc + tile, (tile == 0 ? kDescPrefix : kDescAggregate) | u64(tile_total));

  // ---- pack sign + planes into LDS at the wave's running offset ----
  store_block_planes(c, w, wmax, wl + off_in_wave);

  // ---- look back for the tile's base offset ----
  if (wave == 0) {
    const u64 base = tile ? lookback_exclusive(a.desc, tile, &a.ctl->status) : 0;
    if (lane == 0) {
      if (tile) desc_store(a.desc + tile, kDescPrefix | (base + tile_total));
      sh_base = base;
    }
  }
  if (err) atomicOr(&a.ctl->status, err);
  __syncthreads();

  // ---- copy the wave's packed words out, coalesced ----
  const u64 base = sh_base;
  const u64 tend = tables_end(a.nb);
  const u64 cap_words = a.out_cap > tend ? (a.out_cap - tend) / 4 : 0;
  u32* payload = reinterpret_cast<u32*>(a.out + tend);
  const u64 dst0 = base + wave_off;
  for (u32 i = u32(lane); i < wave_total; i += 64) {
    if (dst0 + i < cap_words) payload[dst0 + i] = wl[i];
  }

  if (tile == ntiles - 1 && threadIdx.x == 0) {
    const u64 total = tend + 4 * (base + tile_total);
    a.ctl->result = total;
    if (total > a.out_cap) {
      atomicOr(&a.ctl->status, status_bit(ZC_ERR_CAPACITY));
    }
    if (a.out_cap >= kHeaderBytes) reinterpret_cast<u64*>(a.out)[3] = total;
  }
}

// Clears the control block and the tile descriptors, and writes the fixed header fields and
// the zero padding of the two tables.  Runs before compress_kernel / reduce_kernel.
struct InitArgs {
  Control* ctl;
  u32* done;        // per-stream counters of the stream index
  u64* desc;
  u32 ntiles;
  u8* out;          // may be null (decompress has no output stream)
  u64 out_cap;
  u64 n, nb;
  u32 eb_bits, nsum;
};

__global__ void init_kernel(InitArgs a) {
  const u64 gid = u64(blockIdx.x) * blockDim.x + threadIdx.x;
  const u64 stride = u64(gridDim.x) * blockDim.x;
  for (u64 i = gid; i < a.ntiles; i += stride) a.desc[i] = 0;
  if (gid < ZC_MAX_K) a.done[gid] = 0;
  if (gid == 0) {
    for (int i = 0; i < kTicketShards; ++i) a.ctl->ticket[i] = 0;
    a.ctl->status = 0;
    a.ctl->result = 0;
    if (a.out) {
      const u64 tend = tables_end(a.nb);
      if (a.out_cap >= tend) {
        u32* h = reinterpret_cast<u32*>(a.out);
        h[0] = kMagic;
        h[1] = 1u | (5u << 16) | (6u << 24);
        h[2] = u32(a.n);
        h[3] = u32(a.n >> 32);
        h[4] = a.eb_bits;
        h[5] = a.nsum;
        h[6] = u32(tend);           // total_bytes of an empty payload; the last tile overwrites it
        h[7] = u32(tend >> 32);
        for (u64 i = a.nb; i < pad16(a.nb); ++i) a.out[kHeaderBytes + i] = 0;
        u8* ot = a.out + kHeaderBytes + pad16(a.nb);
        for (u64 i = 4 * a.nb; i < pad16(4 * a.nb); ++i) ot[i] = 0;
      } else {
        a.ctl->status = status_bit(ZC_ERR_CAPACITY);
      }
      if (a.nb == 0) a.ctl->result = tend;
    }
  }
}

}  // namespace zc

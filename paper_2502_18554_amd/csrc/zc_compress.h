// fZ-light compression kernel (Section 3.3): quantise, per-block Lorenzo delta, code length,
// sign + plane packing, single-pass placement of the variable-size blocks.
//
// Work split.  A tile is 512 blocks (16384 values, 64 KiB of input) handled by a workgroup of
// 8 waves.  Each wave loads 2048 consecutive values with 16-byte loads,
// quantises them where they land, and transposes the integer codes through LDS so that one
// lane owns one block.  Delta, width and the bit-matrix transpose that yields the plane
// words are then in-lane; the packed words wait in registers for the tile's base offset
// from the look-back scan and leave through LDS as coalesced stores.
#pragma once

#include "zc_bitmatrix.h"
#include "zc_common.h"
#include "zc_place.h"

namespace zc {

// A scan tile of the compression kernel: the blocks of one workgroup, one descriptor of the
// look-back scan.  Every tile pays the latency of that scan once, so compression uses tiles
// twice the size of the other kernels' tiles (512 blocks, 64 KiB of input); 1024 blocks
// measured slower, because a compute unit then holds a single workgroup.
constexpr int kPackWaves = 8;
constexpr int kPackThreads = kPackWaves * 64;
constexpr int kPackBlocks = kPackWaves * kWaveBlocks;
constexpr int kPackValues = kPackBlocks * kBlockValues;
__host__ __device__ inline u64 num_pack_tiles(u64 nb) { return (nb + kPackBlocks - 1) / kPackBlocks; }

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

__device__ inline int4 quantize4(const float4& x, const CompressArgs& a, bool checked, u32& err) {
  int4 q;
  if (__builtin_expect(checked, 0)) {
    q.x = quantize_value(x.x, a, err);
    q.y = quantize_value(x.y, a, err);
    q.z = quantize_value(x.z, a, err);
    q.w = quantize_value(x.w, a, err);
  } else {
    q.x = quantize_fast(x.x, a);
    q.y = quantize_fast(x.y, a);
    q.z = quantize_fast(x.z, a);
    q.w = quantize_fast(x.w, a);
  }
  return q;
}

// Raw input of one wave's share of a tile: 8 x 16 bytes per lane, every load in flight at once.
template <bool FULL>
__device__ inline void load_raw(const CompressArgs& a, u64 wblock0, int lane, float4 (&x)[8]) {
  const u64 v0 = wblock0 * kBlockValues;
  if (FULL) {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = *reinterpret_cast<const float4*>(a.in + v0 + u64(256 * i + 4 * lane));
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u64 idx = v0 + u64(256 * i + 4 * lane);
      x[i].x = idx + 0 < a.n ? a.in[idx + 0] : 0.0f;
      x[i].y = idx + 1 < a.n ? a.in[idx + 1] : 0.0f;
      x[i].z = idx + 2 < a.n ? a.in[idx + 2] : 0.0f;
      x[i].w = idx + 3 < a.n ? a.in[idx + 3] : 0.0f;
    }
  }
}

// Quantise the wave's values where they landed, transpose the codes through LDS so that one
// lane owns one block, and take the Lorenzo delta.  Leaves in d[j] delta j of the lane's
// block (d[0] = 0) and returns the block's first code (the outlier).
template <bool FULL>
__device__ inline i32 block_deltas(const CompressArgs& a, const float4 (&x)[8], u64 wblock0, int lane, u32* wl,
                                   i32 (&d)[32], u32& err) {
  // Some value of this wave outside the screened domain: the checked arithmetic for all of it.
  bool flagged = false;
#pragma unroll
  for (int i = 0; i < 8; ++i)
    flagged |= needs_checks(x[i].x, a) | needs_checks(x[i].y, a) | needs_checks(x[i].z, a) | needs_checks(x[i].w, a);
  const bool checked = __any(flagged);

  // Loads 0..3 hold blocks 0..31 (lanes 0..31), loads 4..7 blocks 32..63.
  i32 q[32];
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<int4*>(wl + (8 * i + (lane >> 3)) * kStageRow + 4 * (lane & 7)) =
          quantize4(x[4 * half + i], a, checked, err);
    wave_lds_sync();
    if ((lane >> 5) == half) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int4 r = *reinterpret_cast<const int4*>(wl + (lane & 31) * kStageRow + 4 * t);
        q[4 * t + 0] = r.x; q[4 * t + 1] = r.y; q[4 * t + 2] = r.z; q[4 * t + 3] = r.w;
      }
    }
    wave_lds_sync();
  }
  const u64 b = wblock0 + u64(lane);
  if (!FULL) {
    // the last block repeats its last code up to 32 values
    const u64 cnt = b < a.nb ? a.n - b * kBlockValues : 0;
#pragma unroll
    for (int j = 1; j < 32; ++j) q[j] = u64(j) < cnt ? q[j] : q[j - 1];
  }
  d[0] = 0;
#pragma unroll
  for (int j = 1; j < 32; ++j) d[j] = q[j] - q[j - 1];
  return q[0];
}

// One workgroup per tile.  FULL = the launch covers tiles whose 8192 values all exist (pure
// 16-byte loads, no tail), handed out by the per-XCD tickets over [first_tile, end_tile); the
// ragged last tile of an input runs as a second launch of one workgroup with FULL = false.
template <bool FULL>
__global__ __launch_bounds__(kPackThreads, 16 / kPackWaves) void compress_kernel(CompressArgs a, u32 first_tile, u32 end_tile) {
  __shared__ __attribute__((aligned(16))) u32 lds[kPackWaves * kWaveStage];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kPackWaves];
  __shared__ u32 sh_wave_wmax[kPackWaves];
  __shared__ u64 sh_base;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  const u32 ntiles = u32(num_pack_tiles(a.nb));
  u32* const wl = lds + wave * kWaveStage;
  const bool tables_fit = a.out_cap >= tables_end(a.nb);
  u32 err = 0;

  u32 tile = first_tile;
  if (FULL) {
    if (threadIdx.x == 0) sh_tile = take_tile(a.ctl, end_tile, xcc_id());
    __syncthreads();
    tile = uniform(sh_tile);
    if (tile == kNoTile) return;
  }
  {
    const u64 wblock0 = u64(tile) * kPackBlocks + u64(wave) * kWaveBlocks;
    const u64 b = wblock0 + u64(lane);
    const bool active = b < a.nb;
    float4 x[8];
    load_raw<FULL>(a, wblock0, lane, x);

    i32 d[32];
    const i32 outlier = block_deltas<FULL>(a, x, wblock0, lane, wl, d, err);
    u32 any = 0;
#pragma unroll
    for (int j = 1; j < 32; ++j) any |= u32(d[j] < 0 ? -d[j] : d[j]);
    Placement pl;
    pl.w = (active && any) ? 32u - u32(__builtin_clz(any)) : 0u;
    pl.wmax = wave_max_u32(pl.w);
    if (active && tables_fit) {
      a.out[kHeaderBytes + b] = u8(pl.w);
      reinterpret_cast<i32*>(a.out + kHeaderBytes + pad16(a.nb))[b] = outlier;
    }

    // ---- place the block inside the wave and the wave inside the tile ----
    const u32 words = psize_words(pl.w);
    const u32 incl = wave_inclusive_sum(words);
    pl.wave_total = lane_value(incl, 63);
    pl.half0_total = lane_value(incl, 31);
    pl.off_in_wave = incl - words;
    if (lane == 0) {
      sh_wave_total[wave] = pl.wave_total;
      sh_wave_wmax[wave] = pl.wmax;
    }
    __syncthreads();   // wave totals visible; also fences the previous tile's use of sh_base
    pl.wave_off = 0;
    pl.tile_total = 0;
    u32 tile_wmax = 0;
#pragma unroll
    for (int i = 0; i < kPackWaves; ++i) {
      const u32 t = sh_wave_total[i];
      if (i < wave) pl.wave_off += t;
      pl.tile_total += t;
      tile_wmax = tile_wmax > sh_wave_wmax[i] ? tile_wmax : sh_wave_wmax[i];
    }
    tile_wmax = uniform(tile_wmax);
    // publish the tile's size as early as possible: the tiles after this one wait for it
    const PayloadSink sink{a.out, a.out_cap, a.nb, a.ctl, a.desc};
    if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total);

    // ---- deltas -> sign + plane words in registers, then the back half ----
    // (the empty asm keeps the compiler from hoisting the sign-magnitude split of all 32
    //  deltas above the branches, where it would hold twice as many registers)
    if (tile_wmax <= 15) {
      u32 pw[16];          // pw[0] = sign, pw[1 + p] = plane p
      if (pl.wmax <= 7) {
        u32 r[8];
#pragma unroll
        for (int j = 0; j < 32; ++j) asm volatile("" : "+v"(d[j]));
        planes_from_deltas8(d, r);
        pw[0] = r[7];
#pragma unroll
        for (int p = 0; p < 7; ++p) pw[1 + p] = r[p];
#pragma unroll
        for (int p = 8; p < 16; ++p) pw[p] = 0;
      } else {
        u32 r[16];
#pragma unroll
        for (int j = 0; j < 32; ++j) asm volatile("" : "+v"(d[j]));
        planes_from_deltas16(d, r);
        pw[0] = r[15];
#pragma unroll
        for (int p = 0; p < 15; ++p) pw[1 + p] = r[p];
      }
      finish_tile<16>(sink, [&](auto i) { return pw[decltype(i)::value]; }, pl, tile, ntiles, wl, &sh_base, wave, lane);
    } else {
      // a tile with a block wider than 15 bits (input outside the guaranteed domain): all planes
      u32 lo[16], hi[16];
#pragma unroll
      for (int j = 0; j < 32; ++j) asm volatile("" : "+v"(d[j]));
      planes_from_deltas32(d, lo, hi);
      auto word = [&](auto i) {
        constexpr int I = decltype(i)::value;      // 0: sign, 1..16: low planes, 17..31: high planes
        if constexpr (I == 0) return hi[15];
        else if constexpr (I <= 16) return lo[I - 1];
        else return hi[I - 17];
      };
      finish_tile<32>(sink, word, pl, tile, ntiles, wl, &sh_base, wave, lane);
    }
  }
  if (err) atomicOr(&a.ctl->status, err);
}

// Clears the control block and the tile descriptors, and writes the fixed header fields and
// the zero padding of the two tables.  Runs before compress_kernel / reduce_kernel.
struct InitArgs {
  Control* ctl;
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
  for (u64 i = gid; i < a.ntiles; i += stride) a.desc[desc_slot(i)] = 0;
  if (gid == 0) {
    for (int i = 0; i < kTicketShards; ++i) *ticket_counter(a.ctl, u32(i)) = 0;
    a.ctl->status = 0;
    a.ctl->flags = 0;
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

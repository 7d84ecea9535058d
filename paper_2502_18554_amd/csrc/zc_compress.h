// fZ-light compression kernel (Section 3.3): quantise, per-block Lorenzo delta, code length,
// sign + plane packing, single-pass placement of the variable-size blocks.
//
// Work split.  A tile is 512 blocks (16384 values, 64 KiB of input) handled by a workgroup of
// 8 waves.  Each wave loads 2048 consecutive values with 16-byte loads,
// quantises them where they land, and transposes the integer codes through LDS so that one
// lane owns one block.  Deltas (kept as 16 words of paired 16-bit fields), width and the
// bit-matrix transpose that yields the plane words are then in-lane; the packed words wait
// in registers for the tile's base offset from the look-back scan and leave through LDS as
// coalesced stores.
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
  u32 ticketed;      // tiles handed out by tickets instead of by workgroup id
  u32 coherent;      // the look-back reads the tile's own chain with device-coherent loads too
  u32 ix;            // write an indexed stream (see index_bytes)
  u32 part_end;      // zc_compress_part: one past the last tile of this call; else 0
  u32 adopt;         // this launch continues a call (a later part, the ragged last tile): its tag is in the control block
  u64 nonce;         // drawn by the host per call, goes into the tag (see launch_tag)
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
    for (int i = 0; i < 8; ++i) x[i] = load_once(reinterpret_cast<const float4*>(a.in + v0 + u64(256 * i + 4 * lane)));
    // Nothing moves across this line: left to itself the compiler puts the first use of the first value,
    // and the wait for it, in front of the last four loads, which then go out a round trip late.
    __builtin_amdgcn_sched_barrier(0);
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

// Quantise the wave's values where they landed and transpose the codes through LDS so that one
// lane owns one block: q[j] = code j of the lane's block.
template <bool FULL>
__device__ inline void block_codes(const CompressArgs& a, const float4 (&x)[8], u64 wblock0, int lane, u32* wl,
                                   i32 (&q)[32], u32& err) {
  // Some value of this wave outside the screened domain: the checked arithmetic for all of it.
  u32 flagged = 0;            // (no short-circuit: the four compares of a load are independent)
#pragma unroll
  for (int i = 0; i < 8; ++i)
    flagged |= u32(needs_checks(x[i].x, a)) | u32(needs_checks(x[i].y, a)) | u32(needs_checks(x[i].z, a)) |
               u32(needs_checks(x[i].w, a));
  const bool checked = __any(flagged != 0);

  // Loads 0..3 hold blocks 0..31, loads 4..7 blocks 32..63.  Either half goes through LDS as 32 rows
  // of 32 codes, and every lane takes half a row: lane l and lane l + 32 the first and the second 16
  // codes of block l (then of block 32 + l).  That keeps 16 registers per half and lane instead of 32 in
  // half the lanes; one swap of the upper 32 lanes of a register with the lower 32 of another per pair
  // of codes then gives every lane the 32 codes of its own block.
  i32 h0[16], h1[16];
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<int4*>(wl + (8 * i + (lane >> 3)) * kStageRow + 4 * (lane & 7)) =
          quantize4(x[4 * half + i], a, checked, err);
    wave_lds_sync();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int4 r = *reinterpret_cast<const int4*>(wl + (lane & 31) * kStageRow + 16 * (lane >> 5) + 4 * t);
      i32* const h = half ? h1 : h0;
      h[4 * t + 0] = r.x; h[4 * t + 1] = r.y; h[4 * t + 2] = r.z; h[4 * t + 3] = r.w;
    }
    wave_lds_sync();
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    // -> {lanes 0..31 of h0 | lanes 0..31 of h1}, {lanes 32..63 of h0 | lanes 32..63 of h1}
    const auto r = __builtin_amdgcn_permlane32_swap(u32(h0[j]), u32(h1[j]), false, false);
    q[j] = i32(r[0]);
    q[16 + j] = i32(r[1]);
  }
  if (!FULL) {
    // the last block repeats its last code up to 32 values
    const u64 b = wblock0 + u64(lane);
    const u64 cnt = b < a.nb ? a.n - b * kBlockValues : 0;
#pragma unroll
    for (int j = 1; j < 32; ++j) q[j] = u64(j) < cnt ? q[j] : q[j - 1];
  }
}

// The block as the kernel keeps it: the Lorenzo deltas (d0 = 0) as two's complement fields of
// 16 bits, two per word (exact for widths up to 15), their largest magnitude, which gives the
// width, and the first code (the outlier).
struct BlockFields {
  u32 f[16];
  u32 any;
  i32 outlier;
};

template <bool FULL>
__device__ inline void block_fields(const CompressArgs& a, const float4 (&x)[8], u64 wblock0, int lane, u32* wl,
                                    BlockFields& bf, u32& err) {
  i32 q[32];
  block_codes<FULL>(a, x, wblock0, lane, wl, q, err);
  bf.outlier = q[0];
  i32 top = 0, bottom = 0;              // largest and smallest delta (d0 = 0 is one of them)
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const i32 lo = j ? q[j] - q[j - 1] : 0;
    const i32 hi = q[j + 16] - q[j + 15];
    top = max(top, max(lo, hi));
    bottom = min(bottom, min(lo, hi));
    bf.f[j] = field16_pair(lo, hi);
    // (pins the field here: left to itself the compiler keeps all 32 deltas alive instead and
    //  builds the fields where they are used, after the barrier)
    asm volatile("" : "+v"(bf.f[j]));
  }
  const u32 any = max(u32(top), u32(-bottom));   // largest magnitude: its bit length is the width
  bf.any = any;
}

// A tile that holds a block wider than 15 bits (an input outside the guaranteed domain).
// The 16-bit fields are of no use then.  Once the tile's base offset is known, every wave
// fetches and quantises its values again, half a wave of blocks at a time, and leaves the
// codes in LDS; then 32 lanes take the 32 values of one block (two blocks per step), and a
// plane word is simply the ballot of one bit of the magnitudes.  Slow, rare, and it needs
// next to no registers, so it does not limit how many waves of the kernel fit a SIMD.
template <bool FULL>
__device__ inline void wide_tile(const CompressArgs& a, const PayloadSink& sink, const Placement& pl, u32 tile,
                                 u32 ntiles, u64 wblock0, u32* wl, u64* sh_base, int wave, int lane) {
  const TileBase tb = resolve_tile_base(sink, pl, tile, sh_base, wave, lane);
  const u64 base = tb.words;
  if (lane == 0) write_index_entry(sink, tile * kPackWaves + u32(wave), base + pl.wave_off);
  const u64 tend = tables_end(a.nb, a.ix);
  const u64 cap_words = a.out_cap > tend ? (a.out_cap - tend) / 4 : 0;
  u32* const payload = reinterpret_cast<u32*>(a.out + tend);
  const u64 wave_first = base + pl.wave_off;                      // first payload word of this wave
  const int j = lane & 31;                                        // value inside the block
  u32 ignored = 0;                                                // errors were raised on the first pass

#pragma nounroll
  for (int half = 0; half < 2; ++half) {
    // codes of blocks [32 half, 32 half + 32) of the wave -> LDS rows of 32 codes
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u64 idx = wblock0 * kBlockValues + u64(1024 * half + 256 * i + 4 * lane);
      float4 x;
      if (FULL) {
        x = *reinterpret_cast<const float4*>(a.in + idx);
      } else {
        x.x = idx + 0 < a.n ? a.in[idx + 0] : 0.0f;
        x.y = idx + 1 < a.n ? a.in[idx + 1] : 0.0f;
        x.z = idx + 2 < a.n ? a.in[idx + 2] : 0.0f;
        x.w = idx + 3 < a.n ? a.in[idx + 3] : 0.0f;
      }
      *reinterpret_cast<int4*>(wl + (8 * i + (lane >> 3)) * kStageRow + 4 * (lane & 7)) = quantize4(x, a, true, ignored);
    }
    wave_lds_sync();
#pragma nounroll
    for (int bp = 0; bp < 16; ++bp) {
      const int blk_a = 32 * half + 2 * bp;                       // blocks of this step, inside the wave
      const u32 w_a = lane_value(pl.w, blk_a), w_b = lane_value(pl.w, blk_a + 1);
      if ((w_a | w_b) == 0) continue;
      const u32 off_a = lane_value(pl.off_in_wave, blk_a), off_b = lane_value(pl.off_in_wave, blk_a + 1);
      const int row = 2 * bp + (lane >> 5);                       // LDS row of this lane's block
      int jj = j, jp = j ? j - 1 : 0;                             // this value and the one before it
      if (!FULL) {                                                // the last block repeats its last code
        const u64 b = wblock0 + u64(32 * half + row);
        const u64 cnt = b < a.nb ? a.n - b * kBlockValues : 1;
        if (u64(jj) >= cnt) jj = int(cnt) - 1;
        if (u64(jp) >= cnt) jp = int(cnt) - 1;
      }
      const i32 q = i32(wl[row * kStageRow + jj]);
      const i32 qp = i32(wl[row * kStageRow + jp]);
      const i32 d = j ? q - qp : 0;
      const u32 mag = u32(d < 0 ? -d : d);
      const bool first_lane = j == 0;
      const u32 w_mine = lane < 32 ? w_a : w_b;
      const u64 dst = wave_first + (lane < 32 ? off_a : off_b);   // this block's sign word
      const u64 sign = __ballot(d < 0);
      if (first_lane && w_mine && dst < cap_words) payload[dst] = lane < 32 ? u32(sign) : u32(sign >> 32);
      const u32 w_top = w_a > w_b ? w_a : w_b;
#pragma nounroll
      for (u32 p = 0; p < w_top; ++p) {
        const u64 plane = __ballot(((mag >> p) & 1u) != 0);
        if (first_lane && p < w_mine && dst + 1 + p < cap_words)
          payload[dst + 1 + p] = lane < 32 ? u32(plane) : u32(plane >> 32);
      }
    }
    wave_lds_sync();
  }
  finish_stream(sink, pl, tile, ntiles, tb);
}

// One workgroup per tile.  FULL = the launch covers tiles whose 16384 values all exist
// (pure 16-byte loads, no tail), tile = first_tile + workgroup id, or + a ticket (see
// take_tile), over [first_tile, end_tile); the ragged last tile of an input runs as a launch
// of its own, of one workgroup, with FULL = false on tile first_tile.  There is no set-up
// launch: tile 0 writes the header, and nothing in the workspace needs clearing (see launch_tag).
template <bool FULL>
__global__ __launch_bounds__(kPackThreads, FULL ? 8 : 6) void compress_kernel(CompressArgs a, u32 first_tile, u32 end_tile) {
  __shared__ __attribute__((aligned(16))) u32 lds[kPackWaves * kWaveStage];
  __shared__ u32 sh_tile;
  __shared__ u32 sh_wave_total[kPackWaves];
  __shared__ u32 sh_wave_wmax[kPackWaves];
  __shared__ u64 sh_base;

  const int lane = lane_id();
  const int wave = int(threadIdx.x) >> 6;
  const u32 ntiles = u32(num_pack_tiles(a.nb));
  u32* const wl = lds + wave * kWaveStage;
  const bool tables_fit = a.out_cap >= tables_end(a.nb, a.ix);
  u32 err = 0;

  const u64 ltag = launch_tag(a.nonce, a.ctl);
  const u64 tag = call_tag(a.ctl, ltag, a.adopt != 0);
  u32 tile = first_tile;
  if (FULL) {
    tile = first_tile + blockIdx.x;          // tiles in the order in which workgroups start
    if (a.ticketed) {                        // ... or handed out by tickets, see take_tile
      if (threadIdx.x == 0) {
        const u32 t = take_tile(a.ctl, ltag, end_tile - first_tile, ticket_shard());
        sh_tile = t == kNoTile ? kNoTile : first_tile + t;
      }
      __syncthreads();
      tile = uniform(sh_tile);
    }
    if (tile >= end_tile) return;
  }
  // the first tile also writes the fixed header fields and the padding of the tables
  if (tile == 0 && threadIdx.x == 0) {
    if (tables_fit) write_stream_header(a.out, a.n, a.nb, a.eb_bits, 1u, a.ix != 0, false);
    else raise_status(a.ctl, tag, status_bit(ZC_ERR_CAPACITY));
  }
  {
    const u64 wblock0 = u64(tile) * kPackBlocks + u64(wave) * kWaveBlocks;
    const u64 b = wblock0 + u64(lane);
    const bool active = b < a.nb;
    float4 x[8];
    load_raw<FULL>(a, wblock0, lane, x);

    BlockFields bf;
    block_fields<FULL>(a, x, wblock0, lane, wl, bf, err);
    Placement pl;
    pl.w = (active && bf.any) ? 32u - u32(__builtin_clz(bf.any)) : 0u;
    pl.wmax = wave_max_u32(pl.w);
    // (the width and the outlier go to their tables at the very end: a store that is under way is
    // waited for by the barrier below, and by every poll of the look-back)

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
    lds_barrier();     // wave totals visible
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
    pl.tile_wide = a.ix && tile_wmax > 15;
    const PayloadSink sink{a.out, a.out_cap, a.nb, a.ctl, a.desc, a.ix != 0, a.coherent != 0, a.part_end, tag};
    if (threadIdx.x == 0) publish_tile_size(sink, tile, pl.tile_total, pl.tile_wide);

    // ---- fields -> sign + plane words in registers, then the back half ----
    if (tile_wmax <= 15) {
      finish_staged_tile<16>(sink, pl, tile, ntiles, wl, &sh_base, wave, lane, [&] {
        u32 pw[16];          // pw[0] = sign, pw[1 + p] = plane p
        if (pl.wmax <= 7) {
          u32 r[8];
          planes8_from_fields16(bf.f, r);
          pw[0] = r[7];
#pragma unroll
          for (int p = 0; p < 7; ++p) pw[1 + p] = r[p];
#pragma unroll
          for (int p = 8; p < 16; ++p) pw[p] = 0;
        } else {
          planes16_from_fields(bf.f);
          pw[0] = bf.f[15];
#pragma unroll
          for (int p = 0; p < 15; ++p) pw[1 + p] = bf.f[p];
        }
        stage_wave_words<16>([&](auto i) { return pw[decltype(i)::value]; }, pl, wl);
      });
    } else {
      wide_tile<FULL>(a, sink, pl, tile, ntiles, wblock0, wl, &sh_base, wave, lane);
    }
    if (active && tables_fit) {
      a.out[widths_begin(a.nb, a.ix) + b] = u8(pl.w);
      reinterpret_cast<i32*>(a.out + outliers_begin(a.nb, a.ix))[b] = bf.outlier;
    }
  }
  if (err) raise_status(a.ctl, tag, err);
}

// The stream of no values: a header (and the one closing entry of an indexed stream's index).
struct EmptyStreamArgs {
  Control* ctl;
  u8* out;
  u64 out_cap;
  u32 eb_bits;
  u32 ix;
  u64 nonce;
};

__global__ void empty_stream_kernel(EmptyStreamArgs a) {
  const u64 tag = call_tag(a.ctl, launch_tag(a.nonce, a.ctl), false);
  if (threadIdx.x != 0) return;
  const u64 tend = tables_end(0, a.ix != 0);
  a.ctl->result = tend;
  if (a.out_cap >= tend) write_stream_header(a.out, 0, 0, a.eb_bits, 1u, a.ix != 0, true);
  else raise_status(a.ctl, tag, status_bit(ZC_ERR_CAPACITY));
}

}  // namespace zc

// Shared definitions of the HIP codec: stream geometry, workspace layout, status bits and
// the wave-level building blocks (scan, look-back) used by the kernels.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/zc.h"

namespace zc {

using u8 = uint8_t;
using u16 = uint16_t;
using u32 = uint32_t;
using u64 = uint64_t;
using i32 = int32_t;
using i64 = int64_t;
typedef u32 u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr u32 kMagic = 0x314C435Au;
constexpr u32 kHeaderBytes = 32;
constexpr int kBlockValues = 32;           // values per block (Section 3.3 "small blocks")
constexpr int kWaveBlocks = 64;            // one lane owns one block
constexpr int kTileWaves = 4;
constexpr int kTileThreads = kTileWaves * 64;
constexpr int kTileBlocks = kTileWaves * kWaveBlocks;        // 256 blocks
constexpr int kTileValues = kTileBlocks * kBlockValues;      // 8192 values = 32 KiB of input
constexpr i64 kMaxCode = (i64(1) << 30) - 1;
constexpr u32 kSpinLimit = 1u << 20;       // bound on every look-back wait

__host__ __device__ constexpr u64 pad16(u64 v) { return (v + 15) / 16 * 16; }
__host__ __device__ constexpr u64 num_blocks(u64 n) { return (n + kBlockValues - 1) / kBlockValues; }
__host__ __device__ constexpr u64 num_tiles(u64 nb) { return (nb + kTileBlocks - 1) / kTileBlocks; }
// No stream has more tiles than this (n <= ZC_MAX_N), so block and segment numbers fit 32 bits.
constexpr u64 kMaxTiles = (ZC_MAX_N / kBlockValues + kTileBlocks - 1) / kTileBlocks;
__host__ __device__ inline u32 psize_words(u32 w) { return w ? 1 + w : 0; }

// Stream layout.  The plain stream (version 1) is header, width table, outlier table,
// payload.  The indexed stream (Section 3.5.2 keeps the compressed size of every chunk in
// front of the data, so that a chunk can be handled without looking at the others; here a
// chunk is a segment, the 64 blocks of one wave) has version 2, or 3 when some block is wider
// than 15 bits, and between header and width table an index of nseg + 1 u32: entry i is the
// payload word offset of segment i, entry nseg the number of payload words; zero padded to 16
// bytes.  `ix` says which of the two a kernel reads and writes; it is the same for every
// stream of one call (the call's flags say which).
__host__ __device__ inline u64 num_segments(u64 nb) { return (nb + kWaveBlocks - 1) / kWaveBlocks; }
__host__ __device__ inline u64 index_bytes(u64 nb, bool ix) { return ix ? pad16(4 * (num_segments(nb) + 1)) : 0; }
__host__ __device__ inline u64 widths_begin(u64 nb, bool ix) { return kHeaderBytes + index_bytes(nb, ix); }
__host__ __device__ inline u64 outliers_begin(u64 nb, bool ix) { return widths_begin(nb, ix) + pad16(nb); }
__host__ __device__ inline u64 tables_end(u64 nb, bool ix) { return outliers_begin(nb, ix) + pad16(4 * nb); }
constexpr u32 kVersionPlain = 1u | (5u << 16) | (6u << 24);     // header word 1: version, block_log2, guard_log2
constexpr u32 kVersionIndexed = 2u | (5u << 16) | (6u << 24);   // | 1 when some block is wider than 15 bits

// Device status word: bit i set <=> error code i was raised.
__host__ __device__ constexpr u32 status_bit(int code) { return 1u << code; }

// Errors that stop a call before it writes anything: bad arguments, malformed or mismatched
// input streams.  Every workgroup of a main kernel takes the same decision on them, either
// from the verdict the validation kernel of plain streams left (zc_scan.h) or from the same
// header bytes (indexed streams).
constexpr u32 kGateBits = status_bit(ZC_ERR_ARG) | status_bit(ZC_ERR_FORMAT) | status_bit(ZC_ERR_MISMATCH);

// Control part of the caller's workspace.  Tile tickets, tile descriptors and segment-offset
// tables follow.  Nothing in a workspace is ever cleared: whatever one call shares between its
// workgroups or its launches carries the call's tag (below), and a word with another tag counts
// as empty, so a workspace may hold anything when a call starts.
constexpr int kTicketsPerXcd = 4;
constexpr int kTicketShards = 8 * kTicketsPerXcd;
struct Control {
  u64 status;                  // bits 63..32: high half of the tag of the call that raised them; bits 31..0: OR of status_bit()s and kStatusWide
  u64 call_tag;                // tag of the last call's first launch; its later launches take it from here
  u64 result;                  // total_bytes, or n for decompress
  u64 nsum;                    // sum of the input streams' nsum fields (plain streams: set by index_prep_kernel)
  u32 pad[8];
};
static_assert(sizeof(Control) == 64, "control block is 64 bytes");

// Tile hand-out counters, four per XCD (see take_tile), follow the control block.  Each sits
// in a 128-byte line of its own, and none shares the line of the control block: accesses to
// one line retire one after the other even when they address different words of it, and every
// workgroup reads the control block when it starts.
constexpr int kTicketStride = 16;            // in u64
constexpr u64 kTicketBytes = u64(kTicketShards + 1) * kTicketStride * 8;
__host__ __device__ inline u64* ticket_counter(Control* ctl, u32 shard) {
  return reinterpret_cast<u64*>(ctl + 1) + (shard + 1) * kTicketStride;
}

// A segment is the 64 blocks owned by one wave; a tile is 4 segments.

// Positions inside an existing stream are kept at three levels (see zc_scan.h): the offset of
// every segment inside its scan group of 64 segments, the offset of every group inside its
// index span of 8 groups (the share of one workgroup of the index kernel), and the offset of
// every span.  A reader adds the three.
constexpr int kScanGroupSegs = 64;
constexpr int kScanGroupBlocks = kScanGroupSegs * kWaveBlocks;     // 4096 blocks
constexpr int kIndexGroups = 8;                                    // scan groups per index span
constexpr int kSpanSegs = kIndexGroups * kScanGroupSegs;           // 512 segments = 32768 blocks
__host__ __device__ inline u64 num_scan_groups(u64 nb) { return (nb + kScanGroupBlocks - 1) / kScanGroupBlocks; }
__host__ __device__ inline u64 num_spans(u64 nb) { return (num_scan_groups(nb) + kIndexGroups - 1) / kIndexGroups; }

struct StreamIndex {
  u32* seg_off;     // [k][4 * tiles_cap]   payload word offset of each segment inside its scan group
  u32* grp_off;     // [k][groups_cap]      payload word offset of each scan group inside its span
  u32* span_off;    // [k][spans_cap]       payload word offset of each span (its size between the two index kernels)
  u32* span_flags;  // [k][spans_cap]       what stream_index_kernel saw in each span
  u64 tiles_cap;
  u64 groups_cap;
  u64 spans_cap;
};

// How a workspace of ws_bytes is carved up for calls with k input streams:
//   Control | tickets | desc[tiles_cap] (128 B each) | seg_off[k][4 * tiles_cap] | grp_off[k][groups_cap] |
//   span_off[k][spans_cap] | span_flags[k][spans_cap]
// tiles_cap follows from ws_bytes alone, so kernels can refuse streams that do not fit.
struct WorkspaceLayout {
  u64 tiles_cap;
  Control* ctl;
  u64* desc;        // look-back descriptors, kDescStride words per tile
  StreamIndex index;
};

constexpr u64 kDescBytes = 128;           // per tile, see kDescStride
constexpr u64 kWsFixed = sizeof(Control) + kTicketBytes + 12 * ZC_MAX_K + 64;   // control, tickets, the +1 of every grp_off, span_off and span_flags row, padding

__host__ constexpr u64 workspace_bytes(u64 n_max, int k_max) {
  if (k_max < 1) k_max = 1;
  const u64 t = num_tiles(num_blocks(n_max)) + 16;
  return kWsFixed + t * (kDescBytes + 17 * u64(k_max));      // 17 >= segment offsets (16) + the tile's share of the two coarser levels
}

__host__ inline WorkspaceLayout workspace_layout(void* d_ws, u64 ws_bytes, int k) {
  if (k < 1) k = 1;
  WorkspaceLayout l;
  l.tiles_cap = ws_bytes > kWsFixed ? (ws_bytes - kWsFixed) / (kDescBytes + 17 * u64(k)) : 0;
  u8* p = static_cast<u8*>(d_ws);
  l.ctl = reinterpret_cast<Control*>(p);
  p += sizeof(Control) + kTicketBytes;
  l.desc = reinterpret_cast<u64*>(p);
  p += kDescBytes * l.tiles_cap;
  l.index.tiles_cap = l.tiles_cap;
  l.index.groups_cap = l.tiles_cap / 16 + 1;        // 16 tiles = 64 segments = one scan group
  l.index.spans_cap = l.tiles_cap / (16 * kIndexGroups) + 1;
  l.index.seg_off = reinterpret_cast<u32*>(p);
  p += pad16(16 * l.tiles_cap * u64(k));
  l.index.grp_off = reinterpret_cast<u32*>(p);
  p += 4 * l.index.groups_cap * u64(k);
  l.index.span_off = reinterpret_cast<u32*>(p);
  p += 4 * l.index.spans_cap * u64(k);
  l.index.span_flags = reinterpret_cast<u32*>(p);
  return l;
}

// ---------------------------------------------------------------------------------------
// Wave-level primitives (64 lanes).
// ---------------------------------------------------------------------------------------
__device__ inline int lane_id() { return int(threadIdx.x) & 63; }

// Not an error: the validation kernel of plain streams found a block wider than 15 bits (the
// host ignores the bit).
constexpr u32 kStatusWide = 1u << 16;

// Tile hand-out.  A kernel that places its output by look-back needs every tile below a tile
// in work to be in work too, or finished.  Two ways to get that:
//  - by workgroup id (the default): tile = blockIdx.x.  The dispatcher of this GPU starts the
//    workgroups of a launch in increasing id order (measured: workgroup i always lands on XCD
//    (i + 7) mod 8, and start times follow the ids), so a running workgroup's predecessors have
//    all started.  That order is how the hardware works, not an architectural promise, which
//    is why every look-back wait is bounded and turns into ZC_ERR_HIP instead of a hang.
//  - by tickets: the order of the claims is the order of the tiles, whatever the dispatcher
//    does.  It costs each workgroup one atomic round trip before it can issue its first load
//    (the kernels that read headers first ask for the ticket before that, see ask_ticket).
// Tickets: one atomic counter would serialise the whole kernel: atomics on one
// address retire at about 11 ns each on this machine when nothing else runs and far slower
// under load, which for 16384 tiles is longer than the kernel should run.  So there are 32
// counters, four per XCD: a workgroup asks the one picked by the hardware XCC_ID of its waves
// and two bits of its id (ticket_shard), and counter y hands out tiles y, y + 32, y + 64, ...,
// which are tiles of the XCD's own chains (y mod 8 is the XCD).  With one counter per XCD the
// atomics alone took a tenth of a kernel's time (512^3 compress by ticket 149 us, with four
// 135 us).  A workgroup whose own counter is exhausted helps the others, its XCD's first, so
// every tile is claimed exactly once whatever the placement of workgroups.  Look-back stays
// deadlock-free: the workgroups that ask a counter hold its tiles in increasing order, so the
// smallest unfinished tile overall is either running or is the next one its counter hands out,
// to the next workgroup that asks it, and the workgroups that asked it before hold smaller
// tiles, which finish.  (A counter that no workgroup asks, because the launch is kept off an XCD
// altogether, is served only once the others are exhausted, which the tiles that wait for its
// tiles keep from happening: such a launch ends in ZC_ERR_HIP when the waits run out, and
// should use the other hand-out.)
__device__ inline u32 xcc_id() {
  return u32(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11))) & 7u;   // HW_REG_XCC_ID[3:0]
}
// The counter a workgroup asks: one of the four of its XCD, in turn (workgroup ids go round the XCDs,
// so id / 8 counts the workgroups of an XCD).
__device__ inline u32 ticket_shard() { return xcc_id() | (((blockIdx.x >> 3) & u32(kTicketsPerXcd - 1)) << 3); }

constexpr u32 kNoTile = 0xffffffffu;

__device__ inline u32 tile_of_ticket(u32 shard, u32 ticket, u32 ntiles) {
  const u64 t = u64(ticket) * kTicketShards + shard;
  return t < ntiles ? u32(t) : kNoTile;
}

// A ticket counter is a 64-bit word: the top 40 bits of the tag of the launch that counts in it,
// then 24 bits of count.  A word with another tag is a counter at zero.  The common case is one
// atomic add; the first workgroups of a launch to reach a counter find the tag of an older
// launch (or anything at all) in it and install their own by compare-and-swap.
constexpr u64 kTicketCountMask = (u64(1) << 24) - 1;

// (in two halves, so that a caller can have the add under way while it does other work)
__device__ inline u64 ask_ticket(u64* counter) { return atomicAdd(reinterpret_cast<unsigned long long*>(counter), 1ull); }

__device__ inline u32 take_ticket(u64* counter, u64 ltag, u64 old) {      // old = ask_ticket(counter)
  const u64 mine = ltag & ~kTicketCountMask;
  if ((old & ~kTicketCountMask) == mine) return u32(old & kTicketCountMask);
  old = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (u32 tries = 0; tries < kSpinLimit; ++tries) {
    if ((old & ~kTicketCountMask) == mine) {
      old = atomicAdd(reinterpret_cast<unsigned long long*>(counter), 1ull);
      if ((old & ~kTicketCountMask) == mine) return u32(old & kTicketCountMask);
    } else if (__hip_atomic_compare_exchange_strong(counter, &old, mine | 1ull, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT)) {
      return 0u;
    }
  }
  return u32(kTicketCountMask);            // never handed out as a tile: the caller finds no tile
}

// Claims the next tile (called by one thread of a workgroup).  kNoTile when none is left.
// `asked` = ask_ticket(ticket_counter(ctl, first_shard)), which the caller may have issued earlier.
__device__ inline u32 take_tile(Control* ctl, u64 ltag, u32 ntiles, u32 first_shard, u64 asked) {
#pragma nounroll
  for (u32 i = 0; i < u32(kTicketShards); ++i) {
    const u32 y = (first_shard + 8u * (i % u32(kTicketsPerXcd)) + i / u32(kTicketsPerXcd)) & (kTicketShards - 1);   // the XCD's own counters first
    if (i) asked = ask_ticket(ticket_counter(ctl, y));
    if (y >= ntiles) continue;
    const u32 t = tile_of_ticket(y, take_ticket(ticket_counter(ctl, y), ltag, asked), ntiles);
    if (t != kNoTile) return t;
  }
  return kNoTile;
}
__device__ inline u32 take_tile(Control* ctl, u64 ltag, u32 ntiles, u32 first_shard) {
  return take_tile(ctl, ltag, ntiles, first_shard, ask_ticket(ticket_counter(ctl, first_shard)));
}

// Lane-crossing primitives are built from DPP moves and v_readlane, which need no address
// registers and do not go through the LDS pipe (unlike ds_bpermute shuffles).
template <int CTRL>
__device__ inline u32 dpp_mov(u32 v) {
  return u32(__builtin_amdgcn_update_dpp(int(v), int(v), CTRL, 0xf, 0xf, false));
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

__device__ inline u32 lane_value(u32 v, int lane) { return u32(__builtin_amdgcn_readlane(int(v), lane)); }

// A value known to be the same in every lane, moved to a scalar register so that branches on
// it are scalar branches.
__device__ inline u32 uniform(u32 v) { return u32(__builtin_amdgcn_readfirstlane(int(v))); }
__device__ inline u64 uniform64(u64 v) { return u64(uniform(u32(v))) | (u64(uniform(u32(v >> 32))) << 32); }

// ---------------------------------------------------------------------------------------
// Call tags.  A tag is a 64-bit number that is the same in every workgroup of one launch and
// that no earlier launch on the same workspace has had: the packet number of the dispatch in
// its hardware queue (which a replay of a captured graph renews as well), the queue, a number
// the host draws per call (its clock), and the workspace address, mixed.  A call of several
// launches (a stream compressed in parts, the ragged last tile, the validation kernels of plain
// streams) uses the tag of its first launch throughout: that launch leaves it in the control
// block, the later ones pick it up there (`adopt`).
// ---------------------------------------------------------------------------------------
extern "C" __device__ u64 zc_dispatch_id(void) __asm("llvm.amdgcn.dispatch.id");

__device__ inline u64 mix64(u64 x) {
  x ^= x >> 31;
  x *= 0x9E3779B97F4A7C15ull;
  x ^= x >> 29;
  return x;
}

__device__ inline u64 launch_tag(u64 nonce, const void* ws) {
  const u64 queue = u64(reinterpret_cast<uintptr_t>(__builtin_amdgcn_queue_ptr()));
  u64 t = mix64(zc_dispatch_id() + 0x632BE59BD9B4E019ull * (queue >> 6));
  t = mix64(t ^ nonce);
  t = mix64(t + u64(reinterpret_cast<uintptr_t>(ws)));
  return uniform64(t);
}

// The tag of the call this launch belongs to; the first launch of a call also records it.
__device__ inline u64 call_tag(Control* ctl, u64 ltag, bool adopt) {
  if (adopt) return uniform64(*reinterpret_cast<volatile const u64*>(&ctl->call_tag));
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) ctl->call_tag = ltag;
  return ltag;
}

// Status bits are raised under the call's tag: the first raise of a call replaces whatever an
// earlier call left, later ones add to it.  Rare, so a compare-and-swap loop will do.
__device__ inline void raise_status(Control* ctl, u64 tag, u32 bits) {
  const u64 mine = tag & 0xffffffff00000000ull;
  u64 old = __hip_atomic_load(&ctl->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int tries = 0; tries < 4096; ++tries) {
    const u64 want = ((old & 0xffffffff00000000ull) == mine ? old : mine) | bits;
    if (want == old) return;
    if (__hip_atomic_compare_exchange_strong(&ctl->status, &old, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT))
      return;
  }
}

// The bits raised so far under this tag.
__device__ inline u32 status_bits(const Control* ctl, u64 tag) {
  const u64 v = __hip_atomic_load(&ctl->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return (v >> 32) == (tag >> 32) ? u32(v) : 0u;
}

// Loads and stores of data that a kernel touches once, with the non-temporal hint.  Such data
// then neither pushes the lines that are used again (the stream index, tables shared by
// neighbouring waves, tile descriptors) out of the L2, nor stays behind as dirty lines that
// the next kernel has to write back while it runs.  Where it pays is a matter of measurement
// (times of the three kernels inside one loop): the input values of the compression (-21 us
// for it, +15 us for the kernel after it), the floats the decompression writes (-27 us for
// it, nothing lost elsewhere), the payload loads of the reduce (-23 us; they read several
// streams side by side), the payload it writes (-14 us), and the payload the compression writes
// (nothing for it once every store covers whole lines, see copy_staged_words; -17 us and -5 us
// for the two kernels after it, measured with the decompression reading a stream that is no
// longer in any cache).  It costs time on the payload and outlier loads of the decompression.
__device__ inline uint4 load_once(const uint4* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ inline void store_once(float4* p, const float4& v) {
  const f32x4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4_t*>(p));
}
__device__ inline void store_once(u32* p, u32 v) { __builtin_nontemporal_store(v, p); }
__device__ inline float4 load_once(const float4* p) {
  const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(t.x, t.y, t.z, t.w);
}

// A zero in a vector register that the compiler cannot see through.  An address that has it
// added is not provably the same in every lane, so the access becomes a vector memory load.
// Vector loads return in order and have a counter of their own: several independent loads
// are all in flight behind a single wait.  Loads from a provably uniform address of memory
// not yet written by the kernel are turned into scalar loads instead, which share one
// counter with the fetches of kernel arguments and return in any order, so the compiler has
// to drain all of them at every use: three round trips where one will do.
__device__ inline u32 opaque_zero() {
  u32 z;
  asm volatile("v_mov_b32 %0, 0" : "=v"(z));
  return z;
}
// Index of the calling wave in its workgroup, as a scalar.
__device__ inline int wave_id() { return int(uniform(threadIdx.x >> 6)); }
// base + byte offset, for a base that is the same in every lane: it stays in scalar registers
// and the access needs one 32-bit vector register for the offset instead of a 64-bit address.
template <typename T>
__device__ inline T* at_bytes(T* uniform_base, u32 byte_offset) {
  using Byte = std::conditional_t<std::is_const_v<T>, const char, char>;
  return reinterpret_cast<T*>(reinterpret_cast<Byte*>(uniform_base) + byte_offset);
}

// Sum over the 64 lanes (result uniform).
__device__ inline u32 wave_sum_u32(u32 v) {
  v += dpp_mov<kDppQuadSwap1>(v);
  v += dpp_mov<kDppQuadSwap2>(v);
  v += dpp_mov<kDppRowHalfMirror>(v);
  v += dpp_mov<kDppRowMirror>(v);          // every lane of a row of 16 now holds the row's sum
  return lane_value(v, 0) + lane_value(v, 16) + lane_value(v, 32) + lane_value(v, 48);
}

// Maximum over the 64 lanes (result uniform).
__device__ inline u32 wave_max_u32(u32 v) {
  u32 o;
  o = dpp_mov<kDppQuadSwap1>(v); v = o > v ? o : v;
  o = dpp_mov<kDppQuadSwap2>(v); v = o > v ? o : v;
  o = dpp_mov<kDppRowHalfMirror>(v); v = o > v ? o : v;
  o = dpp_mov<kDppRowMirror>(v); v = o > v ? o : v;
  const u32 a = lane_value(v, 0), b = lane_value(v, 16), c = lane_value(v, 32), d = lane_value(v, 48);
  const u32 ab = a > b ? a : b, cd = c > d ? c : d;
  return ab > cd ? ab : cd;
}

// Row shift right by S lanes inside each row of 16 lanes; lanes without a source get 0.
template <int S>
__device__ inline u32 dpp_row_shr_or_zero(u32 v) {
  return u32(__builtin_amdgcn_update_dpp(0, int(v), 0x110 + S, 0xf, 0xf, false));
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ inline u32 wave_inclusive_sum(u32 v) {
  v += dpp_row_shr_or_zero<1>(v);
  v += dpp_row_shr_or_zero<2>(v);
  v += dpp_row_shr_or_zero<4>(v);
  v += dpp_row_shr_or_zero<8>(v);
  // v is now the scan inside each row of 16; add the totals of the earlier rows
  const u32 t0 = lane_value(v, 15), t1 = lane_value(v, 31), t2 = lane_value(v, 47);
  int row = lane_id() >> 4;
  u32 carry = (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
  return v + carry;
}

// ---------------------------------------------------------------------------------------
// Tile descriptors of the look-back (see "Look-back by chains" below).  A descriptor is two 64-bit
// words in a 128-byte line of its own.  Word 0: bits 63..62 = state (0 empty, 1 the tile's size,
// 2 the sum of the sizes of the tiles of its chain up to and including it), bit 61 = the tile
// (or, in a chain sum, some tile of the chain up to this one) holds a block wider
// than 15 bits, bits 60..32 = the low 29 bits of the call's tag, bits 31..0 = value (payload
// words: a stream has fewer than 2^32).  Word 1: the call's tag.  A descriptor counts only
// when both words carry the reader's tag; anything else is an empty descriptor, so nothing has
// to be cleared before a call.  A reader that catches one new and one old word sees a
// mismatch and polls again.
// Only the descriptor itself is communicated, so relaxed device-scope atomics suffice.
// ---------------------------------------------------------------------------------------
constexpr u64 kDescAggregate = u64(1) << 62;
constexpr u64 kDescChain = u64(2) << 62;
constexpr u64 kDescWide = u64(1) << 61;
constexpr u64 kDescValueMask = (u64(1) << 32) - 1;
constexpr u64 kDescTagMask = ((u64(1) << 29) - 1) << 32;

// Descriptors are polled by every tile in flight, so neighbours must not share a memory
// line (polls of one line queue up behind each other): one descriptor per 128 bytes.
constexpr int kDescStride = 16;            // in u64

// Both words travel in one 16-byte access (a hot line serves its requests one after the other,
// so a second access per poll or publication would double the time the look-back chain takes),
// device-coherent (sc1).  Nothing depends on that access being indivisible: torn halves fail
// the tag check above.
__device__ inline __amdgpu_buffer_rsrc_t desc_resource(const u64* desc) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<u64*>(desc), 0, 0x7fffffff, 0x00020000);
}
constexpr int kCoherentAccess = 16;        // cache policy bits of the buffer builtins: sc1

// v = state | wide mark | value.
__device__ inline void desc_store(u64* desc, u32 tile, u64 v, u64 tag) {
  const u64 a = v | ((tag << 32) & kDescTagMask);
  const u32x4_t words = {u32(a), u32(a >> 32), u32(tag), u32(tag >> 32)};
  __builtin_amdgcn_raw_buffer_store_b128(words, desc_resource(desc), tile * u32(kDescStride * 8), 0, kCoherentAccess);
}

// LDS of one wave: 32 rows (blocks) of 32 codes + 4 words of padding, which keeps the 128-bit
// row reads of 16 consecutive lanes on distinct banks.  A wave's 64 blocks pass through it in
// two halves (blocks of lanes 0..31, then 32..63): codes or reconstructed values on one side,
// packed payload on the other, so that five or more workgroups fit a compute unit.
constexpr int kStageRow = 36;
constexpr int kWaveStage = 32 * kStageRow;              // 1152 words = 4.5 KiB per wave
static_assert(kWaveStage >= 32 * 33, "one half-wave of worst-case blocks must fit the staging area");

// Workgroup barrier that orders LDS accesses only: global loads and stores that are in flight
// stay in flight (a full __syncthreads waits for every outstanding vector memory operation).
__device__ inline void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------------------
// Look-back by chains.  The tiles of one residue class modulo kChains form a chain.  Workgroup
// ids go round the XCDs, so the tiles of a chain run on one XCD (tickets hand tiles out that way
// too), and what one of them publishes reaches the others through that XCD's L2.  A tile
//   1. publishes its size (state 1);
//   2. sums the sizes of its own chain's tiles before it, back to the nearest one that has
//      published a chain sum, reading the descriptors with scalar loads: they go from the scalar
//      cache (which the glc bit makes them miss) straight to L2 and do not queue behind the
//      compute unit's vector loads and stores, so that while the kernel streams one such round
//      trip takes about a third of a vector load's;
//   3. publishes its chain sum (state 2: the sizes of the chain's tiles up to and including it);
//   4. fetches, with device-coherent vector loads, one lane per chain, the newest descriptor of
//      each of the seven other chains: a chain sum ends that chain, a size sends the lane one tile
//      further back.  What lies before the tile is its own chain's exclusive sum plus, per other
//      chain, the nearest chain sum and the sizes after it.
// Against a look-back over the 32 nearest tiles (one lane each, walking back 32 at a time until a
// prefix shows up) this takes a fifth of the vector requests and is 10 % faster over the whole
// kernel on the 512^3 benchmark: every descriptor request waits in the same queue as the
// compute unit's streaming loads and stores, and makes them wait.
// Scalar loads see the XCD's L2, not the other XCDs': if a chain's tiles do not share an XCD
// (a launch of one tile, a workgroup that helps out another XCD's ticket counter), the scalar
// polls may never see the predecessor; after kLocalPolls of them without progress the tile
// reads its own chain the way it reads the others.  Every wait is bounded (kSpinLimit) and
// raises ZC_ERR_HIP in *status when the bound is hit; a tile below `tile` is in work on a
// resident workgroup (or done) and publishes without waiting for anything, so the waits end.
// ---------------------------------------------------------------------------------------
constexpr int kChains = 8;
static_assert(kTicketShards % kChains == 0, "tickets hand out the tiles of a chain on one XCD");
constexpr u32 kLocalPolls = 16;
constexpr u32 kOwnChain = 1u << (kChains - 1);               // lane 7: the chain of tile - 8, the tile's own
constexpr u32 kOtherChains = kOwnChain - 1u;                 // lanes 0..6: the chains of tile - 1 .. tile - 7

// state | wide mark | value of a descriptor as loaded (four 32-bit words); 0 (empty) unless it is of this call.
__device__ inline u64 desc_decode(const u32x4_t& w, u64 tag) {
  const u64 v = u64(w.x) | (u64(w.y) << 32);
  const u64 t = u64(w.z) | (u64(w.w) << 32);
  return (t == tag && (v & kDescTagMask) == ((tag << 32) & kDescTagMask)) ? (v & ~kDescTagMask) : 0ull;
}
__device__ inline u64 desc_load(const u64* desc, u32 tile, u64 tag) {
  return desc_decode(__builtin_amdgcn_raw_buffer_load_b128(desc_resource(desc), tile * u32(kDescStride * 8), 0, kCoherentAccess), tag);
}

// Exclusive sum of the chain of `tile` (tile >= kChains) by scalar loads, two descriptors a round
// (both loads and the wait for them in one statement: the compiler does not track what inline
// assembly has in flight).  False when kLocalPolls rounds in a row found nothing new.
// Uniform values throughout.
__device__ inline bool own_chain_scalar(const u64* desc, u32 tile, u64 tag, u32& sum, u64& wide) {
  i64 look = i64(tile) - kChains;
  u32 idle = 0;
  sum = 0;
  wide = 0;
  while (look >= 0) {
    const i64 next = look - kChains;
    const u64 a0 = uniform64(reinterpret_cast<u64>(desc + u64(look) * kDescStride));
    const u64 a1 = uniform64(reinterpret_cast<u64>(desc + u64(next >= 0 ? next : look) * kDescStride));
    u32x4_t w0, w1;
    asm volatile(
        "s_load_dwordx4 %0, %2, 0x0 glc\n\t"
        "s_load_dwordx4 %1, %3, 0x0 glc\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(w0), "=&s"(w1)
        : "s"(a0), "s"(a1)
        : "memory");
    const u64 d0 = desc_decode(w0, tag), d1 = desc_decode(w1, tag);
    const u32 s0 = u32(d0 >> 62), s1 = u32(d1 >> 62);
    if (s0 == 1 || s0 == 2) {
      sum += u32(d0);
      wide |= d0 & kDescWide;
      if (s0 == 2 || next < 0) return true;
      look = next;
      idle = 0;
      if (s1 == 1 || s1 == 2) {
        sum += u32(d1);
        wide |= d1 & kDescWide;
        if (s1 == 2) return true;
        look = next - kChains;
      }
    } else {
      if (++idle > kLocalPolls) return false;
      __builtin_amdgcn_s_sleep(1);
    }
  }
  return true;
}

// Called by all 64 lanes of one wave.  Sum over the chains in `chains` (bit c = the chain of tile
// - 1 - c, read by lane c) of the sizes of their tiles below `tile`, modulo 2^32 (a stream has
// fewer payload words than that), with kDescWide set if one of those tiles has it set.
__device__ inline u64 chains_lookback(const u64* desc, u32 tile, Control* ctl, u64 tag, u32 chains) {
  const int lane = lane_id();
  bool live = lane < kChains && ((chains >> lane) & 1u) != 0;
  i64 head = i64(tile) - 1 - lane;            // the tile this lane inspects
  live = live && head >= 0;                   // nothing before tile 0
  u32 total = 0;
  bool wide = false;
  u32 spins = 0;
  while (__ballot(live)) {
    u64 d = 0;
    if (live) d = desc_load(desc, u32(head), tag);
    const u32 state = u32(d >> 62);
    const bool there = state == 1 || state == 2;
    if (live && there) {
      total += u32(d);
      wide = wide || (d & kDescWide) != 0;
      head -= kChains;                         // a size: on to the tile before it in the chain
      live = state == 1 && head >= 0;
    }
    if (__ballot(live && !there)) {
      // give up after kSpinLimit polls, or as soon as another tile has given up
      const bool lost = (++spins & 1023u) == 0 && (status_bits(ctl, tag) & status_bit(ZC_ERR_HIP)) != 0;
      if (spins > kSpinLimit || lost) {
        if (lane == 0) raise_status(ctl, tag, status_bit(ZC_ERR_HIP));
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  }
  return u64(wave_sum_u32(total)) | (__ballot(wide) ? kDescWide : 0);
}

}  // namespace zc

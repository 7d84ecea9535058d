// C ABI of the zc library: argument checks and kernel launches.  All arithmetic of the
// method runs in the kernels; the host only divides once (1 / step) and launches.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <chrono>
#include <cmath>
#include <limits>
#include <cstring>
#include <mutex>
#include <vector>

#include "zc_common.h"
#include "zc_compress.h"
#include "zc_decompress.h"
#include "zc_reduce.h"
#include "zc_reduce_op.h"
#include "zc_scan.h"
#include "zc_quality.h"
#include "zc_step.h"
#include "zc_stream_probe.h"

using namespace zc;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool eb_valid(float eb) { return std::isfinite(eb) && eb >= std::ldexp(1.0f, -96); }

// Highest-precedence error in a device status word.
int status_from_bits(u32 bits) {
  static const int order[] = {ZC_ERR_HIP, ZC_ERR_ARG, ZC_ERR_FORMAT, ZC_ERR_MISMATCH, ZC_ERR_NONFINITE,
                              ZC_ERR_RANGE, ZC_ERR_CAPACITY, ZC_ERR_BOUND};
  for (int code : order)
    if (bits & status_bit(code)) return code;
  return ZC_OK;
}

bool launch_ok() { return hipGetLastError() == hipSuccess; }

// Optional timing of the main kernel of each entry point (zc_profile_*): host-side state only.
struct KernelTimer {
  std::mutex mu;
  unsigned kinds = 0;       // bit ZC_KERNEL_x set: the main kernels of that kind are timed
  struct Slot { hipEvent_t a, b; int kind; };
  std::vector<Slot> pool;   // events are created once and reused
  size_t used = 0;
  // A pair of events for one launch (by value: the pool may grow under another thread); false when timing is off.
  bool take(int kind, Slot& out) {
    std::lock_guard<std::mutex> g(mu);
    if (!(kinds & (1u << kind))) return false;
    if (used == pool.size()) {
      Slot s;
      s.kind = 0;
      if (hipEventCreate(&s.a) != hipSuccess) return false;
      if (hipEventCreate(&s.b) != hipSuccess) { (void)hipEventDestroy(s.a); return false; }
      pool.push_back(s);
    }
    pool[used].kind = kind;
    out = pool[used++];
    return true;
  }
};
KernelTimer g_timer;

// Launch of an entry point's main kernel.  When timing is on the two events are handed to the
// launch itself, which stamps them with the kernel's own start and end on its stream: no
// separate event records, which would each hold back the launch behind them.
template <typename... Args>
void launch_main(int kind, void (*kernel)(Args...), dim3 grid, dim3 block, hipStream_t stream, Args... args) {
  KernelTimer::Slot slot;
  if (g_timer.take(kind, slot)) hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, slot.a, slot.b, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, 0, stream, args...);
}

bool flags_valid(unsigned flags) { return (flags & ~(ZC_STREAM_PLAIN | ZC_TILES_BY_TICKET | ZC_CHAINS_COHERENT)) == 0; }
bool is_indexed(unsigned flags) { return (flags & ZC_STREAM_PLAIN) == 0; }

// A number per call for its tag (see launch_tag): the host's monotonic clock.  One workspace
// serves one call at a time, and two calls are never issued within the same nanosecond.
u64 call_nonce() { return u64(std::chrono::steady_clock::now().time_since_epoch().count()); }

// Most blocks a stream of `bytes` bytes can describe: each costs at least 5 table bytes.
u64 blocks_bound(u64 bytes) { return bytes > kHeaderBytes ? (bytes - kHeaderBytes) / 5 : 0; }

// Workgroups of stream_index_kernel per stream: 16 tiles make a scan group.
u32 index_grid(u64 tiles) { return u32(((tiles + 15) / 16 + kIndexGroups - 1) / kIndexGroups); }   // spans

int finish(const void* d_ws, size_t* result, hipStream_t stream) {
  struct { u64 status, call_tag, result; } host;
  if (hipMemcpyAsync(&host, d_ws, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess) return ZC_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return ZC_ERR_HIP;
  if (result) *result = size_t(host.result);
  // status bits count only under the tag of the last call
  return status_from_bits((host.status >> 32) == (host.call_tag >> 32) ? u32(host.status) : 0u);
}

// Validation and block positions of plain input streams, ahead of the kernel that reads them
// (indexed streams bring their positions along and are judged by that kernel itself).
// `tiles`: enough for the largest stream.  index_prep_kernel opens the call: the main kernel
// adopts the tag it leaves in the control block.
void launch_plain_index(ScanArgs& sa, u64 tiles, hipStream_t stream) {
  hipLaunchKernelGGL(stream_index_kernel, dim3(index_grid(tiles), u32(sa.k)), dim3(256), 0, stream, sa);
  hipLaunchKernelGGL(index_prep_kernel, dim3(1), dim3(256), 0, stream, sa);
}

// Tiles that a stream of in_bytes bytes can have, as far as the workspace goes.
u64 tiles_of_stream(u64 in_bytes, const WorkspaceLayout& l, bool ix) {
  u64 tiles = num_tiles(blocks_bound(in_bytes));
  if (!ix && tiles > l.tiles_cap) tiles = l.tiles_cap;
  if (tiles > kMaxTiles) tiles = kMaxTiles;
  return tiles < 1 ? 1 : tiles;
}

struct QuantizeArgs {
  CompressArgs c;
  i32* q;
};

__global__ void quantize_kernel(QuantizeArgs a) {
  const u64 tag = call_tag(a.c.ctl, launch_tag(a.c.nonce, a.c.ctl), false);
  const u64 i = u64(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= a.c.n) return;
  u32 err = 0;
  a.q[i] = quantize_value(a.c.in[i], a.c, err);
  if (err) raise_status(a.c.ctl, tag, err);
}

struct OffsetsArgs {
  StreamRef in;
  StreamIndex index;
  u32* off_words;
  u64 off_cap;
  Control* ctl;
  u64 nonce;
  bool ix;
};

__global__ __launch_bounds__(256) void block_offsets_kernel(OffsetsArgs a) {
  const ParsedHeader h = parse_header(a.in, a.ix);
  u64 tag;
  if (a.ix) {
    tag = call_tag(a.ctl, launch_tag(a.nonce, a.ctl), false);
    if (!h.ok) {
      if (blockIdx.x == 0 && threadIdx.x == 0) raise_status(a.ctl, tag, status_bit(ZC_ERR_FORMAT));
      return;
    }
  } else {
    const Gate gate = parse_gate(load_gate(a.ctl, 0));
    tag = gate.tag;
    if (gate_failed(gate) || !h.ok) return;
  }
  if (h.nb > a.off_cap) {
    if (blockIdx.x == 0 && threadIdx.x == 0) raise_status(a.ctl, tag, status_bit(ZC_ERR_CAPACITY));
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) a.ctl->result = h.nb;
  const u64 seg = u64(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (seg >= num_segments(h.nb) || (!a.ix && seg >= 4 * a.index.tiles_cap)) return;
  const u64 b = seg * kWaveBlocks + u64(lane_id());
  const u32 w = b < h.nb ? u32(a.in.base[widths_begin(h.nb, a.ix) + b]) : 0u;
  const u32 words = psize_words(w);
  const u32 incl = wave_inclusive_sum(words);
  const u32 seg_off = a.ix ? reinterpret_cast<const u32*>(a.in.base + kHeaderBytes)[seg] : u32(segment_offset(a.index, 0, seg));
  if (b < h.nb) a.off_words[b] = seg_off + incl - words;
}

void fill_compress_args(CompressArgs& ca, const float* d_in, u64 n, float abs_eb, void* d_out, u64 out_cap,
                        const WorkspaceLayout& l, unsigned flags) {
  ca.in = d_in;
  ca.n = n;
  ca.nb = num_blocks(n);
  ca.step = double(abs_eb) * 63.0 / 32.0;
  ca.inv = 1.0 / ca.step;
  ca.eb = double(abs_eb);
  ca.screen = std::fmin(abs_eb * 131072.0f, std::numeric_limits<float>::max());   // 2^17 * eb, kept finite: an infinite input must fail the screen
  std::memcpy(&ca.eb_bits, &abs_eb, 4);
  ca.out = static_cast<u8*>(d_out);
  ca.out_cap = out_cap;
  ca.ctl = l.ctl;
  ca.desc = l.desc;
  ca.ticketed = (flags & ZC_TILES_BY_TICKET) != 0;
  ca.coherent = (flags & ZC_CHAINS_COHERENT) != 0;
  ca.ix = is_indexed(flags);
  ca.part_end = 0;
  ca.adopt = 0;
  ca.nonce = call_nonce();
}

// The launches of zc_compress / zc_compress_part over the tiles [first_tile, end_tile) of the stream.
// `adopt`: the call continues one whose tag is in the control block (a later part).
void launch_compress(CompressArgs& ca, u32 first_tile, u32 end_tile, bool timed, hipStream_t stream) {
  const u32 ntiles = u32(num_pack_tiles(ca.nb));
  const u32 full_tiles = u32(ca.n / kPackValues);                       // tiles whose values all exist
  const u32 end_full = end_tile < full_tiles ? end_tile : full_tiles;
  if (ca.nb == 0) {                                                     // the stream of no values
    EmptyStreamArgs ea{ca.ctl, ca.out, ca.out_cap, ca.eb_bits, ca.ix, ca.nonce};
    hipLaunchKernelGGL(empty_stream_kernel, dim3(1), dim3(64), 0, stream, ea);
    return;
  }
  if (end_full > first_tile) {
    if (timed)
      launch_main(ZC_KERNEL_COMPRESS, compress_kernel<true>, dim3(end_full - first_tile), dim3(kPackThreads), stream, ca, first_tile, end_full);
    else
      hipLaunchKernelGGL(compress_kernel<true>, dim3(end_full - first_tile), dim3(kPackThreads), 0, stream, ca, first_tile, end_full);
    ca.adopt = 1;
  }
  if (end_tile > full_tiles)                                            // the ragged last tile of the stream
    hipLaunchKernelGGL(compress_kernel<false>, dim3(1), dim3(kPackThreads), 0, stream, ca, full_tiles, ntiles);
}

// Workspace of zc_compress_noalloc: a device array of the library itself, one copy per GPU,
// held until the process ends.  Host code never uses the array's name as an address (there it
// is only a stand-in for the symbol): the device address is asked for once per device and kept.
constexpr u64 kScratchBytes = (workspace_bytes(ZC_NOALLOC_MAX_N, 1) + 255) / 256 * 256;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, or null when it cannot be had.
void* scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);      // every thread finds the same address
  }
  return p;
}

}  // namespace

namespace {
template <int OP>
void (*pick_step_kernel(bool ix, bool tickets))(StepArgs) {
  if (ix) return tickets ? step_kernel<true, OP, true> : step_kernel<true, OP, false>;
  return tickets ? step_kernel<false, OP, true> : step_kernel<false, OP, false>;
}
}  // namespace

extern "C" {

size_t zc_compress_bound_ex(size_t n, unsigned flags) {
  const u64 nb = num_blocks(n);
  return size_t(tables_end(nb, is_indexed(flags)) + 128 * nb);
}

size_t zc_compress_bound(size_t n) { return zc_compress_bound_ex(n, 0); }

size_t zc_workspace_bytes(size_t n_max, int k_max) { return size_t(workspace_bytes(n_max, k_max)); }

const char* zc_strerror(int status) {
  switch (status) {
    case ZC_OK: return "ok";
    case ZC_ERR_ARG: return "invalid argument";
    case ZC_ERR_CAPACITY: return "output buffer too small";
    case ZC_ERR_FORMAT: return "not a valid zc stream";
    case ZC_ERR_NONFINITE: return "NaN or Inf in the input";
    case ZC_ERR_RANGE: return "quantisation code out of range";
    case ZC_ERR_BOUND: return "error bound not met (input outside the guaranteed domain)";
    case ZC_ERR_MISMATCH: return "reduce operands differ in size or error bound";
    case ZC_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int zc_finish(const void* d_ws, size_t* result, void* hip_stream) {
  if (!d_ws) d_ws = scratch_of_current_device();     // the call to complete was zc_compress_noalloc
  if (!d_ws) return ZC_ERR_HIP;
  return finish(d_ws, result, static_cast<hipStream_t>(hip_stream));
}

int zc_compress_ex(const float* d_in, size_t n, float abs_eb, void* d_out, size_t out_cap, size_t* out_bytes,
                   void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!flags_valid(flags) || !eb_valid(abs_eb) || n > ZC_MAX_N || (n && !d_in) || !d_out || !d_ws) return ZC_ERR_ARG;
  if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_ws)) return ZC_ERR_ARG;
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  const u64 nb = num_blocks(n);
  if (l.tiles_cap < 1 || num_tiles(nb) > l.tiles_cap) return ZC_ERR_ARG;
  CompressArgs ca;
  fill_compress_args(ca, d_in, n, abs_eb, d_out, out_cap, l, flags);
  launch_compress(ca, 0, u32(num_pack_tiles(nb)), true, stream);
  if (!launch_ok()) return ZC_ERR_HIP;
  if (!out_bytes) return ZC_OK;
  return finish(d_ws, out_bytes, stream);
}

int zc_compress(const float* d_in, size_t n, float abs_eb, void* d_out, size_t out_cap, size_t* out_bytes,
                void* d_ws, size_t ws_bytes, void* hip_stream) {
  return zc_compress_ex(d_in, n, abs_eb, d_out, out_cap, out_bytes, d_ws, ws_bytes, hip_stream, 0);
}

int zc_compress_noalloc(const float* d_in, size_t n, float abs_eb, void* d_out, size_t out_cap, size_t* out_bytes,
                        void* hip_stream) {
  if (n > ZC_NOALLOC_MAX_N) return ZC_ERR_ARG;       // the static workspace is sized for that many values
  void* ws = scratch_of_current_device();
  if (!ws) return ZC_ERR_HIP;
  // nothing in a workspace needs clearing (every call tags what it shares), so what the
  // previous call left in the array does not matter
  return zc_compress_ex(d_in, n, abs_eb, d_out, out_cap, out_bytes, ws, kScratchBytes, hip_stream, 0);
}

int zc_compress_part(const float* d_in, size_t n, float abs_eb, size_t first_value, size_t count, void* d_out,
                     size_t out_cap, size_t* out_bytes, void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!flags_valid(flags) || !eb_valid(abs_eb) || n > ZC_MAX_N || (n && !d_in) || !d_out || !d_ws) return ZC_ERR_ARG;
  if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_ws)) return ZC_ERR_ARG;
  if (first_value > n || count > n - first_value || first_value % kPackValues != 0) return ZC_ERR_ARG;
  const bool to_the_end = first_value + count == n;
  if (!to_the_end && count % kPackValues != 0) return ZC_ERR_ARG;
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  const u64 nb = num_blocks(n);
  const u64 ntiles = num_pack_tiles(nb);
  if (l.tiles_cap < 1 || num_tiles(nb) > l.tiles_cap) return ZC_ERR_ARG;
  CompressArgs ca;
  fill_compress_args(ca, d_in, n, abs_eb, d_out, out_cap, l, flags);
  const u32 first_tile = u32(first_value / kPackValues);
  const u32 end_tile = to_the_end ? u32(ntiles) : u32((first_value + count) / kPackValues);
  ca.part_end = end_tile;
  ca.adopt = first_value != 0;          // later parts belong to the call that the first part opened
  if (end_tile > first_tile || nb == 0) launch_compress(ca, first_tile, end_tile, false, stream);
  if (!launch_ok()) return ZC_ERR_HIP;
  if (!out_bytes) return ZC_OK;
  return finish(d_ws, out_bytes, stream);
}

// zc_decompress, zc_decompress_average, zc_decompress_range.
static int decompress_one(const void* d_in, size_t in_bytes, size_t first_value, size_t count, bool ranged, float* d_out,
                          size_t out_cap_elems, size_t* n_out, void* d_ws, size_t ws_bytes, void* hip_stream, bool average,
                          unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  constexpr u64 kSegValues = u64(kWaveBlocks) * kBlockValues;
  if ((flags & ~ZC_STREAM_PLAIN) != 0 || !d_in || !d_ws || (out_cap_elems && !d_out)) return ZC_ERR_ARG;
  if (first_value % kSegValues != 0 || first_value > ZC_MAX_N) return ZC_ERR_ARG;
  if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_ws)) return ZC_ERR_ARG;
  if (in_bytes < kHeaderBytes) return ZC_ERR_FORMAT;
  const bool ix = is_indexed(flags);
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  if (l.tiles_cap < 1) return ZC_ERR_ARG;
  // Tiles of the main kernel: no more than the buffers allow.  (The index of a plain stream is
  // built over the whole stream whatever the output's size: its sums validate total_bytes.)
  u64 wanted = count < out_cap_elems ? count : out_cap_elems;
  const u64 stream_bound = blocks_bound(in_bytes) * kBlockValues;
  if (wanted > stream_bound) wanted = stream_bound;
  u64 grid = (wanted + kTileValues - 1) / kTileValues;
  if (!ix && grid > l.tiles_cap) grid = l.tiles_cap;
  if (grid > kMaxTiles) grid = kMaxTiles;
  if (grid < 1) grid = 1;
  const u64 nonce = call_nonce();
  if (!ix) {
    ScanArgs sa;
    sa.streams[0].base = static_cast<const u8*>(d_in);
    sa.streams[0].bytes = in_bytes;
    sa.k = 1;
    sa.check_match = 0;
    sa.index = l.index;
    sa.ctl = l.ctl;
    sa.nonce = nonce;
    launch_plain_index(sa, tiles_of_stream(in_bytes, l, false), stream);
  }
  DecompressArgs da;
  da.in.base = static_cast<const u8*>(d_in);
  da.in.bytes = in_bytes;
  da.out = d_out;
  da.out_cap_elems = out_cap_elems;
  da.index = l.index;
  da.ctl = l.ctl;
  da.first_value = first_value;
  da.count = count;
  da.nonce = nonce;
  if (ranged) {
    hipLaunchKernelGGL(ix ? decompress_range_kernel<true> : decompress_range_kernel<false>, dim3(u32(grid)),
                       dim3(kTileThreads), 0, stream, da);
  } else {
    void (*kernel)(DecompressArgs) = average ? (ix ? decompress_kernel<true, true> : decompress_kernel<false, true>)
                                             : (ix ? decompress_kernel<true, false> : decompress_kernel<false, false>);
    launch_main(ZC_KERNEL_DECOMPRESS, kernel, dim3(u32(grid)), dim3(kTileThreads), stream, da);
  }
  if (!launch_ok()) return ZC_ERR_HIP;
  if (!n_out) return ZC_OK;
  return finish(d_ws, n_out, stream);
}

int zc_decompress_ex(const void* d_in, size_t in_bytes, float* d_out, size_t out_cap_elems, size_t* n_out,
                     void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  return decompress_one(d_in, in_bytes, 0, ~size_t(0), false, d_out, out_cap_elems, n_out, d_ws, ws_bytes, hip_stream, false, flags);
}

int zc_decompress(const void* d_in, size_t in_bytes, float* d_out, size_t out_cap_elems, size_t* n_out,
                  void* d_ws, size_t ws_bytes, void* hip_stream) {
  return zc_decompress_ex(d_in, in_bytes, d_out, out_cap_elems, n_out, d_ws, ws_bytes, hip_stream, 0);
}

int zc_decompress_average(const void* d_in, size_t in_bytes, float* d_out, size_t out_cap_elems, size_t* n_out,
                          void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  return decompress_one(d_in, in_bytes, 0, ~size_t(0), false, d_out, out_cap_elems, n_out, d_ws, ws_bytes, hip_stream, true, flags);
}

int zc_decompress_range(const void* d_in, size_t in_bytes, size_t first_value, size_t count, float* d_out,
                        size_t out_cap_elems, size_t* n_out, void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  return decompress_one(d_in, in_bytes, first_value, count, true, d_out, out_cap_elems, n_out, d_ws, ws_bytes, hip_stream, false,
                        flags);
}

int zc_decompress_many(const void* const* d_chunks, const size_t* chunk_bytes, int k, float* const* d_outs,
                       const size_t* out_cap_elems, size_t* n_out, void* d_ws, size_t ws_bytes, void* hip_stream,
                       unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if ((flags & ~ZC_STREAM_PLAIN) != 0) return ZC_ERR_ARG;
  if (k < 1 || k > ZC_MAX_K || !d_chunks || !chunk_bytes || !d_outs || !out_cap_elems || !d_ws) return ZC_ERR_ARG;
  if (!aligned16(d_ws)) return ZC_ERR_ARG;
  for (int i = 0; i < k; ++i)
    if (!d_chunks[i] || !aligned16(d_chunks[i]) || !aligned16(d_outs[i]) || (out_cap_elems[i] && !d_outs[i])) return ZC_ERR_ARG;
  for (int i = 0; i < k; ++i)
    if (chunk_bytes[i] < kHeaderBytes) return ZC_ERR_FORMAT;
  const bool ix = is_indexed(flags);
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, k);
  if (l.tiles_cap < 1) return ZC_ERR_ARG;
  ScanArgs sa;
  DecompressManyArgs da;
  u64 tiles = 1, tiles_in = 1;
  for (int i = 0; i < k; ++i) {
    sa.streams[i].base = static_cast<const u8*>(d_chunks[i]);
    sa.streams[i].bytes = chunk_bytes[i];
    da.in[i] = sa.streams[i];
    da.out[i] = d_outs[i];
    da.out_cap_elems[i] = out_cap_elems[i];
    const u64 t_in = tiles_of_stream(chunk_bytes[i], l, ix);
    const u64 t_out = num_tiles(num_blocks(out_cap_elems[i]));
    const u64 t = t_in < t_out ? t_in : t_out;
    if (t > tiles) tiles = t;
    if (t_in > tiles_in) tiles_in = t_in;
  }
  const u64 nonce = call_nonce();
  if (!ix) {
    sa.k = k;
    sa.check_match = 0;
    sa.index = l.index;
    sa.ctl = l.ctl;
    sa.nonce = nonce;
    launch_plain_index(sa, tiles_in, stream);
  }
  da.k = k;
  da.index = l.index;
  da.ctl = l.ctl;
  da.nonce = nonce;
  void (*kernel)(DecompressManyArgs) = ix ? decompress_many_kernel<true> : decompress_many_kernel<false>;
  launch_main(ZC_KERNEL_DECOMPRESS, kernel, dim3(u32(tiles), u32(k)), dim3(kTileThreads), stream, da);
  if (!launch_ok()) return ZC_ERR_HIP;
  if (!n_out) return ZC_OK;
  // every header that passes validation holds its stream's n: fetch them along with the status
  u64 ns[ZC_MAX_K];
  for (int i = 0; i < k; ++i)
    if (hipMemcpyAsync(&ns[i], static_cast<const u8*>(d_chunks[i]) + 8, 8, hipMemcpyDeviceToHost, stream) != hipSuccess)
      return ZC_ERR_HIP;
  size_t total = 0;
  const int st = finish(d_ws, &total, stream);
  if (st == ZC_ERR_HIP || st == ZC_ERR_ARG || st == ZC_ERR_FORMAT) return st;
  for (int i = 0; i < k; ++i) n_out[i] = size_t(ns[i]);
  return st;
}

// zc_reduce_compressed_op and zc_reduce_compressed_part.  ranged: the values [first_value, first_value + count)
// of streams of n values, as one part of a reduce done in parts.
static int reduce_impl(const void* const* d_chunks, const size_t* chunk_bytes, int k, int op, bool ranged, size_t n,
                       size_t first_value, size_t count, void* d_out, size_t out_cap, size_t* out_bytes, void* d_ws,
                       size_t ws_bytes, void* hip_stream, unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!flags_valid(flags) || (op != ZC_OP_SUM && op != ZC_OP_MAX && op != ZC_OP_MIN)) return ZC_ERR_ARG;
  if (k < 1 || k > ZC_MAX_K || !d_chunks || !chunk_bytes || !d_out || !d_ws) return ZC_ERR_ARG;
  if (!aligned16(d_out) || !aligned16(d_ws)) return ZC_ERR_ARG;
  for (int i = 0; i < k; ++i)
    if (!d_chunks[i] || !aligned16(d_chunks[i])) return ZC_ERR_ARG;
  for (int i = 0; i < k; ++i)
    if (chunk_bytes[i] < kHeaderBytes) return ZC_ERR_FORMAT;
  const bool ix = is_indexed(flags);
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, k);
  if (l.tiles_cap < 1) return ZC_ERR_ARG;
  // the output's tiles need a look-back descriptor each, whatever the variant
  u64 tiles = l.tiles_cap, tiles_in = 1;
  for (int i = 0; i < k; ++i) {
    const u64 t = num_tiles(blocks_bound(chunk_bytes[i]));
    if (t < tiles) tiles = t;
    if (t > tiles_in) tiles_in = t;
  }
  if (tiles > kMaxTiles) tiles = kMaxTiles;
  if (tiles < 1) tiles = 1;
  if (tiles_in > l.tiles_cap) tiles_in = l.tiles_cap;
  ScanArgs sa;
  ReduceArgs ra;
  for (int i = 0; i < k; ++i) {
    sa.streams[i].base = static_cast<const u8*>(d_chunks[i]);
    sa.streams[i].bytes = chunk_bytes[i];
    ra.in[i] = sa.streams[i];
  }
  const u64 nonce = call_nonce();
  if (!ix) {
    sa.k = k;
    sa.check_match = 1;
    sa.index = l.index;
    sa.ctl = l.ctl;
    sa.nonce = nonce;
    launch_plain_index(sa, tiles_in, stream);
  }
  ra.k = k;
  ra.index = l.index;
  ra.out = static_cast<u8*>(d_out);
  ra.out_cap = out_cap;
  ra.ctl = l.ctl;
  ra.desc = l.desc;
  ra.ticketed = (flags & ZC_TILES_BY_TICKET) != 0;
  ra.coherent = (flags & ZC_CHAINS_COHERENT) != 0;
  ra.nonce = nonce;
  ra.first_tile = ra.end_tile = ra.adopt = 0;
  ra.n_part = 0;
  if (ranged) {
    // parts are laid out in tiles of the reduce kernel; only indexed streams can be taken up in parts
    if (!ix || op != ZC_OP_SUM || n > ZC_MAX_N || n == 0 || first_value % kTileValues != 0 || first_value >= n ||
        count == 0 || count > n - first_value)
      return ZC_ERR_ARG;
    const bool to_the_end = first_value + count == n;
    if (!to_the_end && count % kTileValues != 0) return ZC_ERR_ARG;
    const u64 all_tiles = num_tiles(num_blocks(n));
    if (all_tiles > l.tiles_cap) return ZC_ERR_ARG;
    ra.first_tile = u32(first_value / kTileValues);
    ra.end_tile = to_the_end ? u32(all_tiles) : u32((first_value + count) / kTileValues);
    ra.adopt = first_value != 0;
    ra.n_part = n;
    tiles = ra.end_tile - ra.first_tile;
  }
  if (op == ZC_OP_SUM) {
    launch_main(ZC_KERNEL_REDUCE, ix ? reduce_kernel<true> : reduce_kernel<false>, dim3(u32(tiles)), dim3(kTileThreads), stream, ra);
    // plain streams with blocks wider than 15 bits have a kernel of their own, which returns at once otherwise
    if (!ix) hipLaunchKernelGGL(reduce_wide_kernel, dim3(u32(tiles)), dim3(kTileThreads), 0, stream, ra);
  } else {
    // Max and Min: a kernel for operands without blocks wider than 15 bits and one for the others;
    // each returns at once when the operands are not its
    void (*narrow)(ReduceArgs) = op == ZC_OP_MAX ? (ix ? reduce_op_kernel<true, ZC_OP_MAX> : reduce_op_kernel<false, ZC_OP_MAX>)
                                                 : (ix ? reduce_op_kernel<true, ZC_OP_MIN> : reduce_op_kernel<false, ZC_OP_MIN>);
    void (*wide)(ReduceArgs) = op == ZC_OP_MAX ? (ix ? reduce_op_wide_kernel<true, ZC_OP_MAX> : reduce_op_wide_kernel<false, ZC_OP_MAX>)
                                               : (ix ? reduce_op_wide_kernel<true, ZC_OP_MIN> : reduce_op_wide_kernel<false, ZC_OP_MIN>);
    launch_main(ZC_KERNEL_REDUCE, narrow, dim3(u32(tiles)), dim3(kTileThreads), stream, ra);
    hipLaunchKernelGGL(wide, dim3(u32(tiles)), dim3(kTileThreads), 0, stream, ra);
  }
  if (!launch_ok()) return ZC_ERR_HIP;
  if (!out_bytes) return ZC_OK;
  return finish(d_ws, out_bytes, stream);
}

int zc_reduce_compressed_op(const void* const* d_chunks, const size_t* chunk_bytes, int k, int op, void* d_out, size_t out_cap,
                            size_t* out_bytes, void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  return reduce_impl(d_chunks, chunk_bytes, k, op, false, 0, 0, 0, d_out, out_cap, out_bytes, d_ws, ws_bytes, hip_stream, flags);
}

int zc_reduce_compressed_ex(const void* const* d_chunks, const size_t* chunk_bytes, int k, void* d_out, size_t out_cap,
                            size_t* out_bytes, void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  return reduce_impl(d_chunks, chunk_bytes, k, ZC_OP_SUM, false, 0, 0, 0, d_out, out_cap, out_bytes, d_ws, ws_bytes, hip_stream,
                     flags);
}

int zc_reduce_compressed_part(const void* const* d_chunks, const size_t* chunk_bytes, int k, size_t n, size_t first_value,
                              size_t count, void* d_out, size_t out_cap, size_t* out_bytes, void* d_ws, size_t ws_bytes,
                              void* hip_stream, unsigned flags) {
  return reduce_impl(d_chunks, chunk_bytes, k, ZC_OP_SUM, true, n, first_value, count, d_out, out_cap, out_bytes, d_ws, ws_bytes,
                     hip_stream, flags);
}

int zc_reduce_compressed(const void* const* d_chunks, const size_t* chunk_bytes, int k, void* d_out, size_t out_cap,
                         size_t* out_bytes, void* d_ws, size_t ws_bytes, void* hip_stream) {
  return zc_reduce_compressed_ex(d_chunks, chunk_bytes, k, d_out, out_cap, out_bytes, d_ws, ws_bytes, hip_stream, 0);
}

static int step_impl(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, int op, bool ranged,
                     size_t first_value, size_t count, void* d_out, size_t out_cap, size_t* out_bytes, void* d_ws,
                     size_t ws_bytes, void* hip_stream, unsigned flags);

int zc_reduce_step(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, void* d_out,
                   size_t out_cap, size_t* out_bytes, void* d_ws, size_t ws_bytes, void* hip_stream) {
  return step_impl(d_chunk, chunk_bytes, d_local, n_local, ZC_OP_SUM, false, 0, 0, d_out, out_cap, out_bytes, d_ws, ws_bytes,
                   hip_stream, 0);
}

// zc_reduce_step_op and zc_reduce_step_part.
static int step_impl(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, int op, bool ranged,
                     size_t first_value, size_t count, void* d_out, size_t out_cap, size_t* out_bytes, void* d_ws,
                     size_t ws_bytes, void* hip_stream, unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!flags_valid(flags) || (op != ZC_OP_SUM && op != ZC_OP_MAX && op != ZC_OP_MIN)) return ZC_ERR_ARG;
  if (!d_chunk || !d_out || !d_ws || (n_local && !d_local) || n_local > ZC_MAX_N) return ZC_ERR_ARG;
  if (!aligned16(d_chunk) || !aligned16(d_local) || !aligned16(d_out) || !aligned16(d_ws)) return ZC_ERR_ARG;
  if (chunk_bytes < kHeaderBytes) return ZC_ERR_FORMAT;
  const bool ix = is_indexed(flags);
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  u64 tiles = num_tiles(num_blocks(n_local));
  if (l.tiles_cap < 1 || tiles > l.tiles_cap) return ZC_ERR_ARG;
  if (tiles < 1) tiles = 1;
  const u64 nonce = call_nonce();
  StepArgs ta;
  ta.in.base = static_cast<const u8*>(d_chunk);
  ta.in.bytes = chunk_bytes;
  if (!ix) {
    ScanArgs sa;
    sa.streams[0] = ta.in;
    sa.k = 1;
    sa.check_match = 0;
    sa.index = l.index;
    sa.ctl = l.ctl;
    sa.nonce = nonce;
    launch_plain_index(sa, tiles_of_stream(chunk_bytes, l, false), stream);
  }
  ta.local = d_local;
  ta.n_local = n_local;
  ta.index = l.index;
  ta.out = static_cast<u8*>(d_out);
  ta.out_cap = out_cap;
  ta.ctl = l.ctl;
  ta.desc = l.desc;
  ta.ticketed = (flags & ZC_TILES_BY_TICKET) != 0;
  ta.coherent = (flags & ZC_CHAINS_COHERENT) != 0;
  ta.nonce = nonce;
  ta.first_tile = ta.end_tile = ta.adopt = 0;
  if (ranged) {
    if (!ix || n_local == 0 || first_value % kTileValues != 0 || first_value >= n_local || count == 0 ||
        count > n_local - first_value)
      return ZC_ERR_ARG;
    const bool to_the_end = first_value + count == n_local;
    if (!to_the_end && count % kTileValues != 0) return ZC_ERR_ARG;
    ta.first_tile = u32(first_value / kTileValues);
    ta.end_tile = to_the_end ? u32(num_tiles(num_blocks(n_local))) : u32((first_value + count) / kTileValues);
    ta.adopt = first_value != 0;
    tiles = ta.end_tile - ta.first_tile;
  }
  void (*kernel)(StepArgs) = nullptr;
  const bool tickets = ta.ticketed != 0;
  if (op == ZC_OP_SUM) kernel = pick_step_kernel<ZC_OP_SUM>(ix, tickets);
  else if (op == ZC_OP_MAX) kernel = pick_step_kernel<ZC_OP_MAX>(ix, tickets);
  else kernel = pick_step_kernel<ZC_OP_MIN>(ix, tickets);
  launch_main(ZC_KERNEL_REDUCE_STEP, kernel, dim3(u32(tiles)), dim3(kTileThreads), stream, ta);
  if (!launch_ok()) return ZC_ERR_HIP;
  if (!out_bytes) return ZC_OK;
  return finish(d_ws, out_bytes, stream);
}

int zc_reduce_step_op(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, int op, void* d_out,
                      size_t out_cap, size_t* out_bytes, void* d_ws, size_t ws_bytes, void* hip_stream, unsigned flags) {
  return step_impl(d_chunk, chunk_bytes, d_local, n_local, op, false, 0, 0, d_out, out_cap, out_bytes, d_ws, ws_bytes, hip_stream,
                   flags);
}

int zc_reduce_step_part(const void* d_chunk, size_t chunk_bytes, const float* d_local, size_t n_local, int op,
                        size_t first_value, size_t count, void* d_out, size_t out_cap, size_t* out_bytes, void* d_ws,
                        size_t ws_bytes, void* hip_stream, unsigned flags) {
  return step_impl(d_chunk, chunk_bytes, d_local, n_local, op, true, first_value, count, d_out, out_cap, out_bytes, d_ws, ws_bytes,
                   hip_stream, flags);
}

int zc_quality(const float* d_ref, const float* d_test, size_t n, double* out4, void* d_ws, size_t ws_bytes,
               void* hip_stream) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!out4 || !d_ws || (n && (!d_ref || !d_test)) || n > ZC_MAX_N) return ZC_ERR_ARG;
  if (!aligned16(d_ref) || !aligned16(d_test) || !aligned16(d_ws)) return ZC_ERR_ARG;
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  if (l.tiles_cap < 1 || num_tiles(num_blocks(n)) > l.tiles_cap) return ZC_ERR_ARG;
  // partial results live where the other calls keep their tile descriptors: 128 bytes per tile
  u64 groups = l.tiles_cap * kDescBytes / sizeof(QualityPartial) - 1;
  const u64 wanted = (n / 4 + kQualityThreads - 1) / kQualityThreads;
  if (groups > wanted) groups = wanted;
  if (groups > 2048) groups = 2048;
  if (groups < 1) groups = 1;
  QualityArgs qa;
  qa.ref = d_ref;
  qa.test = d_test;
  qa.n = n;
  qa.partials = reinterpret_cast<QualityPartial*>(l.desc);
  hipLaunchKernelGGL(quality_partial_kernel, dim3(u32(groups)), dim3(kQualityThreads), 0, stream, qa);
  hipLaunchKernelGGL(quality_final_kernel, dim3(1), dim3(kQualityThreads), 0, stream, qa, u32(groups));
  if (!launch_ok()) return ZC_ERR_HIP;
  QualityPartial host;
  if (hipMemcpyAsync(&host, qa.partials + groups, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess) return ZC_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return ZC_ERR_HIP;
  out4[0] = host.worst;
  out4[1] = host.sse;
  out4[2] = host.lo;
  out4[3] = host.hi;
  return ZC_OK;
}

int zc_profile_enable(int on) {
  std::lock_guard<std::mutex> g(g_timer.mu);
  g_timer.kinds = on == 1 ? ~0u : unsigned(on) & ~1u;      // 1: every kind; else a set of (1 << ZC_KERNEL_x)
  g_timer.used = 0;
  return ZC_OK;
}

int zc_profile_collect(float* ms, int* kernel, int cap) {
  std::lock_guard<std::mutex> g(g_timer.mu);
  int count = 0;
  for (size_t i = 0; i < g_timer.used && count < cap; ++i) {
    KernelTimer::Slot& s = g_timer.pool[i];
    float t = 0.f;
    if (hipEventSynchronize(s.b) != hipSuccess || hipEventElapsedTime(&t, s.a, s.b) != hipSuccess) {
      g_timer.used = 0;
      return -ZC_ERR_HIP;
    }
    if (ms) ms[count] = t;
    if (kernel) kernel[count] = s.kind;
    ++count;
  }
  g_timer.used = 0;
  return count;
}

int zc_peek_header(const void* d_in, size_t in_bytes, size_t* n, float* abs_eb, unsigned* nsum,
                   size_t* total_bytes, unsigned* flags, void* hip_stream) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!d_in) return ZC_ERR_ARG;
  if (in_bytes < kHeaderBytes) return ZC_ERR_FORMAT;
  u32 w[8];
  if (hipMemcpyAsync(w, d_in, sizeof(w), hipMemcpyDeviceToHost, stream) != hipSuccess) return ZC_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return ZC_ERR_HIP;
  const u64 nn = u64(w[2]) | (u64(w[3]) << 32);
  const u64 total = u64(w[6]) | (u64(w[7]) << 32);
  float eb;
  std::memcpy(&eb, &w[4], 4);
  // the version word tells the variant
  const bool plain = w[1] == kVersionPlain, indexed = (w[1] | 1u) == (kVersionIndexed | 1u);
  if (w[0] != kMagic || !(plain || indexed) || nn > ZC_MAX_N || !eb_valid(eb) || w[5] < 1 || total > in_bytes ||
      total < tables_end(num_blocks(nn), indexed))
    return ZC_ERR_FORMAT;
  if (n) *n = size_t(nn);
  if (abs_eb) *abs_eb = eb;
  if (nsum) *nsum = w[5];
  if (total_bytes) *total_bytes = size_t(total);
  if (flags) *flags = plain ? ZC_STREAM_PLAIN : 0u;
  return ZC_OK;
}

int zc_debug_quantize(const float* d_in, size_t n, float abs_eb, int32_t* d_q, void* d_ws, size_t ws_bytes,
                      void* hip_stream) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (!eb_valid(abs_eb) || n > ZC_MAX_N || (n && (!d_in || !d_q)) || !d_ws || ws_bytes < sizeof(Control))
    return ZC_ERR_ARG;
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  QuantizeArgs qa;
  fill_compress_args(qa.c, d_in, n, abs_eb, nullptr, 0, l, 0);
  qa.q = d_q;
  // (at least one workgroup: the first one opens the call, which zc_finish reads back)
  hipLaunchKernelGGL(quantize_kernel, dim3(u32(n ? (n + 255) / 256 : 1)), dim3(256), 0, stream, qa);
  if (!launch_ok()) return ZC_ERR_HIP;
  return finish(d_ws, nullptr, stream);
}

int zc_debug_stream(const void* d_in, void* d_out, size_t tiles, int loads, int stores, void* hip_stream) {
  if (loads < 0 || stores < 0 || loads > kProbeMaxAccesses || stores > kProbeMaxAccesses || loads + stores == 0) return ZC_ERR_ARG;
  if ((loads && !d_in) || (stores && !d_out) || !aligned16(d_in) || !aligned16(d_out) || tiles > 0x7fffffffull) return ZC_ERR_ARG;
  if (tiles == 0) return ZC_OK;
  StreamProbeArgs pa{static_cast<const uint4*>(d_in), static_cast<uint4*>(d_out), u32(loads), u32(stores)};
  launch_main(ZC_KERNEL_STREAM, stream_probe_by_loads(loads), dim3(u32(tiles)), dim3(kProbeThreads), static_cast<hipStream_t>(hip_stream), pa);
  return launch_ok() ? ZC_OK : ZC_ERR_HIP;
}

int zc_debug_block_offsets(const void* d_in, size_t in_bytes, uint32_t* d_off_words, size_t off_cap, void* d_ws,
                           size_t ws_bytes, void* hip_stream, unsigned flags) {
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if ((flags & ~ZC_STREAM_PLAIN) != 0) return ZC_ERR_ARG;
  if (!d_in || !d_ws || (off_cap && !d_off_words) || !aligned16(d_in) || !aligned16(d_ws)) return ZC_ERR_ARG;
  if (in_bytes < kHeaderBytes) return ZC_ERR_FORMAT;
  const bool ix = is_indexed(flags);
  const WorkspaceLayout l = workspace_layout(d_ws, ws_bytes, 1);
  if (l.tiles_cap < 1) return ZC_ERR_ARG;
  const u64 tiles = tiles_of_stream(in_bytes, l, ix);
  const u64 nonce = call_nonce();
  if (!ix) {
    ScanArgs sa;
    sa.streams[0].base = static_cast<const u8*>(d_in);
    sa.streams[0].bytes = in_bytes;
    sa.k = 1;
    sa.check_match = 0;
    sa.index = l.index;
    sa.ctl = l.ctl;
    sa.nonce = nonce;
    launch_plain_index(sa, tiles, stream);
  }
  OffsetsArgs oa;
  oa.in.base = static_cast<const u8*>(d_in);
  oa.in.bytes = in_bytes;
  oa.index = l.index;
  oa.off_words = d_off_words;
  oa.off_cap = off_cap;
  oa.ctl = l.ctl;
  oa.nonce = nonce;
  oa.ix = ix;
  hipLaunchKernelGGL(block_offsets_kernel, dim3(u32(tiles)), dim3(256), 0, stream, oa);
  if (!launch_ok()) return ZC_ERR_HIP;
  return finish(d_ws, nullptr, stream);
}

}  // extern "C"

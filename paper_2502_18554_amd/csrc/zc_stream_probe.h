// A kernel that only streams, in the access shape of the codec's kernels: what the memory
// system gives a kernel of a given read : write mix that does nothing else (a measuring aid).
#pragma once

#include <utility>

#include "zc_common.h"

namespace zc {

constexpr int kProbeThreads = 512;
constexpr int kProbeMaxAccesses = 16;
constexpr u64 kProbeBytesPerAccess = u64(kProbeThreads) * 16;       // 8 KiB per workgroup and access

struct StreamProbeArgs {
  const uint4* in;
  uint4* out;
  u32 loads, stores;       // per lane
};

// LOADS is a template parameter so that the loads are unconditional and all go out before the first wait.
template <int LOADS>
__global__ __launch_bounds__(kProbeThreads) void stream_probe_kernel(StreamProbeArgs a) {
  const u64 t = blockIdx.x;
  uint4 x[LOADS ? LOADS : 1];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) x[i] = load_once(a.in + (t * LOADS + u32(i)) * kProbeThreads + threadIdx.x);
  u32x4_t v = {u32(threadIdx.x), u32(t), 0u, 0u};
#pragma unroll
  for (int i = 0; i < LOADS; ++i) v ^= u32x4_t{x[i].x, x[i].y, x[i].z, x[i].w};
  if (a.stores == 0) {
    // nothing is written: the loads stay alive through a store that never happens
    if (v.x == 0x9e3779b9u && v.y == 0x7f4a7c15u && v.z == 0xf39cc060u && v.w == 0x5cedc834u && a.out)
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(a.out));
    return;
  }
#pragma unroll
  for (int i = 0; i < kProbeMaxAccesses; ++i)
    if (u32(i) < a.stores)
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(a.out + (t * a.stores + u32(i)) * kProbeThreads + threadIdx.x));
}

using StreamProbeKernel = void (*)(StreamProbeArgs);
template <int... L>
inline StreamProbeKernel stream_probe_by_loads(int loads, std::integer_sequence<int, L...>) {
  static constexpr StreamProbeKernel table[] = {stream_probe_kernel<L>...};
  return table[loads];
}
inline StreamProbeKernel stream_probe_by_loads(int loads) {
  return stream_probe_by_loads(loads, std::make_integer_sequence<int, kProbeMaxAccesses + 1>{});
}

}  // namespace zc

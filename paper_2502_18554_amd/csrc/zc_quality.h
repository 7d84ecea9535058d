// Quality of a reconstruction against its original: the four sums from which the paper's
// quality figures follow (NRMSE in the compressor comparison of Section 3.3, PSNR and NRMSE
// of the stacked image in Section 4.6): max |ref - test|, sum of squared differences, min and
// max of ref, accumulated in binary64.
//
// Two kernels, both with a fixed order of accumulation, so that repeated runs give the same
// bits: workgroups stride over the input with 16-byte loads and leave one partial result
// each; one workgroup then folds the partials.  Pure streaming: 8 bytes per value.
#pragma once

#include "zc_common.h"

namespace zc {

struct QualityPartial {
  double worst, sse, lo, hi;
};

struct QualityArgs {
  const float* ref;
  const float* test;
  u64 n;
  QualityPartial* partials;      // gridDim.x entries, then the result
};

constexpr int kQualityThreads = 256;

__device__ inline void quality_take(QualityPartial& p, float r, float t) {
  const double d = double(r) - double(t);
  const double a = __builtin_fabs(d);
  if (a > p.worst || a != a) p.worst = a;       // a NaN difference is reported, not skipped
  p.sse = __dadd_rn(p.sse, __dmul_rn(d, d));
  const double rd = double(r);
  if (rd < p.lo) p.lo = rd;
  if (rd > p.hi) p.hi = rd;
}

__device__ inline void quality_fold(QualityPartial& p, const QualityPartial& o) {
  if (o.worst > p.worst || o.worst != o.worst) p.worst = o.worst;
  p.sse = __dadd_rn(p.sse, o.sse);
  if (o.lo < p.lo) p.lo = o.lo;
  if (o.hi > p.hi) p.hi = o.hi;
}

// Folds the partials of a workgroup's threads in a fixed tree; thread 0 returns the result.
__device__ inline QualityPartial quality_fold_workgroup(QualityPartial p, QualityPartial* sh) {
  sh[threadIdx.x] = p;
  __syncthreads();
  for (int half = kQualityThreads / 2; half > 0; half >>= 1) {
    if (int(threadIdx.x) < half) {
      QualityPartial a = sh[threadIdx.x];
      quality_fold(a, sh[threadIdx.x + half]);
      sh[threadIdx.x] = a;
    }
    __syncthreads();
  }
  return sh[0];
}

__global__ __launch_bounds__(kQualityThreads) void quality_partial_kernel(QualityArgs a) {
  __shared__ QualityPartial sh[kQualityThreads];
  QualityPartial p{0.0, 0.0, __builtin_inf(), -__builtin_inf()};
  const u64 quads = a.n / 4;
  const u64 stride = u64(gridDim.x) * kQualityThreads;
  for (u64 i = u64(blockIdx.x) * kQualityThreads + threadIdx.x; i < quads; i += stride) {
    const float4 r = load_once(reinterpret_cast<const float4*>(a.ref) + i);
    const float4 t = load_once(reinterpret_cast<const float4*>(a.test) + i);
    quality_take(p, r.x, t.x);
    quality_take(p, r.y, t.y);
    quality_take(p, r.z, t.z);
    quality_take(p, r.w, t.w);
  }
  if (blockIdx.x == 0 && threadIdx.x < (a.n & 3)) {             // the last one to three values
    const u64 i = quads * 4 + threadIdx.x;
    quality_take(p, a.ref[i], a.test[i]);
  }
  const QualityPartial w = quality_fold_workgroup(p, sh);
  if (threadIdx.x == 0) a.partials[blockIdx.x] = w;
}

__global__ __launch_bounds__(kQualityThreads) void quality_final_kernel(QualityArgs a, u32 count) {
  __shared__ QualityPartial sh[kQualityThreads];
  QualityPartial p{0.0, 0.0, __builtin_inf(), -__builtin_inf()};
  for (u32 i = threadIdx.x; i < count; i += kQualityThreads) quality_fold(p, a.partials[i]);
  const QualityPartial w = quality_fold_workgroup(p, sh);
  if (threadIdx.x == 0) a.partials[count] = w;
}

}  // namespace zc

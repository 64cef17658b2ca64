// Small kernels of the C-ABI's export and diagnostic calls.
#pragma once
#include "common.h"
#include "decode.h"

namespace mkv {

// ---- plain copy: the yardstick hardware counters are scaled by (known bytes read and written)
__global__ __launch_bounds__(256) void calib_copy_kernel(uint4 *dst, const uint4 *src, size_t nvec) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// ---- plain read: every workgroup streams a contiguous share, 8 independent 16-byte loads per thread in flight,
// everything folded into one word per workgroup (so that the loads stay); what the device sustains when a kernel
// does nothing but stream.  STREAM: non-temporal loads, as the decode kernels use for what does not fit the
// memory-side cache.
template <bool STREAM>
__global__ __launch_bounds__(1024) void calib_read_kernel(uint32_t *sink, const uint4 *src, size_t nvec, size_t per_block) {
  constexpr int UNR = 8;
  const size_t lo = (size_t)blockIdx.x * per_block, hi = lo + per_block < nvec ? lo + per_block : nvec;
  const int NT = blockDim.x;
  uint32_t acc = 0;
  size_t i = lo + threadIdx.x;
  for (; i + (size_t)(UNR - 1) * NT < hi; i += (size_t)UNR * NT) {
    uint4 r[UNR];
#pragma unroll
    for (int k = 0; k < UNR; ++k) r[k] = ldg16<STREAM>(src + i + (size_t)k * NT);
#pragma unroll
    for (int k = 0; k < UNR; ++k) acc ^= r[k].x ^ r[k].y ^ r[k].z ^ r[k].w;
  }
  for (; i < hi; i += NT) {
    const uint4 v = ldg16<STREAM>(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) acc ^= __shfl_xor(acc, m);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x & 255], acc);
}

// ---- exports
// out rows are `row` long: the unit's n slots (in the cache's own order, -1 = free), then -1; out_nsnap = how many of
// the tokens are older than the window of the R most recent
__global__ void export_positions_kernel(const int32_t *pos, const int32_t *meta, int32_t *out_pos,
                                        int32_t *out_nsnap, int n, int n_pad, int row, int R) {
  const int u = blockIdx.y, i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < row) out_pos[(size_t)u * row + i] = i < n ? pos[(size_t)u * n_pad + i] : -1;
  if (i == 0 && out_nsnap) {
    const int32_t *m = meta + (size_t)u * META;
    const int tokens = m[0] - m[5], p = m[1];
    out_nsnap[u] = tokens - (p < R ? p : R);
  }
}
__global__ void fill_i32_kernel(int32_t *dst, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = v;
}
__global__ void export_evicted_kernel(const int32_t *meta, int32_t *out, int U) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u < U) out[u] = meta[(size_t)u * META + 2];
}

}  // namespace mkv

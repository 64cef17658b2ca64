// Shared device helpers of libmorphkv (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mkv {

constexpr int WAVE = 64;

struct bf16_t { uint16_t bits; };  // storage only; arithmetic is fp32

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int EPL = 4;  // elements in one 16-byte lane load
  __device__ static inline void unpack(const uint4 &r, float *f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};
template <> struct Elem<bf16_t> {
  static constexpr int EPL = 8;
  __device__ static inline void unpack(const uint4 &r, float *f) {
    // bf16 -> fp32 is a 16-bit shift: exact
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

// 2^x as the one hardware instruction (1 ulp).  The library routine wraps it in a range reduction that keeps
// results below 2^-126 as denormals; the softmax has no use for those (they vanish in sums of order 1), and the
// five extra instructions per exponential sit on every wave's critical path.
__device__ inline float exp2_native(float x) { return __builtin_amdgcn_exp2f(x); }

// non-negative remainder
__device__ __host__ inline int pmod(int a, int m) { int r = a % m; return r < 0 ? r + m : r; }

// fusion of two recorded weights: sum (Eq.5; also the running-sum comparison policy, fusion 2) or max (Eq.6);
// identity is 0 for both (weights >= 0)
__device__ inline float fuse2(int fusion, float a, float b) { return fusion == 1 ? fmaxf(a, b) : a + b; }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
  return v;
}

// State of the sliding-window score aggregate of one column (one older token).
//
// For column c the fused score over the R newest rows is kept as f(old part, new part):
//   nw[c]      = f(rows recorded after the column's last rebuild point p0)
//   sfx[r][c]  = f(rows t..p0) with t = p' - R + 1, for the one future step p' in (p0, p0+R] with p' mod R == r
// so a step reads one sfx row and updates nw: no re-read of the R rows (Eq.4-6 evaluated incrementally).
// Columns are rebuilt in turn: column c has phase phi(c) and is rebuilt from the R rows after every step
// p0 with p0 mod R == phi(c).
//
// column_scan computes that state for one column from its R row values, as of the end of step p_end with
// rebuild point p0 in [p_end-R, p_end]:  v(t) = value of the row of query t (0 for rows that do not exist),
// st(r, x) stores sfx[r][c] = x.  Returns nw[c].
template <class LoadV, class StoreSfx>
__device__ inline float column_scan(int p_end, int p0, int R, int fusion, LoadV v, StoreSfx st) {
  float nwv = 0.f;
  for (int t = p0 + 1; t <= p_end; ++t) nwv = fuse2(fusion, nwv, v(t));
  float acc = 0.f;
  for (int t = p0; t >= p_end - R + 2; --t) {
    acc = fuse2(fusion, acc, v(t));
    st(pmod(t - 1, R), acc);
  }
  st(pmod(p0, R), 0.f);
  return nwv;
}

// most recent rebuild point of a column with phase phi that lies strictly before step p
__device__ inline int last_rebuild_before(int p, int phi, int R) { return p - 1 - pmod(p - 1 - phi, R); }

}  // namespace mkv

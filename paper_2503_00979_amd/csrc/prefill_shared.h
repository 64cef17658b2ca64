// The prompt-time kernels that are not templates (one copy in the library: prefill_f32.hip holds them and exports
// their launchers): fused scores from stored rows and the recorded rows (fp32 path), the top-C radix select and
// the aggregate state of the columns (both paths).
#pragma once
#include "prefill.h"

namespace mkv {

// ---- P2: fused score of every older token (Eq.5 / Eq.6 over the window rows)
__global__ __launch_bounds__(256) void prefill_fuse_kernel(PrefillParams P) {
  const int u = blockIdx.y, k = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = (u / P.Mkv) % P.B, N = P.plen[b], R = P.R, Rw = N < R ? N : R, n_old = N - Rw;
  if (k >= n_old) return;
  const float *Sr = P.Srow + (size_t)u * R * P.Nmax;
  float F = Sr[k];
  for (int j = 1; j < Rw; ++j) F = fuse2(P.fusion, F, Sr[(size_t)j * P.Nmax + k]);
  P.F[(size_t)u * P.Nmax + k] = F;
}

// ---- P3: keep the min(C, n_old) largest scores, ties keep the lower position; ascending positions out.
// Radix select (4 x 8 bits, scores are non-negative floats so their bit patterns order like integers)
// finds the value of the C-th largest; an ordered compaction then keeps everything above it and the
// first few equal to it.
__global__ __launch_bounds__(1024) void prefill_select_kernel(PrefillParams P) {
  __shared__ unsigned hist[256];
  __shared__ unsigned s_prefix, s_need;
  __shared__ int wsum[16][2];
  __shared__ int carry[2];
  const int u = blockIdx.x, tid = threadIdx.x, NT = blockDim.x, lane = tid % WAVE, wave = tid / WAVE;
  const int b = (u / P.Mkv) % P.B, N = P.plen[b], R = P.R, Rw = N < R ? N : R, n_old = N - Rw;
  const float *F = P.F + (size_t)u * P.Nmax;
  int32_t *sel = P.sel + (size_t)u * P.Cs;
  const int keep = n_old < P.C ? n_old : P.C;
  if (tid == 0) {
    int32_t *m = P.meta + (size_t)u * META;
    m[0] = keep + Rw; m[1] = N; m[2] = -1; m[3] = N % R; m[4] = N; m[5] = 0;  // slots in use, next position, .., free slots
  }
  if (tid < P.T) P.evl[(size_t)u * P.T + tid] = -1;
  if (tid == 0 && P.sp_cnt) P.sp_cnt[u] = 0;
  if (n_old <= P.C) {
    for (int k = tid; k < n_old; k += NT) sel[k] = k;
    return;
  }
  if (tid == 0) { s_prefix = 0u; s_need = (unsigned)keep; }
  __syncthreads();
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = tid; i < 256; i += NT) hist[i] = 0u;
    __syncthreads();
    const unsigned prefix = s_prefix;
    const unsigned himask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
    for (int k = tid; k < n_old; k += NT) {
      const unsigned bits = __float_as_uint(F[k]);
      if ((bits & himask) == prefix) atomicAdd(&hist[(bits >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      unsigned need = s_need, cum = 0u;
      int bin = 255;
      for (; bin > 0; --bin) {
        if (cum + hist[bin] >= need) break;
        cum += hist[bin];
      }
      s_need = need - cum;  // how many are wanted from this bin
      s_prefix = prefix | ((unsigned)bin << shift);
    }
    __syncthreads();
  }
  const unsigned tau = s_prefix;  // bit pattern of the C-th largest score
  const int need_eq = (int)s_need; // how many of the scores equal to it are kept (lowest positions first)
  if (tid == 0) { carry[0] = 0; carry[1] = 0; }
  __syncthreads();
  for (int base = 0; base < n_old; base += NT) {
    const int k = base + tid;
    unsigned bits = 0u;
    if (k < n_old) bits = __float_as_uint(F[k]);
    const int is_eq = (k < n_old && bits == tau) ? 1 : 0;
    const int is_gt = (k < n_old && bits > tau) ? 1 : 0;
    // exclusive rank among equals
    int xe = is_eq;
#pragma unroll
    for (int s = 1; s < WAVE; s <<= 1) { const int o = __shfl_up(xe, s); if (lane >= s) xe += o; }
    if (lane == WAVE - 1) wsum[wave][0] = xe;
    __syncthreads();
    int eoff = carry[0];
    for (int x = 0; x < wave; ++x) eoff += wsum[x][0];
    const int eq_rank = eoff + xe - is_eq;
    const int kept = is_gt | (is_eq && eq_rank < need_eq ? 1 : 0);
    int xk = kept;
#pragma unroll
    for (int s = 1; s < WAVE; s <<= 1) { const int o = __shfl_up(xk, s); if (lane >= s) xk += o; }
    if (lane == WAVE - 1) wsum[wave][1] = xk;
    __syncthreads();
    int koff = carry[1];
    for (int x = 0; x < wave; ++x) koff += wsum[x][1];
    if (kept) sel[koff + xk - 1] = k;
    __syncthreads();
    if (tid == NT - 1) { carry[0] = eoff + xe; carry[1] = koff + xk; }
    __syncthreads();
  }
}

// ---- P4b: recorded rows restricted to the resident columns
__global__ __launch_bounds__(256) void prefill_ring_kernel(PrefillParams P) {
  const int u = blockIdx.y, col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= P.n_pad) return;
  const int b = (u / P.Mkv) % P.B, N = P.plen[b], R = P.R, Rw = N < R ? N : R;
  const int n_snap = prefill_n_old(P, N);
  const int src = col < P.n ? prefill_slot_source(P, u, col, N, n_snap) : -1;
  const float *Sr = P.Srow + (size_t)u * R * P.Nmax;
  float *ringu = P.ring + (size_t)u * R * P.n_pad;
  for (int r = 0; r < R; ++r) {
    // the window query whose position is congruent to r, if any
    int j = -1;
    if (N >= R) j = pmod(r - (N - R), R);
    else if (r < N) j = r;
    float v = 0.f;
    if (j >= 0 && src >= 0) {
      const int pj = N - Rw + j;
      if (src < pj) v = Sr[(size_t)j * P.Nmax + src];  // rows after the token's own
    }
    ringu[(size_t)r * P.n_pad + col] = v;
  }
}

// ---- P5: aggregate state of every slot's column, as of the end of step N-1
__global__ __launch_bounds__(256) void prefill_state_kernel(PrefillParams P) {
  const int u = blockIdx.y, c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= P.CsP) return;
  const int b = (u / P.Mkv) % P.B, N = P.plen[b], R = P.R;
  const int n_snap = prefill_n_old(P, N);
  const float *ringu = P.ring + (size_t)u * R * P.n_pad;
  float *sfxu = P.sfx + (size_t)u * R * P.CsP;
  float nwv = 0.f;
  if (c < n_snap + (N < R ? N : R)) {  // every slot in use is a column (rows up to a token's own are zero in the recorded rows)
    const int p_end = N - 1;
    const int p0 = P.fusion == 2 ? p_end - R : last_rebuild_before(p_end, c / P.cps, R);  // running sum: no old part
    nwv = column_scan(
        p_end, p0, R, P.fusion, [&](int t) { return t >= 0 ? ringu[(size_t)pmod(t, R) * P.n_pad + c] : 0.f; },
        [&](int r, float x) { sfxu[(size_t)r * P.CsP + c] = x; });
  } else {
    for (int r = 0; r < R; ++r) sfxu[(size_t)r * P.CsP + c] = 0.f;
  }
  P.nw[(size_t)u * P.CsP + c] = nwv;
}

}  // namespace mkv

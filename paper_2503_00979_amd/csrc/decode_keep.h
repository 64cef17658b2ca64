// Decode step of a layer that keeps every token (Appendix A.6, selective layer retention): attention of the new
// token over everything the unit holds, then the token is appended.  Nothing is
// recorded, fused or selected in such a layer, so no weight has to outlive the tile it was computed for: the
// softmax runs ONLINE (running maximum and sum per head, the output accumulators rescaled when the maximum
// moves), a block of 32 slots goes K tiles -> logits -> weights -> V tile -> output without ever being written
// down, and the cache's length is bounded by nothing but the memory the caller gave.
//
// S workgroups of 256 or 512 threads per unit (grid S x units); the waves of a unit's workgroups take the blocks of
// its slots in use in turn, each with its own (maximum, sum,
// output); a workgroup's waves are merged through LDS (Eq.1: softmax over all resident tokens and the token
// itself).  With S > 1 -- launches of few units, so that every compute unit gets a share -- each workgroup leaves
// its merged (maximum, sum, output) in the split kernel's workspace with agent-scope stores, counts in, and the
// last one to arrive merges the S records and finishes the step (the protocol of decode_split.h).
// bf16 caches in MFMA tile order (Layout<bf16_t, D>), like the fused kernel.
#pragma once
#include "decode.h"
#include "decode_split.h"  // the workspace accesses at agent scope, SPLIT_MAX, the layout of a workgroup's record

namespace mkv {

constexpr int KEEP_NT = 512;  // threads of a workgroup (256 works too and was measured no faster)
constexpr int KEEP_PS = 36;  // floats per head row of a wave's weight staging tile (32 slots + 4: rows start 4 banks apart)

// dynamic LDS of decode_keep_kernel launched with `threads` threads a workgroup
inline size_t decode_keep_lds_bytes(int G, int D, int threads) {
  const size_t NW = (size_t)threads / WAVE;
  return (NW * 16 * KEEP_PS /*weights of a block per wave*/ + NW * 16 /*rescale factors*/ + 2 * NW * 16 /*maxima, sums*/ +
          NW * G * D /*outputs*/ + 16 + 16 + 2 * SPLIT_MAX * 8 /*the workgroups' maxima and sums*/) * 4;
}

template <int D, int G>
__global__ __launch_bounds__(KEEP_NT) void decode_keep_kernel(DecodeParams P) {
  using T = bf16_t;
  using L = Layout<T, D>;
  constexpr int KB = L::KB, CB = L::CB;
  const int NT = blockDim.x, NW = NT / WAVE;
  extern __shared__ __align__(16) float smem[];

  const int s = blockIdx.x, S = gridDim.x, u = blockIdx.y + P.u0, uio = u - P.io_u0, tid = threadIdx.x;
  const int wave = tid / WAVE, lane = tid % WAVE, head = lane & 15, kq = lane >> 4;
  const int n_pad = P.n_pad;

  float *stg = smem + (size_t)wave * 16 * KEEP_PS;            // [16][KEEP_PS] this wave's weights of one block
  float *scw = smem + (size_t)NW * 16 * KEEP_PS + wave * 16;  // [16] this wave's rescale factors
  float *mW = smem + (size_t)NW * 16 * KEEP_PS + NW * 16;     // [NW][16] maxima
  float *zW = mW + NW * 16;                                   // [NW][16] sums
  float *OW = zW + NW * 16;                                   // [NW][G][D] outputs
  int *sh = (int *)(OW + (size_t)NW * G * D);                 // [16] 2..6: see StepTail; 7: arrival count
  float *shf = (float *)(sh + 16);                            // [16] 1..8: logits of the token against its own key
  float *msl = shf + 16;                                      // [SPLIT_MAX][8] the workgroups' maxima (S > 1)
  float *zsl = msl + SPLIT_MAX * 8;                           // [SPLIT_MAX][8] ... and sums

  const T *Kb = (const T *)P.K + (size_t)u * n_pad * D;
  const T *Vb = (const T *)P.V + (size_t)u * n_pad * D;
  const T *qb = (const T *)P.q + (size_t)uio * G * D;
  const T *knew = (const T *)P.k_new + (size_t)uio * D;
  const T *vnew = (const T *)P.v_new + (size_t)uio * D;
  int32_t *posu = P.pos + (size_t)u * n_pad;

  const int32_t *meta = P.meta + (size_t)u * META;
  const int n_used = meta[0], p = meta[1], w = meta[3];

  // ---- the blocks of 32 slots that hold tokens
  const int total = (n_used + 31) >> 5;
  const bool zig = P.zig != 0;
  auto block_of = [&](int i) { return zig ? total - 1 - i : i; };
  // the newest blocks (as many as the handle's share of the memory-side cache holds per unit) are read with ordinary
  // loads and stay there from step to step; the older ones stream past it
  const int thr = total - P.keep_cached_blocks;
  auto streams = [&](int blk) { return blk < thr; };

  uint4 ka[2][KB], vb[CB];
  auto load_k = [&](int blk) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const T *a = Kb + ((size_t)(2 * blk + t) * KB + kb) * 512 + lane * 8;
        ka[t][kb] = streams(blk) ? ldg16<true>(a) : ldg16<false>(a);
      }
  };
  auto load_v = [&](int blk) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const T *a = Vb + ((size_t)blk * CB + cb) * 512 + lane * 8;
      vb[cb] = streams(blk) ? ldg16<true>(a) : ldg16<false>(a);
    }
  };
  // block i of the unit goes to workgroup (i / NW) mod S, wave i mod NW
  const int i0 = s * NW + wave, istep = S * NW;
  if (i0 < total) {
    const int blk = block_of(i0);
    load_k(blk);
    load_v(blk);
  }
  // query fragments: B operand of the K product, 32 channels x 16 heads (heads >= G are zero)
  bf16x8_t qfr[KB];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    uint4 r = {0u, 0u, 0u, 0u};
    if (head < G) r = *(const uint4 *)(qb + (size_t)head * D + kb * 32 + kq * 8);
    qfr[kb] = __builtin_bit_cast(bf16x8_t, r);
  }

  // ---- the wave's blocks: running maximum m and sum zp of the lane's head (m is the same in the four lanes of a
  // head, zp is the lane's own part), output acc[cb][i] of head 4 kq + i and channel cb * 16 + (lane & 15)
  float m = -INFINITY, zp = 0.f;
  f32x4_t acc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) acc[cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  for (int i = i0; i < total; i += istep) {
    const int blk = block_of(i);
    // logits of the block's 32 slots: lane holds slots t*16 + 4 kq + e (t = 0, 1; e = 0..3) of its head
    float l[8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[t][kb]), qfr[kb], c, 0, 0, 0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = blk * 32 + t * 16 + 4 * kq + e;
        l[4 * t + e] = slot_valid(j, n_used) ? c[e] * P.scale_log2 : -INFINITY;
      }
    }
    // the K registers are free: the next block's K tiles are asked for now
    const bool more = i + istep < total;
    const int nblk = more ? block_of(i + istep) : 0;
    if (more) load_k(nblk);

    float bmax = fmaxf(fmaxf(fmaxf(l[0], l[1]), fmaxf(l[2], l[3])), fmaxf(fmaxf(l[4], l[5]), fmaxf(l[6], l[7])));
    bmax = max_over_rows(bmax);
    const float m_new = fmaxf(m, bmax);
    if (__ballot(m_new > m) != 0ull) {
      // the maximum of some head moved: what has been summed so far is rescaled.  The output accumulators of
      // this lane belong to the heads 4 kq .. 4 kq + 3: their factors come through LDS
      const float sc = m == -INFINITY ? 0.f : exp2_native(m - m_new);
      zp *= sc;
      if (kq == 0) scw[head] = sc;
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_wave_barrier();
      const float4 s4 = *(const float4 *)(scw + 4 * kq);
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        acc[cb][0] *= s4.x; acc[cb][1] *= s4.y; acc[cb][2] *= s4.z; acc[cb][3] *= s4.w;
      }
      m = m_new;
    }
    float pw[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pw[e] = l[e] == -INFINITY ? 0.f : exp2_native(l[e] - m);
      zp += pw[e];
    }
    // weights into the order the V product wants them: lane (head, kq) needs the slots 8 kq .. 8 kq + 7
    *(float4 *)(stg + head * KEEP_PS + 4 * kq) = make_float4(pw[0], pw[1], pw[2], pw[3]);
    *(float4 *)(stg + head * KEEP_PS + 16 + 4 * kq) = make_float4(pw[4], pw[5], pw[6], pw[7]);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
    const float4 x = *(const float4 *)(stg + head * KEEP_PS + 8 * kq);
    const float4 y = *(const float4 *)(stg + head * KEEP_PS + 8 * kq + 4);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
    const float pv[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
    bf16x8_t ahi, alo;  // bf16 hi + lo parts, so that the product keeps ~16 bits of the weight
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const __bf16 h = (__bf16)pv[e];
      ahi[e] = h;
      alo[e] = (__bf16)(pv[e] - (float)h);
    }
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, vb[cb]);
      acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi, bv, acc[cb], 0, 0, 0);
      acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo, bv, acc[cb], 0, 0, 0);
    }
    if (more) load_v(nblk);
  }

  // ---- the token's logits against its own key: wave 0, the key as slot 0 of one more tile (as in the fused kernel)
  if (wave == 0) {
    f32x4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      uint4 a = {0u, 0u, 0u, 0u};
      if (head == 0) a = *(const uint4 *)(knew + kb * 32 + kq * 8);
      c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), qfr[kb], c, 0, 0, 0);
    }
    if (lane < G) shf[1 + lane] = c[0] * P.scale_log2;  // lanes 0..15 (kq = 0): slot 0, head = lane
  }
  // ---- the wave's results
  const float zs = sum_over_rows(zp);
  if (kq == 0) { mW[wave * 16 + head] = m; zW[wave * 16 + head] = zs; }
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int g = 4 * kq + e;
      if (g < G) OW[(size_t)(wave * G + g) * D + cb * 16 + head] = acc[cb][e];
    }
  if (tid == 0) {
    // every token is kept: the new one is appended (the host has made sure there is room)
    sh[2] = n_used;
    sh[3] = -1;
    sh[4] = n_used + 1;
    sh[5] = 0;
    sh[6] = 0;
  }
  __syncthreads();

  constexpr int PART = 2 * G + G * D;
  if (S == 1) {
    // ---- merge of the waves and the token itself (Eq.1), output
    for (int idx = tid; idx < G * D; idx += NT) {
      const int g = idx / D, ch = idx % D;
      const float ls = shf[1 + g];
      float M = ls;
      for (int x = 0; x < NW; ++x) M = fmaxf(M, mW[x * 16 + g]);
      const float es = exp2_native(ls - M);
      float Z = es;
      float o = es * __uint_as_float(((uint32_t)((const uint16_t *)vnew)[ch]) << 16);
      for (int x = 0; x < NW; ++x) {
        const float mx = mW[x * 16 + g];
        const float f = mx == -INFINITY ? 0.f : exp2_native(mx - M);
        Z = fmaf(f, zW[x * 16 + g], Z);
        o = fmaf(f, OW[(size_t)(x * G + g) * D + ch], o);
      }
      P.out[((size_t)uio * G + g) * D + ch] = o / Z;
    }
  } else {
    // ---- this workgroup's record: its waves merged at their common maximum (no token of its own yet)
    const __amdgpu_buffer_rsrc_t part = ws_rsrc(P.sp_part + ((size_t)u * P.sp_smax) * PART, (uint32_t)P.sp_smax * PART * 4u);
    for (int idx = tid; idx < G * D; idx += NT) {
      const int g = idx / D, ch = idx % D;
      float M = -INFINITY;
      for (int x = 0; x < NW; ++x) M = fmaxf(M, mW[x * 16 + g]);
      float Z = 0.f, o = 0.f;
      for (int x = 0; x < NW; ++x) {
        const float mx = mW[x * 16 + g];
        const float f = mx == -INFINITY ? 0.f : exp2_native(mx - M);
        Z = fmaf(f, zW[x * 16 + g], Z);
        o = fmaf(f, OW[(size_t)(x * G + g) * D + ch], o);
      }
      ws_store1(part, (uint32_t)(s * PART + 2 * G + idx), o);
      if (ch == 0) {
        ws_store1(part, (uint32_t)(s * PART + g), M);
        ws_store1(part, (uint32_t)(s * PART + G + g), Z);
      }
    }
    // count in: every thread waits until its stores have been acknowledged, then one thread bumps the unit's
    // counter; the last workgroup of the unit carries on
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
    __syncthreads();
    if (tid == 0) sh[7] = atomicAdd(&P.sp_cnt[u], 1);
    __syncthreads();
    if (sh[7] != S - 1) return;
    for (int i = tid; i < S * G; i += NT) {
      const int ss = i / G, g = i - ss * G;
      msl[ss * 8 + g] = ws_load1(part, (uint32_t)(ss * PART + g));
      zsl[ss * 8 + g] = ws_load1(part, (uint32_t)(ss * PART + G + g));
    }
    if (tid == 0) P.sp_cnt[u] = 0;  // for the unit's next step
    __syncthreads();
    // ---- merge of the workgroups and the token itself (Eq.1), output; the records are asked for eight at a time
    for (int idx = tid; idx < G * D; idx += NT) {
      const int g = idx / D, ch = idx % D;
      const float ls = shf[1 + g];
      float M = ls;
      for (int ss = 0; ss < S; ++ss) M = fmaxf(M, msl[ss * 8 + g]);
      const float es = exp2_native(ls - M);
      float Z = es;
      float o = es * __uint_as_float(((uint32_t)((const uint16_t *)vnew)[ch]) << 16);
      for (int s0 = 0; s0 < S; s0 += 8) {
        float ob[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) ob[k] = s0 + k < S ? ws_load1(part, (uint32_t)((s0 + k) * PART + 2 * G + idx)) : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (s0 + k < S) {
            const float mx = msl[(s0 + k) * 8 + g];
            const float f = mx == -INFINITY ? 0.f : exp2_native(mx - M);
            Z = fmaf(f, zsl[(s0 + k) * 8 + g], Z);
            o = fmaf(f, ob[k], o);
          }
      }
      P.out[((size_t)uio * G + g) * D + ch] = o / Z;
    }
  }
  // the tail: shared with the other kernels
  StepTail<T> tc{P, u, tid, NT, NW, wave, lane, n_pad, n_used, p, w, 1, sh, nullptr, nullptr, nullptr, nullptr, posu, knew, vnew};
  commit_step<T, D, false>(tc);
}

}  // namespace mkv

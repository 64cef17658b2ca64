// MorphKV decode step with a unit's cache split over several workgroups (bf16 caches).
//
// Why: the fused kernel (decode.h) gives a unit one workgroup and keeps every weight of the step in LDS: a unit
// whose C + R does not fit there (a layer that keeps every token, Appendix A.6; very large C) cannot run in it.
// A launch with fewer units than the device has compute units also leaves most of the device idle there.  Here
// S workgroups share a unit.  (Chosen by the library for caches beyond the fused kernel's LDS; for launches with
// few units only on request, MORPHKV_SPLIT_BPS: measured, its longer chain -- partial results out, count in,
// merge -- costs more than the shorter streaming saves at 544 and 1088 slots.)
//
//   phase A (every workgroup, on its share of 32-slot blocks): logits (Eq.1) -> LOCAL maximum m_s and
//     exponentials p~ = exp2(l - m_s) -> local sum Z_s -> partial output O_s = sum_j p~_j V_j.  The logits, m_s, Z_s
//     and O_s go to a workspace; the workgroup then counts itself in.  Whoever arrives last carries on alone:
//   phase B (one workgroup per unit): global maximum M and sum Z from the S pairs (m_s, Z_s) and the token's own
//     logit; weights p = exp2(l - M) / Z from the logits; out = sum_s O_s exp2(m_s - M) / Z + p_self v_new; then exactly what
//     the fused kernel does after its softmax: record the group-summed row (Algorithm 1), update the aggregates,
//     fused scores (Eq.4-6), eviction (Eq.7), the new token into the freed slot.  No weight is held in LDS in this phase, so C + R is
//     bounded by the workspace only.
//
// Nobody waits for anybody: the last arrival is found with one atomic counter per unit, so the grid needs no
// co-residency and every wave reaches its end.  The workgroups of a unit may sit on different XCDs, whose L2
// caches are not coherent with one another; a device-scope fence would write back and invalidate a whole L2 per
// workgroup (measured: the step got 3x slower than unsplit).  Instead everything that crosses workgroups is
// written and read at agent scope (the sc1 forms the compiler uses for agent-scope atomics, here as 16-byte
// buffer accesses): stores go through to the memory side, loads never take a stale line; a workgroup waits for
// its own stores to be acknowledged, then counts itself in.
#pragma once
#include "decode.h"

namespace mkv {

constexpr int SPLIT_NT = 256, SPLIT_NW = SPLIT_NT / WAVE;
constexpr int SPLIT_RB = 32;  // rows per lane of the rebuild: a lane's whole chunk in one batch
constexpr int SPLIT_MAX = 32;  // workgroups per unit at most

// agent-scope (sc1) accesses to the workspace
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr int AUX_AGENT = 16;  // cache-policy operand of the buffer builtins: sc1
__device__ inline __amdgpu_buffer_rsrc_t ws_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ inline void ws_store4(__amdgpu_buffer_rsrc_t r, uint32_t idx, float4 v) {
  const u32x4_t t = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
  __builtin_amdgcn_raw_buffer_store_b128(t, r, idx * 4u, 0, AUX_AGENT);
}
__device__ inline void ws_store1(__amdgpu_buffer_rsrc_t r, uint32_t idx, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, idx * 4u, 0, AUX_AGENT);
}
__device__ inline float4 ws_load4(__amdgpu_buffer_rsrc_t r, uint32_t idx) {
  const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(r, idx * 4u, 0, AUX_AGENT);
  return make_float4(__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w));
}
__device__ inline float ws_load1(__amdgpu_buffer_rsrc_t r, uint32_t idx) {
  return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, idx * 4u, 0, AUX_AGENT));
}

// floats of one (unit, split) record in the workspace: m[G], Z[G], O[G][D]
__host__ __device__ inline int split_part_floats(int G, int D) { return 2 * G + G * D; }

// LDS bytes of decode_split_kernel (bps = blocks of 32 slots per workgroup): the share's logits, and beside them
// what the end of the step needs (rebuilt aggregates, small arrays)
inline size_t decode_split_lds_bytes(int bps, int G, int D, int R, int cps, int CsP, int T) {
  const size_t cpt = (size_t)turn_cols_padded(cps);
  const size_t lgA = (size_t)G * (bps * 32 + 4), omA = (size_t)SPLIT_NW * G * D;
  const size_t a = (lgA > omA ? lgA : omA) + 2 * SPLIT_NW * 8 + 16;
  size_t b = (size_t)R * cpt + cpt + 3 * 16 + 16 + 16 + 3 * SPLIT_MAX * 8 + 4 * 8;
  if (T > 1) b += 2 * (size_t)CsP + 2 * 3 * 16 + (size_t)CsP / 32;  // (CsP = n_pad: one bit per slot)
  return (a + b) * 4;
}

template <int D, int G>
__global__ __launch_bounds__(SPLIT_NT) void decode_split_kernel(DecodeParams P) {
  using T = bf16_t;
  using L = Layout<T, D>;
  constexpr int NT = SPLIT_NT, NW = SPLIT_NW, KB = L::KB, CB = L::CB, PART = 2 * G + G * D;
  extern __shared__ __align__(16) float smem[];

  const int s = blockIdx.x, S = gridDim.x, u = blockIdx.y + P.u0, uio = u - P.io_u0;
  const int tid = threadIdx.x, wave = tid / WAVE, lane = tid % WAVE, head = lane & 15, kq = lane >> 4;
  const int Cs = P.Cs, CsP = P.CsP, R = P.R, n_pad = P.n_pad, cps = P.cps, cpt = P.cpt, bps = P.sp_bps;
  const bool cum = P.fusion == 2;
  const int fusion = cum ? 0 : P.fusion;
  const int Tev = P.T;
  const bool keep = P.keep_all != 0;  // a layer that keeps every token: attention and append only

  const T *Kb = (const T *)P.K + (size_t)u * n_pad * D;
  const T *Vb = (const T *)P.V + (size_t)u * n_pad * D;
  const T *qb = (const T *)P.q + (size_t)uio * G * D;
  const T *knew = (const T *)P.k_new + (size_t)uio * D;
  const T *vnew = (const T *)P.v_new + (size_t)uio * D;
  // the unit's part of the workspace, addressed in floats through agent-scope buffer accesses
  const __amdgpu_buffer_rsrc_t part = ws_rsrc(P.sp_part + ((size_t)u * P.sp_smax) * PART, (uint32_t)P.sp_smax * PART * 4u);  // [S][PART]
  const __amdgpu_buffer_rsrc_t wts = ws_rsrc(P.sp_w + (size_t)u * G * n_pad, (uint32_t)G * n_pad * 4u);  // [G][n_pad] logits

  const int nblk = n_pad / 32;
  const int b0 = s * bps, b1 = min(nblk, b0 + bps), j0s = b0 * 32, nsl = (b1 - b0) * 32;

  // ---- LDS carve-up: the share's logits first, then what the end of the step needs
  const int lgs = bps * 32 + 4;
  const size_t lgsz = max((size_t)G * lgs, (size_t)NW * G * D);
  float *lg = smem;                          // [G][lgs] logits -> p~; later [NW][G][D] output partials
  float *redA = lg + lgsz;                   // [NW][8] maxima
  float *redB = redA + NW * 8;               // [NW][8] sums
  int *shi = (int *)(redB + NW * 8);         // [16]
  float *stage = (float *)(shi + 16);        // [R][cpt] rebuilt aggregates on their way to the sfx rows
  float *turn = stage + (size_t)R * cpt;     // [cpt]
  float *bestF = turn + cpt;                 // [16]
  int *bestC = (int *)(bestF + 16);          // [16]
  int *bestP = bestC + 16;                   // [16]
  int *sh = bestP + 16;                      // [16]
  float *shf = (float *)(sh + 16);           // [16]
  float *fac = shf + 16;                     // [SPLIT_MAX][8] exp2(m_s - M) / Z
  float *msl = fac + SPLIT_MAX * 8;          // [SPLIT_MAX][8] m_s
  float *zsl = msl + SPLIT_MAX * 8;          // [SPLIT_MAX][8] Z_s
  float *invl = zsl + SPLIT_MAX * 8;         // [8] 1 / Z
  float *psl = invl + 8;                     // [8] weight of the token on itself
  float *sfl = psl + 8;                      // [8] its own logits
  float *Mgl = sfl + 8;                      // [8] global maximum per head
  float *Fl = Mgl + 8;                                    // [CsP]   (T > 1 only, as the ones below)
  int *Pl = (int *)(Fl + (Tev > 1 ? CsP : 0));            // [CsP]
  float *best2 = (float *)(Pl + (Tev > 1 ? CsP : 0));     // [2][3][16]
  unsigned *hbits = (unsigned *)(best2 + 2 * 3 * 16);     // [n_pad / 32] one bit per free slot (see free_slot_bits)

  // ================= phase A: this workgroup's share =================
  // A wave takes the blocks wave, wave + NW, .. of the share, NB of them in flight at a time (K tile pair and V tile
  // each): a share of up to NB * NW blocks is asked for in full before anything is waited for -- the addresses
  // depend on nothing -- and costs one round trip to memory.
  constexpr int NB = 2;
  uint4 ka[NB][2][KB], vb[NB][CB];
  auto load_k = [&](uint4 (&dst)[2][KB], int blk) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const T *a = Kb + ((size_t)(2 * blk + t) * KB + kb) * 512 + lane * 8;
        dst[t][kb] = blk < P.nt_k ? ldg16<true>(a) : ldg16<false>(a);
      }
  };
  auto load_v = [&](uint4 (&dst)[CB], int blk) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const T *a = Vb + ((size_t)blk * CB + cb) * 512 + lane * 8;
      dst[cb] = blk < P.nt_v ? ldg16<true>(a) : ldg16<false>(a);
    }
  };
  const int blk_first = b0 + wave;
#pragma unroll
  for (int i = 0; i < NB; ++i)
    if (blk_first + i * NW < b1) load_k(ka[i], blk_first + i * NW);
#pragma unroll
  for (int i = 0; i < NB; ++i)
    if (blk_first + i * NW < b1) load_v(vb[i], blk_first + i * NW);
  bf16x8_t qfr[KB];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    uint4 r = {0u, 0u, 0u, 0u};
    if (head < G) r = *(const uint4 *)(qb + (size_t)head * D + kb * 32 + kq * 8);
    qfr[kb] = __builtin_bit_cast(bf16x8_t, r);
  }
  const int32_t *meta = P.meta + (size_t)u * META;
  const int n_used = meta[0], p = meta[1], w = meta[3];
  const int gen_step = p - meta[4] + 1;
  const bool sel_step = P.T > 1 && gen_step % P.T == 0;
  const int n_holes = P.T > 1 ? meta[5] : 0;  // free slots below n_used (coarse schedule)
  const int wm1 = w == 0 ? R - 1 : w - 1;
  const int turn0 = wm1 * cps;
  int turn_n = n_used - turn0;
  turn_n = turn_n < 0 || cum ? 0 : (turn_n > cps ? cps : turn_n);
  float *ringu = P.ring + (size_t)u * R * n_pad;
  float *sfxu = P.sfx + (size_t)u * R * CsP;
  float *nwu = P.nw + (size_t)u * CsP;
  int32_t *posu = P.pos + (size_t)u * n_pad;

  // Whichever workgroup ends up merging needs the rebuilt aggregates of this step's turn columns.  Nobody knows yet
  // who that is, and the rebuild is a chain of small gathers: every workgroup does it now, under its K/V loads (a
  // few KB per workgroup, from L2 after the first), instead of the merging one alone after everybody else is done.
  int hole_top = -1;
  if (n_holes > 0) {  // (the same for the whole workgroup)
    hole_top = P.holes[(size_t)u * Tev + n_holes - 1];
    free_slot_bits(hbits, n_pad, P.holes + (size_t)u * Tev, n_holes, tid, NT);
    lds_barrier();
  }
  // the rebuild's loads (one batch: a lane's whole chunk of rows) go out now, are consumed after the K loop
  TurnRebuildT<SPLIT_RB> tr;
  float rbv[SPLIT_RB];
  const int tgw = turn_group_width(R, SPLIT_RB);
  int nrw = (cps + tgw - 1) / tgw;
  nrw = nrw > NW / 2 ? NW / 2 : nrw;
  const bool rebuilds = wave >= NW - nrw && !keep;
  if (rebuilds) {
    tr.init(lane, p, wm1, cum ? 0 : n_used, R, n_pad, cps, cpt, fusion, ringu, posu, NW - 1 - wave, nrw, tgw);
    tr.begin(rbv);
  }
  // ---- logits of the share
  float mx[G];
#pragma unroll
  for (int g = 0; g < G; ++g) mx[g] = -INFINITY;
  for (int blk0 = blk_first; blk0 < b1; blk0 += NB * NW) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int blk = blk0 + i * NW;
      if (blk < b1) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[i][t][kb]), qfr[kb], acc, 0, 0, 0);
          if (head < G) {
            float l4[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              const int j = blk * 32 + t * 16 + 4 * kq + x;
              l4[x] = slot_valid(j, n_used) ? acc[x] * P.scale_log2 : -INFINITY;
            }
            if (n_holes > 0) {
              const unsigned fb = free_bits4(hbits, blk * 32 + t * 16 + 4 * kq);
#pragma unroll
              for (int x = 0; x < 4; ++x) l4[x] = (fb >> x) & 1u ? -INFINITY : l4[x];
            }
            const float m4 = fmaxf(fmaxf(l4[0], l4[1]), fmaxf(l4[2], l4[3]));
#pragma unroll
            for (int g = 0; g < G; ++g) mx[g] = g == head ? fmaxf(mx[g], m4) : mx[g];
            *(float4 *)(lg + (size_t)head * lgs + (blk - b0) * 32 + t * 16 + 4 * kq) = make_float4(l4[0], l4[1], l4[2], l4[3]);
          }
        }
        if (blk + NB * NW < b1) load_k(ka[i], blk + NB * NW);
      }
    }
  }
  if (rebuilds) tr.finish(rbv, stage, turn);
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float v = wave_max_dpp(mx[g]);
    if (lane == 0) redA[wave * 8 + g] = v;
  }
  lds_barrier();
  // ---- local maximum, exponentials, local sum; the logits themselves go to the workspace: the merging workgroup
  // turns them into weights against the GLOBAL maximum in one step, exactly as the fused kernel does, so that
  // slots with equal logits get bit-equal weights whichever workgroup they fell to (ties stay ties)
  float mref[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = redA[g];
#pragma unroll
    for (int x = 1; x < NW; ++x) v = fmaxf(v, redA[x * 8 + g]);
    mref[g] = v == -INFINITY ? 0.f : v;  // a share without a valid slot: every exponential is 0
  }
  {
    float zs[G];
#pragma unroll
    for (int g = 0; g < G; ++g) zs[g] = 0.f;
    for (int jq = tid; jq < nsl / 4; jq += NT) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float4 *pl = (float4 *)(lg + (size_t)g * lgs + 4 * jq);
        float4 l = *pl;
        if (!keep) ws_store4(wts, (uint32_t)(g * n_pad + j0s + 4 * jq), l);
        l.x = exp2_native(l.x - mref[g]); l.y = exp2_native(l.y - mref[g]); l.z = exp2_native(l.z - mref[g]); l.w = exp2_native(l.w - mref[g]);
        *pl = l;
        zs[g] += (l.x + l.y) + (l.z + l.w);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float v = wave_sum_dpp(zs[g]);
      if (lane == 0) redB[wave * 8 + g] = v;
    }
  }
  lds_barrier();
  if (tid < G) {
    float z = 0.f;
    for (int x = 0; x < NW; ++x) z += redB[x * 8 + tid];
    float m = redA[tid];
    for (int x = 1; x < NW; ++x) m = fmaxf(m, redA[x * 8 + tid]);
    ws_store1(part, (uint32_t)(s * PART + tid), m);
    ws_store1(part, (uint32_t)(s * PART + G + tid), z);
  }
  // ---- partial output of the share: A = 16 heads x 32 slots of p~ (bf16 hi + lo), B = 32 slots x 16 channels of V
  {
    f32x4_t acc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) acc[cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int blk0 = blk_first; blk0 < b1; blk0 += NB * NW) {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int blk = blk0 + i * NW;
        if (blk < b1) {
          bf16x8_t ahi, alo;
          {
            float pv[8];
            if (head < G) {
              const float4 x = *(const float4 *)(lg + (size_t)head * lgs + (blk - b0) * 32 + kq * 8);
              const float4 y = *(const float4 *)(lg + (size_t)head * lgs + (blk - b0) * 32 + kq * 8 + 4);
              pv[0] = x.x; pv[1] = x.y; pv[2] = x.z; pv[3] = x.w; pv[4] = y.x; pv[5] = y.y; pv[6] = y.z; pv[7] = y.w;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e) pv[e] = 0.f;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const __bf16 h = (__bf16)pv[e];
              ahi[e] = h;
              alo[e] = (__bf16)(pv[e] - (float)h);
            }
          }
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) {
            const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, vb[i][cb]);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi, bv, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo, bv, acc[cb], 0, 0, 0);
          }
          if (blk + NB * NW < b1) load_v(vb[i], blk + NB * NW);
        }
      }
    }
    lds_barrier();  // every wave is done reading the exponentials: lg may be reused
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int g = 4 * kq + i;
        if (g < G) lg[(size_t)(wave * G + g) * D + cb * 16 + head] = acc[cb][i];
      }
  }
  lds_barrier();
  for (int idx = tid; idx < G * D; idx += NT) {
    float o = 0.f;
#pragma unroll
    for (int x = 0; x < NW; ++x) o += lg[(size_t)x * G * D + idx];
    ws_store1(part, (uint32_t)(s * PART + 2 * G + idx), o);
  }
  // ---- count in.  Every thread first waits until its stores to the workspace have been acknowledged (they went
  // through to the memory side); after the barrier one thread bumps the unit's counter.  The last workgroup of the
  // unit carries on.
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  __syncthreads();
  if (tid == 0) shi[0] = atomicAdd(&P.sp_cnt[u], 1);
  __syncthreads();
  if (shi[0] != S - 1) return;  // (the whole workgroup takes the same way; shi is not reused below)

  // ================= phase B: the unit's merging workgroup =================
  // everything it reads of the other workgroups comes through agent-scope loads, all asked for at once:
  // the S local maxima and sums, and the logits and per-column state of the first slots each thread records
  const int nq = n_pad / 4;
  float4 lq[G], nw0 = make_float4(0.f, 0.f, 0.f, 0.f), sf0 = nw0;
  int4 pp0 = make_int4(-1, -1, -1, -1);
  if (tid < nq && !keep) {
#pragma unroll
    for (int g = 0; g < G; ++g) lq[g] = ws_load4(wts, (uint32_t)(g * n_pad + 4 * tid));
    if (4 * tid < n_used) {
      nw0 = *(const float4 *)(nwu + 4 * tid);
      sf0 = *(const float4 *)(sfxu + (size_t)w * CsP + 4 * tid);
      pp0 = *(const int4 *)(posu + 4 * tid);
    }
  }
  // partial outputs of the first SH workgroups, for the OPT output elements this thread owns
  constexpr int SH = 8, OPT = (G * D + NT - 1) / NT;
  float ob[OPT][SH];
#pragma unroll
  for (int x = 0; x < OPT; ++x)
#pragma unroll
    for (int ss = 0; ss < SH; ++ss) {
      const int idx = tid + x * NT;
      ob[x][ss] = (ss < S && idx < G * D) ? ws_load1(part, (uint32_t)(ss * PART + 2 * G + idx)) : 0.f;
    }
  for (int i = tid; i < S * G; i += NT) {
    const int ss = i / G, g = i - ss * G;
    msl[ss * 8 + g] = ws_load1(part, (uint32_t)(ss * PART + g));
    zsl[ss * 8 + g] = ws_load1(part, (uint32_t)(ss * PART + G + g));
  }
  // the token's own logits (wave 0, from the same MFMA as the cached keys')
  if (wave == 0) {
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      uint4 a = {0u, 0u, 0u, 0u};
      if (head == 0) a = *(const uint4 *)(knew + kb * 32 + kq * 8);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), qfr[kb], acc, 0, 0, 0);
    }
    if (lane < G) sfl[lane] = acc[0] * P.scale_log2;
  }
  lds_barrier();
  if (tid < G) {
    const int g = tid;
    float M = sfl[g];
    for (int ss = 0; ss < S; ++ss) M = fmaxf(M, msl[ss * 8 + g]);
    const float es = exp2_native(sfl[g] - M);
    float z = es;
    for (int ss = 0; ss < S; ++ss) {
      const float f = msl[ss * 8 + g] == -INFINITY ? 0.f : exp2_native(msl[ss * 8 + g] - M);
      fac[ss * 8 + g] = f;
      z += zsl[ss * 8 + g] * f;
    }
    const float inv = 1.0f / z;
    for (int ss = 0; ss < S; ++ss) fac[ss * 8 + g] *= inv;
    invl[g] = inv;
    psl[g] = es * inv;
    Mgl[g] = M;
  }
  lds_barrier();

  // ---- output: the S partial outputs brought to the common maximum and normalised, plus the token's own value
#pragma unroll
  for (int x = 0; x < OPT; ++x) {
    const int idx = tid + x * NT;
    if (idx < G * D) {
      const int g = idx / D, ch = idx % D;
      float o = 0.f;
#pragma unroll
      for (int ss = 0; ss < SH; ++ss) o = fmaf(ob[x][ss], ss < S ? fac[ss * 8 + g] : 0.f, o);
      for (int ss = SH; ss < S; ++ss) o = fmaf(ws_load1(part, (uint32_t)(ss * PART + 2 * G + idx)), fac[ss * 8 + g], o);
      const float vn = __uint_as_float(((uint32_t)((const uint16_t *)vnew)[ch]) << 16);
      o = fmaf(psl[g], vn, o);
      P.out[((size_t)uio * G + g) * D + ch] = o;
    }
  }

  // ---- record the row, update per-column aggregates, fused scores, local argmin (as the fused kernel does)
  float bF = INFINITY;
  int bP = -1, bC = -1;
  // (the same rules as in the fused kernel: see record4 in decode.h)
  auto record4 = [&](int j0, const float4 (&l4)[G], float4 nw_old, float4 sfx_old, int4 pj4, int phi, int rem) {
    float S4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float Mg = Mgl[g], ig = invl[g];
      S4[0] += exp2_native(l4[g].x - Mg) * ig; S4[1] += exp2_native(l4[g].y - Mg) * ig;
      S4[2] += exp2_native(l4[g].z - Mg) * ig; S4[3] += exp2_native(l4[g].w - Mg) * ig;
    }
    stg16_stream(ringu + (size_t)w * n_pad + j0, make_float4(S4[0], S4[1], S4[2], S4[3]));
    if (j0 < n_used) {
      float nwo[4] = {nw_old.x, nw_old.y, nw_old.z, nw_old.w};
      const float sfo[4] = {sfx_old.x, sfx_old.y, sfx_old.z, sfx_old.w};
      const int pj[4] = {pj4.x, pj4.y, pj4.z, pj4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = j0 + i;
        int d = wm1 - phi;
        d += d < 0 ? R : 0;
        const int age = p - 1 - pj[i];
        float so = (cum || pj[i] < 0 || d > age) ? 0.f : sfo[i];
        if (j >= turn0 && j < turn0 + turn_n) { nwo[i] = 0.f; so = turn[j - turn0]; }
        if (pj[i] == p - 1) nwo[i] = 0.f;  // born at the last step: what is stored is the former occupant's
        nwo[i] = fuse2(fusion, nwo[i], S4[i]);
        const bool cand = j < n_used && pj[i] >= 0 && pj[i] <= p - R;
        const float Fv = fuse2(fusion, so, nwo[i]);
        const float F = cand && Fv == Fv ? Fv : INFINITY;  // (not a number: counts as the largest, see decode.h)
        if (cand && P.dbgF) P.dbgF[(size_t)u * n_pad + j] = F;
        if (sel_step && j < n_used) { Fl[j] = F; Pl[j] = cand ? pj[i] : -1; }
        if (cand && cand_before(bF, bP, F, pj[i])) { bF = F; bP = pj[i]; bC = j; }
        ++rem;
        if (rem == cps) { rem = 0; ++phi; }
      }
      stg16_stream(nwu + j0, make_float4(nwo[0], nwo[1], nwo[2], nwo[3]));
    }
  };
  int cphi = (4 * tid) / cps, crem = (4 * tid) % cps;
  const int qstep = (4 * NT) / cps, rstep = (4 * NT) % cps;
  for (int jq = tid; jq < nq && !keep; jq += NT) {
    // the next group's loads go out before this group's arithmetic
    const int jn = jq + NT;
    float4 ln[G], an = make_float4(0.f, 0.f, 0.f, 0.f), bn = an;
    int4 pn = make_int4(-1, -1, -1, -1);
    if (jn < nq) {
#pragma unroll
      for (int g = 0; g < G; ++g) ln[g] = ws_load4(wts, (uint32_t)(g * n_pad + 4 * jn));
      if (4 * jn < n_used) {
        an = *(const float4 *)(nwu + 4 * jn);
        bn = *(const float4 *)(sfxu + (size_t)w * CsP + 4 * jn);
        pn = *(const int4 *)(posu + 4 * jn);
      }
    }
    record4(4 * jq, lq, nw0, sf0, pp0, cphi, crem);
    cphi += qstep;
    crem += rstep;
    if (crem >= cps) { crem -= cps; ++cphi; }
#pragma unroll
    for (int g = 0; g < G; ++g) lq[g] = ln[g];
    nw0 = an; sf0 = bn; pp0 = pn;
  }
  wave_argmin(bF, bP, bC);
  if (lane == 0) { bestF[wave] = bF; bestP[wave] = bP; bestC[wave] = bC; }
  if (turn_n > 0 && !keep) {
    const int rz = wm1, r0 = wm1 == 0 ? R - 1 : wm1 - 1;
    const int total = R * cpt;
    const int csh = P.cpt_shift;
    for (int idx = tid; idx < total; idx += NT) {
      const int i = csh >= 0 ? idx >> csh : idx / cpt, cc = idx - i * cpt;
      if (cc < turn_n) {
        int r = r0 - i;
        if (r < 0) r += R;
        const bool last = i == R - 1;
        sfxu[(size_t)(last ? rz : r) * CsP + turn0 + cc] = last ? 0.f : stage[idx];
      }
    }
  }
  lds_barrier();

  // ---- decision (wave 0)
  if (keep) {
    // every token is kept: the new one is appended (the host has made sure there is room)
    if (tid == 0) {
      sh[2] = n_used;
      sh[3] = -1;
      sh[4] = n_used + 1;
      sh[5] = 0;
      sh[6] = 0;
    }
  } else if (wave == 0) {
    float f = INFINITY;
    int bp = -1, bc = -1;
    if (lane < NW) { f = bestF[lane]; bp = bestP[lane]; bc = bestC[lane]; }
    wave_argmin(f, bp, bc);
    if (lane == 0) {
      const int older = n_used - n_holes + 1 - (p + 1 < R ? p + 1 : R);
      int dest = n_used, evicted = -1, nu = n_used + 1, multi = 0, nh = n_holes;
      if (Tev > 1) {
        if (sel_step && older > P.C) {
          multi = older - P.C;
          dest = -1; nu = n_used; nh = multi - 1;
        } else if (n_holes > 0) {
          dest = hole_top; nu = n_used; nh = n_holes - 1;
        }
      } else if (older > Cs && bc >= 0) {
        dest = bc; evicted = bp; nu = n_used;
      }
      if (dest >= n_pad) { dest = -1; nu = n_used; }
      sh[2] = dest;
      sh[3] = evicted;
      sh[4] = nu;
      sh[5] = multi;
      sh[6] = nh;
    }
  }

  // the decision is visible (nothing the commit below stores is an address the record phase has stored to)
  lds_barrier();
  if (tid == 0) P.sp_cnt[u] = 0;  // for the unit's next step

  StepTail<T> tc{P, u, tid, NT, NW, wave, lane, n_pad, n_used, p, w, Tev, sh, Fl, Pl, best2, nwu, posu, knew, vnew};
  coarse_select<T, D>(tc);
  commit_step<T, D, false>(tc);
}

}  // namespace mkv

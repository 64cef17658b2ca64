// Fused MorphKV decode step: one workgroup per unit (layer, sequence, KV head).
//
// Per unit and step (Eq.1, Algorithm 1, Eq.4-7):
//   K pass   : logits of the G query heads against every resident slot (wave-level split over slots)
//   softmax  : exact max / sum over slots + the token itself; weights stay in LDS
//   record   : S[j] = sum_g p_g[j] -> newest ring row; per-column running aggregate and fused score
//   V pass   : O_g = sum_j p_g[j] V_j + p_g[self] v_new
//   select   : evict argmin fused score among C older tokens + the token leaving the window
//              (ties evict the higher position), or append while fewer than C are held
//   compact  : token leaving the window takes the freed slot (K, V, position, its column of the R rows,
//              its aggregate state); the new token takes the window slot.
#pragma once
#include "common.h"

namespace mkv {

constexpr int META = 4;  // per unit: n_snap, next_pos, last_evicted, reserved

struct DecodeParams {
  void *K, *V;             // [U][n][D]
  int32_t *pos;            // [U][n]
  int32_t *meta;           // [U][META]
  float *ring;             // [U][R][n]   recorded rows, row index = query position mod R
  float *sfx;              // [U][R][Cs]  old-part aggregates (see column_scan)
  float *nw;               // [U][Cs]     new-part aggregates
  const void *q, *k_new, *v_new;
  float *out;
  float *dbgF;             // nullable: [U][Cs+1]
  int32_t Cs, R, n, Mq, Mkv, fusion, cps;
  float scale_log2;        // softmax scale * log2(e)
};

template <int G> struct GPad { static constexpr int v = G <= 1 ? 1 : G <= 2 ? 2 : G <= 4 ? 4 : 8; };

// LDS floats needed by decode_fused_kernel
inline size_t decode_lds_bytes(int n, int GPv, int G, int D, int NT, int R) {
  size_t lg = (size_t)n * GPv, om = (size_t)(NT / 64) * G * D;
  size_t fl = (lg > om ? lg : om) + 16 * 8 * 2 + 8 + (size_t)R + 16 * 3 + 8 + 4;
  return fl * 4;
}

template <typename T, int D, int G>
__global__ __launch_bounds__(1024) void decode_fused_kernel(DecodeParams P) {
  constexpr int EPL = Elem<T>::EPL, LPR = D / EPL, RPL = WAVE / LPR, UNR = 4, RPT = RPL * UNR;
  constexpr int GP = GPad<G>::v;
  static_assert(LPR <= WAVE && WAVE % LPR == 0, "row must fit a wave");
  extern __shared__ float smem[];

  const int u = blockIdx.x, tid = threadIdx.x, NT = blockDim.x, NW = NT / WAVE;
  const int wave = tid / WAVE, lane = tid % WAVE, chunk = lane % LPR, rowsub = lane / LPR;
  const int Cs = P.Cs, R = P.R, n = P.n, fusion = P.fusion;
  const int lb = u / P.Mkv, kh = u % P.Mkv;

  // ---- LDS carve-up
  const size_t lgsz = max((size_t)n * GP, (size_t)NW * G * D);
  float *lg = smem;                  // [n][GP] logits -> exp -> weights; later [NW][G][D] output partials
  float *red = lg + lgsz;            // [16][8]
  float *red2 = red + 16 * 8;        // [16][8]
  float *colv = red2 + 16 * 8 + 8;   // [R] column of the token leaving the window, oldest row first
  float *bestF = colv + R;           // [16]
  int *bestC = (int *)(bestF + 16);  // [16]
  int *bestP = bestC + 16;           // [16]
  int *sh = bestP + 16;              // [8]  2: dest slot, 3: evicted position
  float *shf = (float *)(sh + 8);    // [4]  0: weight of the new row on the token leaving the window

  const int32_t *meta = P.meta + (size_t)u * META;
  const int n_snap = meta[0], p = meta[1];
  const int w = p % R, nwin = p < R ? p : R;
  const bool win_full = p >= R;

  const T *Kb = (const T *)P.K + (size_t)u * n * D;
  const T *Vb = (const T *)P.V + (size_t)u * n * D;
  float *ringu = P.ring + (size_t)u * R * n;
  float *sfxu = P.sfx + (size_t)u * R * Cs;
  float *nwu = P.nw + (size_t)u * Cs;
  int32_t *posu = P.pos + (size_t)u * n;

  // ---- query fragments (pre-scaled so that weights are exp2 of the logit), self logit
  float qf[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const T *qp = (const T *)P.q + ((size_t)(lb * P.Mq + kh * G + g)) * D;
    uint4 r = ((const uint4 *)qp)[chunk];
    Elem<T>::unpack(r, qf[g]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[g][e] *= P.scale_log2;
  }
  float selfl[G];
  {
    uint4 r = ((const uint4 *)((const T *)P.k_new + (size_t)u * D))[chunk];
    float kf[EPL];
    Elem<T>::unpack(r, kf);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[e], d);
#pragma unroll
      for (int m = 1; m < LPR; m <<= 1) d += __shfl_xor(d, m);
      selfl[g] = d;
    }
  }

  // ---- columns whose turn it is: rebuild their aggregate state from the R rows of steps p-R .. p-1
  if (p >= 1) {
    const int phi = (p - 1) % R;
    for (int cc = tid; cc < P.cps; cc += NT) {
      const int c = phi * P.cps + cc;
      if (c < n_snap) {
        float nwv = column_scan(
            p - 1, p - 1, R, fusion, [&](int t) { return ringu[(size_t)pmod(t, R) * n + c]; },
            [&](int r, float x) { sfxu[(size_t)r * Cs + c] = x; });
        nwu[c] = nwv;
      }
    }
  }

  // ---- K pass
  float mx[G];
#pragma unroll
  for (int g = 0; g < G; ++g) mx[g] = -INFINITY;
  for (int tile = wave; tile * RPT < n; tile += NW) {
    uint4 r[UNR];
    bool ok[UNR];
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int j = tile * RPT + i * RPL + rowsub;
      ok[i] = j < n_snap || (j >= Cs && j < Cs + nwin);
      if (ok[i]) r[i] = ((const uint4 *)(Kb + (size_t)j * D))[chunk];
    }
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int j = tile * RPT + i * RPL + rowsub;
      float kf[EPL];
      if (ok[i]) Elem<T>::unpack(r[i], kf);
      float l[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
        if (ok[i]) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[e], d);
        }
#pragma unroll
        for (int m = 1; m < LPR; m <<= 1) d += __shfl_xor(d, m);
        l[g] = ok[i] ? d : -INFINITY;
        mx[g] = fmaxf(mx[g], l[g]);
      }
      if (chunk == 0 && j < n) {
#pragma unroll
        for (int g = 0; g < G; ++g) lg[(size_t)j * GP + g] = l[g];
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int m = LPR; m < WAVE; m <<= 1) mx[g] = fmaxf(mx[g], __shfl_xor(mx[g], m));
    if (lane == 0) red[wave * 8 + g] = mx[g];
  }
  __syncthreads();

  // ---- softmax: exact max, sum, weights
  float M[G], inv[G], pself[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float m = selfl[g];
    for (int x = 0; x < NW; ++x) m = fmaxf(m, red[x * 8 + g]);
    M[g] = m;
  }
  {
    float zs[G];
#pragma unroll
    for (int g = 0; g < G; ++g) zs[g] = 0.f;
    for (int j = tid; j < n; j += NT) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float e = exp2f(lg[(size_t)j * GP + g] - M[g]);
        lg[(size_t)j * GP + g] = e;
        zs[g] += e;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float s = wave_sum(zs[g]);
      if (lane == 0) red2[wave * 8 + g] = s;
    }
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float es = exp2f(selfl[g] - M[g]);
    float z = es;
    for (int x = 0; x < NW; ++x) z += red2[x * 8 + g];
    inv[g] = 1.0f / z;
    pself[g] = es * inv[g];
  }

  // ---- record the row, update per-column aggregates, fused scores, local argmin
  float bF = INFINITY;
  int bP = -1, bC = -1;
  for (int j = tid; j < n; j += NT) {
    float S = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float pg = lg[(size_t)j * GP + g] * inv[g];
      lg[(size_t)j * GP + g] = pg;
      S += pg;
    }
    ringu[(size_t)w * n + j] = S;
    if (j < n_snap) {
      const float nv = fuse2(fusion, nwu[j], S);
      nwu[j] = nv;
      const float F = fuse2(fusion, sfxu[(size_t)w * Cs + j], nv);
      if (P.dbgF) P.dbgF[(size_t)u * (Cs + 1) + j] = F;
      const int pj = posu[j];
      if (F < bF || (F == bF && pj > bP)) { bF = F; bP = pj; bC = j; }
    }
    if (j == Cs + w) shf[0] = S;
  }
  for (int a = tid; a < R - 1; a += NT) {
    const int t = p - R + 1 + a;
    colv[a] = win_full ? ringu[(size_t)pmod(t, R) * n + Cs + w] : 0.f;
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const float oF = __shfl_xor(bF, m);
    const int oP = __shfl_xor(bP, m), oC = __shfl_xor(bC, m);
    if (oF < bF || (oF == bF && oP > bP)) { bF = oF; bP = oP; bC = oC; }
  }
  if (lane == 0) { bestF[wave] = bF; bestP[wave] = bP; bestC[wave] = bC; }
  __syncthreads();

  // ---- V pass
  float acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  for (int tile = wave; tile * RPT < n; tile += NW) {
    uint4 r[UNR];
    bool ok[UNR];
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int j = tile * RPT + i * RPL + rowsub;
      ok[i] = j < n_snap || (j >= Cs && j < Cs + nwin);
      if (ok[i]) r[i] = ((const uint4 *)(Vb + (size_t)j * D))[chunk];
    }
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int j = tile * RPT + i * RPL + rowsub;
      if (ok[i]) {
        float vf[EPL];
        Elem<T>::unpack(r[i], vf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float pg = lg[(size_t)j * GP + g];
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pg, vf[e], acc[g][e]);
        }
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e)
#pragma unroll
      for (int m = LPR; m < WAVE; m <<= 1) acc[g][e] += __shfl_xor(acc[g][e], m);
  __syncthreads();  // every wave is done reading the weights: lg may be reused

  if (rowsub == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) lg[(size_t)(wave * G + g) * D + chunk * EPL + e] = acc[g][e];
  }
  // ---- decision (wave 0)
  if (wave == 0) {
    float fd = 0.f;  // fused score of the token leaving the window
    for (int a = lane; a < R; a += WAVE) {
      const float v = a == R - 1 ? shf[0] : colv[a];
      fd = fuse2(fusion, fd, v);
    }
    fd = fusion == 0 ? wave_sum(fd) : wave_max(fd);
    if (lane == 0) {
      colv[R - 1] = shf[0];
      int dest = -1, evicted = -1, ns = n_snap;
      if (win_full) {
        if (n_snap < Cs) {
          dest = n_snap;
          ns = n_snap + 1;
        } else {
          float f = bestF[0];
          int bp = bestP[0], bc = bestC[0];
          for (int x = 1; x < NW; ++x)
            if (bestF[x] < f || (bestF[x] == f && bestP[x] > bp)) { f = bestF[x]; bp = bestP[x]; bc = bestC[x]; }
          if (fd <= f) {  // tie: the token leaving the window has the higher position, it goes
            evicted = p - R;
          } else {
            dest = bc;
            evicted = bp;
          }
        }
        if (P.dbgF) P.dbgF[(size_t)u * (Cs + 1) + Cs] = fd;
      }
      sh[2] = dest;
      sh[3] = evicted;
      sh[4] = ns;
    }
  }
  __syncthreads();

  // ---- output
  for (int idx = tid; idx < G * D; idx += NT) {
    const int g = idx / D, ch = idx % D;
    float o = 0.f;
    for (int x = 0; x < NW; ++x) o += lg[(size_t)(x * G + g) * D + ch];
    float vn;
    {
      const T *vp = (const T *)P.v_new + (size_t)u * D;
      if constexpr (sizeof(T) == 4) vn = ((const float *)vp)[ch];
      else vn = __uint_as_float(((uint32_t)((const uint16_t *)vp)[ch]) << 16);
    }
    float ps = 0.f;
#pragma unroll
    for (int gg = 0; gg < G; ++gg) ps = gg == g ? pself[gg] : ps;
    o = fmaf(ps, vn, o);
    P.out[((size_t)(lb * P.Mq + kh * G + g)) * D + ch] = o;
  }

  // ---- compaction
  const int dest = sh[2];
  if (tid < 2 * LPR) {
    const int which = tid / LPR, ck = tid % LPR;
    T *base = (which ? (T *)P.V : (T *)P.K) + (size_t)u * n * D;
    const T *nsrc = (which ? (const T *)P.v_new : (const T *)P.k_new) + (size_t)u * D;
    uint4 *wslot = (uint4 *)(base + (size_t)(Cs + w) * D) + ck;
    if (dest >= 0) {
      const uint4 r = *wslot;
      ((uint4 *)(base + (size_t)dest * D))[ck] = r;
    }
    *wslot = ((const uint4 *)nsrc)[ck];
  }
  if (dest >= 0) {
    for (int a = tid; a < R; a += NT) ringu[(size_t)pmod(p - R + 1 + a, R) * n + dest] = colv[a];
    if (tid == NT - 1) {
      posu[dest] = p - R;
      const int p0 = last_rebuild_before(p, dest / P.cps, R);
      const float nwv = column_scan(
          p, p0, R, fusion, [&](int t) { return colv[t - (p - R + 1)]; },
          [&](int r, float x) { sfxu[(size_t)r * Cs + dest] = x; });
      nwu[dest] = nwv;
    }
  }
  if (tid == 0) {
    posu[Cs + w] = p;
    int32_t *m = P.meta + (size_t)u * META;
    m[0] = sh[4];
    m[1] = p + 1;
    m[2] = sh[3];
  }
}

}  // namespace mkv

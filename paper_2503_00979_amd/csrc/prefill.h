// Selection over the prompt (Section 4 "Implementation"; Eq.4-7): window-query softmax rows over the
// whole prompt, group sum (Algorithm 1), fusion over the rows, top-C with ties to the lower position,
// gather into cache slots, and the recorded rows / aggregate state the decode step continues from.
#pragma once
#include "common.h"
#include "decode.h"

namespace mkv {

struct PrefillParams {
  const void *Qw, *K, *V;  // [L][B][M][q_rows][D], [L][B][M'][Nmax][D] x2
  int32_t q_rows, q_prompt;  // rows per head in Qw; 0: row j is window query j (q_rows = R), 1: Qw holds every
                             // prompt position's query (q_rows = Nmax) and window query j is row N - min(R,N) + j
  const int32_t *plen;     // device [B]
  float *Srow;             // scratch [U][R][Nmax]: group-summed weights of window query j on key k
  const float *lse;        // nullable, [L][B][M][R]: natural-log sum of exp of the window rows' causal logits, from the caller
  float2 *Spart, *Sfin;    // scratch (bf16 passes): [U][nblk][G][R16] per-block and [U][G][R16] final softmax statistics
  float *F;                // scratch [U][Nmax]: fused score per older token
  int32_t *sel;            // scratch [U][Cs]: retained positions, ascending
  // state written
  void *Kc, *Vc;
  int32_t *pos, *meta;
  int32_t *evl;            // [U][T] positions evicted by the last step: none yet
  int32_t keep_all;        // a layer that keeps every token: no scores, no recorded rows; select keeps all, gather
  int32_t *sp_cnt;         // nullable, [U]: arrival counters of the split decode kernel, zeroed here
  float *ring, *sfx, *nw;
  int32_t B, Mq, Mkv, C, Cs, CsP, R, n, n_pad, Nmax, fusion, cps, T;
  float scale_log2;
};

// ---- P1: one workgroup per (window query j, unit): softmax statistics, then the group-summed row
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void prefill_rows_kernel(PrefillParams P) {
  constexpr int EPL = Elem<T>::EPL, LPR = D / EPL, RPL = WAVE / LPR, UNR = 4, RPT = RPL * UNR;
  __shared__ float sm[4][8], sz[4][8];
  const int j = blockIdx.x, u = blockIdx.y, tid = threadIdx.x, NW = blockDim.x / WAVE;
  const int wave = tid / WAVE, lane = tid % WAVE, chunk = lane % LPR, rowsub = lane / LPR;
  const int lb = u / P.Mkv, kh = u % P.Mkv, b = lb % P.B;
  const int N = P.plen[b], R = P.R, Rw = N < R ? N : R;
  if (j >= Rw) return;
  const int pj = N - Rw + j, nk = pj + 1;  // causal: keys 0..pj
  const T *Kb = (const T *)P.K + (size_t)u * P.Nmax * D;

  float qf[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const T *qp = (const T *)P.Qw + (((size_t)(lb * P.Mq + kh * G + g)) * P.q_rows + (P.q_prompt ? N - Rw : 0) + j) * D;
    uint4 r = ((const uint4 *)qp)[chunk];
    Elem<T>::unpack(r, qf[g]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[g][e] *= P.scale_log2;
  }

  auto logits = [&](int tile, float (&l)[UNR][G], bool (&ok)[UNR]) {
    uint4 r[UNR];
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int k = tile * RPT + i * RPL + rowsub;
      ok[i] = k < nk;
      if (ok[i]) r[i] = ((const uint4 *)(Kb + (size_t)k * D))[chunk];
    }
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      float kf[EPL];
      if (ok[i]) Elem<T>::unpack(r[i], kf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
        if (ok[i]) {
#pragma unroll
          for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[e], d);
        }
#pragma unroll
        for (int m = 1; m < LPR; m <<= 1) d += __shfl_xor(d, m);
        l[i][g] = d;
      }
    }
  };

  // pass A: running (max, sum of exp2) per head -- skipped when the caller brought the rows' log-sum-exp
  float m[G], z[G];
#pragma unroll
  for (int g = 0; g < G; ++g) { m[g] = -INFINITY; z[g] = 0.f; }
  for (int tile = wave; !P.lse && tile * RPT < nk; tile += NW) {
    float l[UNR][G];
    bool ok[UNR];
    logits(tile, l, ok);
#pragma unroll
    for (int i = 0; i < UNR; ++i)
      if (ok[i]) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float mn = fmaxf(m[g], l[i][g]);
          z[g] = z[g] * exp2f(m[g] - mn) + exp2f(l[i][g] - mn);
          m[g] = mn;
        }
      }
  }
  // merge row groups of the wave (lanes of one row group hold identical values), then the waves
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int s = LPR; s < WAVE; s <<= 1) {
      const float om = __shfl_xor(m[g], s), oz = __shfl_xor(z[g], s);
      const float mn = fmaxf(m[g], om);
      const float a = m[g] == -INFINITY ? 0.f : z[g] * exp2f(m[g] - mn);
      const float c = om == -INFINITY ? 0.f : oz * exp2f(om - mn);
      z[g] = a + c;
      m[g] = mn;
    }
    if (lane == 0) { sm[wave][g] = m[g]; sz[wave][g] = z[g]; }
  }
  __syncthreads();
  float Mx[G], inv[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mm = -INFINITY;
    for (int x = 0; x < NW; ++x) mm = fmaxf(mm, sm[x][g]);
    float zz = 0.f;
    for (int x = 0; x < NW; ++x) zz += sm[x][g] == -INFINITY ? 0.f : sz[x][g] * exp2f(sm[x][g] - mm);
    Mx[g] = mm;
    inv[g] = 1.0f / zz;
    if (P.lse) {
      Mx[g] = P.lse[((size_t)(lb * P.Mq + kh * G + g)) * R + j] * 1.4426950408889634f;
      inv[g] = 1.0f;
    }
  }
  // pass B: weights, summed over the group's heads
  float *Sr = P.Srow + ((size_t)u * R + j) * P.Nmax;
  for (int tile = wave; tile * RPT < nk; tile += NW) {
    float l[UNR][G];
    bool ok[UNR];
    logits(tile, l, ok);
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int k = tile * RPT + i * RPL + rowsub;
      if (ok[i] && chunk == 0) {
        float S = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) S += exp2f(l[i][g] - Mx[g]) * inv[g];
        Sr[k] = S;
      }
    }
  }
}

// ---- bf16, key-major passes ---------------------------------------------------------------------------
// The prompt-time selection needs the R window rows twice: once for their softmax statistics and once
// for the weights themselves.  Both passes walk the prompt in blocks of keys: a workgroup keeps 256 keys
// as MFMA A-operand fragments in registers (4 waves x 4 tiles of 16 keys) and streams every (query tile,
// head) of its unit past them, B fragments straight from the row-major window queries (they stay in L2).
// K is read from HBM once per pass and no row of weights is ever written out:
//   PF_STATS  per-block (max, sum of exp2) of every (head, query)      -> Spart, merged by prefill_stats_merge
//   PF_FUSE   weights -> sum over the group's heads -> fused over the R queries (Eq.4-6) -> F[key]
//   PF_RING   the same weights for the slots of the cache after the gather, stored as the recorded rows
// MFMA 16x16x32: D[key][query]; a lane owns one query (column) and 4 consecutive keys of each tile.
enum { PF_STATS = 0, PF_FUSE = 1, PF_RING = 2 };
constexpr int PF_KT = 4;                  // key tiles a wave holds
constexpr int PF_BLOCK = 4 * PF_KT * 16;  // keys (slots) per workgroup

template <int D, int G, int MODE>
__global__ __launch_bounds__(256, 2) void prefill_pass_kernel(PrefillParams P) {
  constexpr int KB = D / 32, KT = PF_KT;
  constexpr int JC = 16 / G;  // query tiles whose statistics are collected in LDS before they are flushed
  constexpr bool ST = MODE == PF_STATS;
  // the window queries of one query tile (16 queries x G heads), in B-fragment order, two buffers: the next
  // tile is fetched by the whole workgroup while the current one is worked on
  // rows of 16 pieces (one 8-channel group of the 16 queries) are 17 apart: the writes of a staging thread
  // row (one query, consecutive channel groups) then fall into different banks, as the reads do anyway
  constexpr int QROW = 17;
  __shared__ uint4 qs[2][G * KB * 4 * QROW];
  __shared__ float2 sts[2][ST ? 1 : G * 16];           // .x = log2-sum-exp of (head, query), what a weight's exponent is taken against
  __shared__ float2 wst[ST ? 4 : 1][ST ? G : 1][ST ? JC * 16 : 1];
  const int blk = blockIdx.x, u = blockIdx.y, tid = threadIdx.x;
  const int wave = tid / WAVE, lane = tid % WAVE, col = lane & 15, kq = lane >> 4;
  const int b = (u / P.Mkv) % P.B;
  const int N = P.plen[b], R = P.R, Rw = N < R ? N : R, n_old = N - Rw, R16 = (R + 15) & ~15;
  const int nkeys = MODE == PF_STATS ? N : MODE == PF_FUSE ? n_old : P.n_pad;
  if (blk * PF_BLOCK >= nkeys) return;
  const int kbase = blk * PF_BLOCK + wave * (KT * 16);
  const int njt = (Rw + 15) >> 4;
  const float scale = P.scale_log2;
  // keys below the window are seen by every window query: only a wave that reaches into the window masks
  [[maybe_unused]] const bool need_mask = kbase + KT * 16 > n_old;

  // ---- this wave's keys: A fragments (and, for cache slots, the positions behind them)
  uint4 ka[KT][KB];
  [[maybe_unused]] int4 kp[KT];
  if constexpr (MODE == PF_RING) {
    const bf16_t *Kc = (const bf16_t *)P.Kc + (size_t)u * P.n_pad * D;
    const int32_t *posu = P.pos + (size_t)u * P.n_pad;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      int tile = (kbase >> 4) + t;
      const bool tok = tile * 16 < P.n_pad;
      tile = tok ? tile : 0;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) ka[t][kb] = *(const uint4 *)(Kc + ((size_t)tile * KB + kb) * 512 + lane * 8);
      kp[t] = tok ? *(const int4 *)(posu + tile * 16 + 4 * kq) : make_int4(-1, -1, -1, -1);
    }
  } else {
    const bf16_t *Kb = (const bf16_t *)P.K + (size_t)u * P.Nmax * D;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const int key = min(kbase + t * 16 + col, N - 1);  // rows past the prompt are masked or never stored
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) ka[t][kb] = *(const uint4 *)(Kb + (size_t)key * D + kb * 32 + kq * 8);
    }
  }
  // rows of the recorded-row array that no window query maps to (prompt shorter than R) are zero
  if constexpr (MODE == PF_RING) {
    if (N < R) {
      const int s0 = blk * PF_BLOCK + lane * 4;
      if (s0 < P.n_pad)
        for (int r = N + wave; r < R; r += 4)
          *(float4 *)(P.ring + ((size_t)u * R + r) * P.n_pad + s0) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }

  // ---- staging of a query tile: thread -> (query jq, 8 channels c8) of every head; a row of 16 threads
  // reads one 256-byte query row, and the piece lands where lane (kq, jq) of k-block kb will look for it
  const bf16_t *Qu = (const bf16_t *)P.Qw + ((size_t)u * G * P.q_rows + (P.q_prompt ? N - Rw : 0)) * D;
  const float2 *stu = P.Sfin + (size_t)u * G * R16;
  constexpr int C8 = D / 8;                      // 16-byte pieces per query row
  constexpr int QPT = (16 * C8 + 255) / 256;     // query rows a thread fetches per head (1 for d <= 128)
  uint4 sq[G][QPT];
  [[maybe_unused]] float2 sst = make_float2(0.f, 0.f);
  // head g of query tile jt: global -> registers, and later registers -> LDS buffer.  The two halves are
  // called a few steps apart so that only a few heads are in registers at a time.
  auto fetch = [&](int jt, int g) {
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
      const int e = tid + qi * 256, jq = e / C8, c8 = e % C8, j = jt * 16 + jq;
      sq[g][qi] = make_uint4(0u, 0u, 0u, 0u);
      if (jq < 16 && j < Rw) sq[g][qi] = *(const uint4 *)(Qu + ((size_t)g * P.q_rows + j) * D + c8 * 8);
    }
  };
  auto stash = [&](int buf, int g) {
#pragma unroll
    for (int qi = 0; qi < QPT; ++qi) {
      const int e = tid + qi * 256, jq = e / C8, c8 = e % C8;
      if (jq < 16) qs[buf][(g * C8 + c8) * QROW + jq] = sq[g][qi];
    }
  };
  auto fetch_stats = [&](int jt) {
    if constexpr (!ST) {
      if (tid < G * 16) {
        const int g = tid >> 4, j = jt * 16 + (tid & 15);
        sst = j < Rw ? stu[g * R16 + j] : make_float2(INFINITY, 0.f);
      }
    }
  };
  auto stash_stats = [&](int buf) {
    if constexpr (!ST) {
      if (tid < G * 16) sts[buf][tid] = sst;
    }
  };

  [[maybe_unused]] float S[KT][4], Facc[KT][4];
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) { S[t][i] = 0.f; Facc[t][i] = 0.f; }

  // One step = (query tile jt, head g) against this wave's keys: 16 matrix instructions, then the arithmetic
  // on their 16 results per lane.  The two are software-pipelined: the matrix instructions of the next step
  // are issued before the arithmetic of the current one, so the matrix pipe works under it.
  auto ldq = [&](int buf, int g, uint4 (&q)[KB]) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) q[kb] = qs[buf][((g * KB + kb) * 4 + kq) * QROW + col];
  };
  // k-block outermost: consecutive matrix instructions belong to different key tiles and do not wait for
  // one another's result
  auto mfma16 = [&](const uint4 (&q)[KB], f32x4_t (&acc)[KT]) {
#pragma unroll
    for (int t = 0; t < KT; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int t = 0; t < KT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[t][kb]),
                                                         __builtin_bit_cast(bf16x8_t, q[kb]), acc[t], 0, 0, 0);
  };
  // asks the instruction scheduler to lay the region before it out as: one matrix instruction, then three
  // vector instructions (the fma / exp2 / fma of one result), and so on
  auto interleave = [&]() {
    if constexpr (!ST) {
      // the running sums are pinned here, so that the arithmetic above is not sunk past the next step's
      // matrix instructions
#pragma unroll
      for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(S[t][i]));
    }
#pragma unroll
    for (int i = 0; i < KT * KB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
    }
  };
  // st.x = log2-sum-exp of (head g, query j); +inf: no such query
  auto valu = [&](int jt, int g, float2 st, f32x4_t (&acc)[KT]) {
    const int j = jt * 16 + col;
    const int pj = j < Rw ? N - Rw + j : -1;  // causal: query j sees keys 0..pj
    if constexpr (ST) {
      // maximum on the raw products (the scale is positive), then one fma and one exp2 per logit
      float m = -INFINITY;
      if (need_mask) {
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int k = kbase + t * 16 + 4 * kq + i;
            acc[t][i] = k <= pj ? acc[t][i] : -INFINITY;
          }
      }
#pragma unroll
      for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) m = fmaxf(m, acc[t][i]);
      // one reference for the wave's 64 keys of this query (the 4 lanes that share the column), so that their
      // sums add up without rescaling
      m = fmaxf(m, __shfl_xor(m, 16));
      m = fmaxf(m, __shfl_xor(m, 32));
      m *= scale;
      const float mr = m == -INFINITY ? 0.f : m;
      float z = 0.f;
#pragma unroll
      for (int t = 0; t < KT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) z += __builtin_amdgcn_exp2f(fmaf(acc[t][i], scale, -mr));
      z += __shfl_xor(z, 16);
      z += __shfl_xor(z, 32);
      if (kq == 0) wst[wave][g][(jt % JC) * 16 + col] = make_float2(m, z);
    } else {
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        [[maybe_unused]] const int kpp[4] = {kp[t].x, kp[t].y, kp[t].z, kp[t].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float e = __builtin_amdgcn_exp2f(fmaf(acc[t][i], scale, -st.x));  // st.x = +inf: no such query, weight 0
          if constexpr (MODE == PF_RING) e = (kpp[i] >= 0 && kpp[i] < pj) ? e : 0.f;  // rows after the token's own
          S[t][i] += e;
        }
      }
      if (g == G - 1) {
        if constexpr (MODE == PF_FUSE) {
#pragma unroll
          for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) { Facc[t][i] = fuse2(P.fusion, Facc[t][i], S[t][i]); S[t][i] = 0.f; }
        } else {
          const int r = pj >= 0 ? pj % R : 0;
          float *row = P.ring + ((size_t)u * R + r) * P.n_pad;
#pragma unroll
          for (int t = 0; t < KT; ++t) {
            const int s0 = kbase + t * 16 + 4 * kq;
            if (pj >= 0 && s0 < P.n_pad) *(float4 *)(row + s0) = make_float4(S[t][0], S[t][1], S[t][2], S[t][3]);
#pragma unroll
            for (int i = 0; i < 4; ++i) S[t][i] = 0.f;
          }
        }
      }
    }
  };
  // statistics of query tiles [jt0, jt_end) (one chunk of JC at most): the 4 waves' shares merged, out to
  // the block's partials.  The caller's barrier has made the waves' shares visible.
  [[maybe_unused]] auto flush = [&](int jt_end) {
    const int jt0 = (jt_end - 1) / JC * JC, nj = (jt_end - jt0) * 16;
    float2 *part = P.Spart + ((size_t)u * gridDim.x + blk) * G * R16;
    for (int idx = tid; idx < G * nj; idx += 256) {
      const int g = idx / nj, jj = idx - g * nj;
      float m = -INFINITY, z = 0.f;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) {
        const float2 o = wst[wv][g][jj];
        const float mn = fmaxf(m, o.x), mnr = mn == -INFINITY ? 0.f : mn;
        z = z * __builtin_amdgcn_exp2f(m - mnr) + o.y * __builtin_amdgcn_exp2f(o.x - mnr);
        m = mn;
      }
      part[g * R16 + jt0 * 16 + jj] = make_float2(m, z);
    }
  };

#pragma unroll
  for (int g = 0; g < G; ++g) fetch(0, g);
  fetch_stats(0);
#pragma unroll
  for (int g = 0; g < G; ++g) stash(0, g);
  stash_stats(0);
  __syncthreads();
  // accumulators and query fragments of the step in flight and the one after it, used in turn
  f32x4_t aA[KT], aB[KT];
  uint4 qA[KB], qB[KB];
  ldq(0, 0, qA);
  mfma16(qA, aA);
  for (int jt = 0; jt < njt; ++jt) {
    const int buf = jt & 1;
    const bool more = jt + 1 < njt;
    // staging of the next tile: fetched now, written to its LDS buffer (not read since the last barrier) at
    // the end of this tile
    if (more) {
#pragma unroll
      for (int g = 0; g < G; ++g) fetch(jt + 1, g);
      fetch_stats(jt + 1);
    }
    if constexpr (G > 1) ldq(buf, 1, qB);
    // heads 0 .. G-2, two per trip: results of head g are in aA for even g, in aB for odd g
    constexpr int NP = (G - 1) / 2;
#pragma unroll 1
    for (int gp = 0; gp < NP; ++gp) {
      const int g = 2 * gp;
      {
        const float2 st = ST ? make_float2(0.f, 0.f) : sts[buf][g * 16 + col];
        mfma16(qB, aB);
        ldq(buf, g + 2, qA);  // g + 2 <= G - 1
        valu(jt, g, st, aA);
        interleave();
      }
      __builtin_amdgcn_sched_barrier(0);
      {
        const float2 st = ST ? make_float2(0.f, 0.f) : sts[buf][(g + 1) * 16 + col];
        mfma16(qA, aA);
        ldq(buf, g + 3 < G ? g + 3 : G - 1, qB);  // unconditional: the step stays one block of straight code
        valu(jt, g + 1, st, aB);
        interleave();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (((G - 1) & 1) != 0) {  // one more head before the last: G - 2 (even), results in aA
      const float2 st = ST ? make_float2(0.f, 0.f) : sts[buf][(G - 2) * 16 + col];
      mfma16(qB, aB);
      valu(jt, G - 2, st, aA);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
    }
    // last head: the next tile is staged first, so that its first step can be issued under this arithmetic
    const float2 st_last = ST ? make_float2(0.f, 0.f) : sts[buf][(G - 1) * 16 + col];
    if (more) {
#pragma unroll
      for (int g = 0; g < G; ++g) stash(buf ^ 1, g);
      stash_stats(buf ^ 1);
    }
    __syncthreads();  // next tile in place; every read of this one has been issued
    constexpr bool lastB = ((G - 1) & 1) != 0;  // where the results of head G-1 are
    if constexpr (lastB) {
      if (more) { ldq(buf ^ 1, 0, qA); mfma16(qA, aA); }
      valu(jt, G - 1, st_last, aB);
    } else {
      if (more) { ldq(buf ^ 1, 0, qB); mfma16(qB, aB); }
      valu(jt, G - 1, st_last, aA);
      if (more) {
#pragma unroll
        for (int t = 0; t < KT; ++t) aA[t] = aB[t];
      }
    }
    if constexpr (ST) {
      if ((jt + 1) % JC == 0 || !more) {
        __syncthreads();  // this chunk's shares are complete
        flush(jt + 1);
        __syncthreads();  // before the next chunk overwrites them
      }
    }
  }

  if constexpr (MODE == PF_FUSE) {
    // fuse over the 16 queries of a tile column: lanes of one row of 16 hold the same keys
    float *Fu = P.F + (size_t)u * P.Nmax;
#pragma unroll
    for (int t = 0; t < KT; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float f = Facc[t][i];
#pragma unroll
        for (int sft = 1; sft < 16; sft <<= 1) f = fuse2(P.fusion, f, __shfl_xor(f, sft));
        const int k = kbase + t * 16 + 4 * kq + i;
        if (col == 0 && k < n_old) Fu[k] = f;
      }
  }
}

// merges the per-block statistics of a unit: Sfin[g][j].x = max + log2(sum of exp2(logit - max)) over the
// whole causal row of query j (the row's log-sum-exp, base 2), +inf for queries that do not exist: a weight is
// exp2(logit - .x), one fma and one exp2, no multiplication by 1/sum
template <int G>
__global__ __launch_bounds__(64) void prefill_stats_merge_kernel(PrefillParams P, int nblk) {
  const int u = blockIdx.x, g = blockIdx.y, j = blockIdx.z * 64 + threadIdx.x;
  const int b = (u / P.Mkv) % P.B;
  const int N = P.plen[b], R = P.R, Rw = N < R ? N : R, R16 = (R + 15) & ~15;
  if (j >= R16) return;
  const int nb = (N + PF_BLOCK - 1) / PF_BLOCK, idx = g * R16 + j;
  float m = -INFINITY, z = 0.f;
  if (j < Rw) {
    for (int bk = 0; bk < nb; ++bk) {
      const float2 o = P.Spart[((size_t)u * nblk + bk) * G * R16 + idx];
      const float mn = fmaxf(m, o.x), mnr = mn == -INFINITY ? 0.f : mn;
      z = z * exp2f(m - mnr) + o.y * exp2f(o.x - mnr);
      m = mn;
    }
  }
  P.Sfin[(size_t)u * G * R16 + idx] = z > 0.f ? make_float2(m + log2f(z), 1.0f) : make_float2(INFINITY, 0.f);
}

// the same from the caller's log-sum-exp of the window rows (natural log, as attention kernels return it):
// weight = exp2(logit * scale_log2 - lse * log2(e))
template <int G>
__global__ __launch_bounds__(64) void prefill_stats_from_lse_kernel(PrefillParams P) {
  const int u = blockIdx.x, g = blockIdx.y, j = blockIdx.z * 64 + threadIdx.x;
  const int b = (u / P.Mkv) % P.B;
  const int N = P.plen[b], R = P.R, Rw = N < R ? N : R, R16 = (R + 15) & ~15;
  if (j >= R16) return;
  float2 st = make_float2(INFINITY, 0.f);
  if (j < Rw) st = make_float2(P.lse[((size_t)u * G + g) * R + j] * 1.4426950408889634f, 1.0f);
  P.Sfin[((size_t)u * G + g) * R16 + j] = st;
}

// source prompt position of cache slot `slot` of a unit after prefill, -1 if empty: the n_old retained older tokens
// first (ascending positions), the window's tokens after them (ascending), no gaps.  (A token never changes its
// slot afterwards: the decode step writes a new token into the slot its eviction has freed.)
__device__ inline int prefill_n_old(const PrefillParams &P, int N) {
  const int o = N - (N < P.R ? N : P.R);
  return o < P.C ? o : P.C;
}
__device__ inline int prefill_slot_source(const PrefillParams &P, int u, int slot, int N, int n_old) {
  if (slot < n_old) return P.sel[(size_t)u * P.Cs + slot];
  const int x = slot - n_old, Rw = N < P.R ? N : P.R;
  return x < Rw ? N - Rw + x : -1;
}

// ---- P4a: gather K/V rows and positions into the cache slots (layout of the element type);
// empty and padding slots are zero-filled so that a zero weight times their content stays zero
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_gather_kernel(PrefillParams P) {
  using L = Layout<T, D>;
  constexpr int EPL = Elem<T>::EPL, LPR = D / EPL;  // 16-byte pieces per row
  constexpr int SPB = 256 / (2 * LPR);              // slots per block
  const int u = blockIdx.y, tid = threadIdx.x;
  const int slot = blockIdx.x * SPB + tid / (2 * LPR), which = (tid / LPR) & 1, ck = tid % LPR;
  if (slot >= P.n_pad) return;
  const int b = (u / P.Mkv) % P.B, N = P.plen[b];
  const int n_snap = prefill_n_old(P, N);
  const int src = slot < P.n ? prefill_slot_source(P, u, slot, N, n_snap) : -1;
  if (which == 0 && ck == 0) P.pos[(size_t)u * P.n_pad + slot] = src;
  uint4 r = {0u, 0u, 0u, 0u};
  if (src >= 0) {
    const T *in = (which ? (const T *)P.V : (const T *)P.K) + ((size_t)u * P.Nmax + src) * D;
    r = ((const uint4 *)in)[ck];
  }
  T *outp = (which ? (T *)P.Vc : (T *)P.Kc) + (size_t)u * P.n_pad * D;
  const int ch0 = ck * EPL;
  if (which == 0) {
    *(uint4 *)(outp + L::k_off(slot, ch0)) = r;
  } else if constexpr (L::tiled) {
    const uint16_t *e = (const uint16_t *)&r;
#pragma unroll
    for (int i = 0; i < EPL; ++i) ((uint16_t *)outp)[L::v_off(slot, ch0 + i)] = e[i];
  } else {
    *(uint4 *)(outp + L::v_off(slot, ch0)) = r;
  }
}

// ---- P4a (bf16): the same through LDS, one workgroup per 32 slots: the rows come in as whole 2*D-byte reads,
// the tiles go out as what they are in memory -- two K tiles and one V tile, each contiguous -- in 16-byte stores
template <int D>
__global__ __launch_bounds__(256) void prefill_gather_tiled_kernel(PrefillParams P) {
  constexpr int C8 = D / 8;               // 16-byte pieces per row
  constexpr int KB = D / 32, CB = D / 16;
  constexpr int ROW = C8 + 1;             // LDS row stride in pieces (+1: the column reads below spread over the banks)
  __shared__ uint4 kr[32 * ROW], vr[32 * ROW];
  __shared__ int srcs[32];
  const int u = blockIdx.y, tid = threadIdx.x, slot0 = blockIdx.x * 32;
  const int b = (u / P.Mkv) % P.B, N = P.plen[b];
  const int n_snap = prefill_n_old(P, N);
  if (tid < 32) {
    const int slot = slot0 + tid;
    const int src = slot < P.n ? prefill_slot_source(P, u, slot, N, n_snap) : -1;
    srcs[tid] = src;
    P.pos[(size_t)u * P.n_pad + slot] = src;   // n_pad is a multiple of 32: the slot exists
  }
  __syncthreads();
  const bf16_t *Ku = (const bf16_t *)P.K + (size_t)u * P.Nmax * D;
  const bf16_t *Vu = (const bf16_t *)P.V + (size_t)u * P.Nmax * D;
  for (int e = tid; e < 32 * C8; e += 256) {
    const int row = e / C8, c8 = e % C8, src = srcs[row];
    uint4 k = {0u, 0u, 0u, 0u}, v = k;
    if (src >= 0) {
      k = *(const uint4 *)(Ku + (size_t)src * D + c8 * 8);
      v = *(const uint4 *)(Vu + (size_t)src * D + c8 * 8);
    }
    kr[row * ROW + c8] = k;
    vr[row * ROW + c8] = v;
  }
  __syncthreads();
  // K: tile t (16 slots), k-block kb: lane l = kq*16 + m holds channels kb*32 + kq*8 .. +8 of slot m
  bf16_t *Kc = (bf16_t *)P.Kc + (size_t)u * P.n_pad * D + (size_t)(slot0 / 16) * 16 * D;
  for (int e = tid; e < 2 * KB * 64; e += 256) {
    const int t = e / (KB * 64), kb = (e / 64) % KB, l = e % 64, kq = l >> 4, m = l & 15;
    *(uint4 *)(Kc + ((size_t)(t * KB + kb) * 64 + l) * 8) = kr[(t * 16 + m) * ROW + kb * 4 + kq];
  }
  // V: channel block cb: lane l = kq*16 + nn holds slots kq*8 .. +8 of channel cb*16 + nn
  bf16_t *Vc = (bf16_t *)P.Vc + (size_t)u * P.n_pad * D + (size_t)(slot0 / 32) * 32 * D;
  const uint16_t *vr16 = (const uint16_t *)vr;
  for (int e = tid; e < CB * 64; e += 256) {
    const int cb = e / 64, l = e % 64, kq = l >> 4, ch = cb * 16 + (l & 15);
    uint16_t x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = vr16[(size_t)((kq * 8 + i) * ROW) * 8 + ch];
    uint4 o;
    o.x = x[0] | ((uint32_t)x[1] << 16); o.y = x[2] | ((uint32_t)x[3] << 16);
    o.z = x[4] | ((uint32_t)x[5] << 16); o.w = x[6] | ((uint32_t)x[7] << 16);
    *(uint4 *)(Vc + ((size_t)cb * 64 + l) * 8) = o;
  }
}

}  // namespace mkv

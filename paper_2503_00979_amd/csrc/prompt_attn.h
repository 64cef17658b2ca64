// Causal attention over the whole prompt (Eq.1 at every prompt position, a token attends to itself) that also
// hands the window rows' softmax normalisers to the selection over the prompt (Eq.4-7): the statistics pass of
// that selection disappears, the prompt's keys are scored with the normalisers this pass has already made
// (the integration of selection with the attention kernel that Section 8, "Future Work", plans).
//
// bf16 in, fp32 accumulate, bf16 out, v_mfma_f32_32x32x16_bf16.  The work of one KV head is a list of tasks
// (32-row query block, query head of the group), row blocks outermost; a workgroup of 8 waves takes 8
// consecutive tasks, one per wave, whatever G is: every SIMD holds two waves, and every K/V tile staged in LDS
// is used by all 8 (they share the KV head; each wave follows its own causal limit).  A wave owns 32 rows of one
// head and keeps, per lane, ONE query column of the transposed problem
//     S^T[key][query] = K Q^T          (A = keys from LDS, B = the wave's query fragments, in registers)
//     O^T[dv][query] += V^T P^T        (A = values from LDS through the transposing read, B = the exponentials)
// so the results of the first product are, as they lie in registers, the B operand of the second, and the row
// statistics (running maximum, running sum) are per-lane scalars shared by the two lanes l and l+32.
#pragma once
#include "common.h"

namespace mkv {

typedef __bf16 pa_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 pa_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pa_f32x16 __attribute__((ext_vector_type(16)));
typedef float pa_f32x2 __attribute__((ext_vector_type(2)));
typedef short pa_s16x4 __attribute__((ext_vector_type(4)));
typedef short pa_s16x8 __attribute__((ext_vector_type(8)));
typedef pa_s16x4 __attribute__((address_space(3))) pa_lds_s16x4;

struct PromptAttnParams {
  const bf16_t *Q, *K, *V;  // [L][B][M][Nmax][D], [L][B][M'][Nmax][D] x2
  bf16_t *O;                // [L][B][M][Nmax][D]; rows at or beyond a sequence's prompt length are not written
  float *lse;               // nullable, [L][B][M][Nmax]: natural-log sum of exp of each row's causal logits
  float *lse_w;             // [L][B][M][R]: the same for the last min(R, N) rows (row j = position N - min(R,N) + j)
  const int32_t *plen;      // device [B]
  int32_t B, Mq, Mkv, R, Nmax;
  float scale_log2;         // softmax scale * log2(e), > 0
};

template <int D, int G>
struct PromptAttnCfg {
  static constexpr int NWV = 8, NT = NWV * 64;    // tasks (waves) per workgroup
  static constexpr int BN = 64;                  // keys per tile
  static constexpr int NSUB = 2, NBUF = 2 * NSUB; // tiles per barrier; tile buffers in LDS
  static constexpr int KS = D / 16, DB = D / 32, C8 = D / 8;
  static constexpr int KROW = D + 8;             // bf16 per K row in LDS: 16-byte reads of 16 rows hit 64 distinct banks
  static constexpr int VROW = D + 32;            // bf16 per V row in LDS: 4 consecutive rows start 16 banks apart, so
                                                 // the 4-key x 16-channel blocks of a transposing read (two per
                                                 // 32 lanes) cover all 64 banks
  static constexpr int K_ITEMS = BN * C8;        // 16-byte pieces of a K tile, and of a V tile
  static constexpr int KI = (K_ITEMS + NT - 1) / NT;
  static constexpr size_t lds_bytes = (size_t)NBUF * BN * (KROW + VROW) * 2;
};

template <int D, int G>
__global__ __launch_bounds__((PromptAttnCfg<D, G>::NT)) void prompt_attn_kernel(PromptAttnParams P) {
  using Cf = PromptAttnCfg<D, G>;
  constexpr int NT = Cf::NT, NWV = Cf::NWV, BN = Cf::BN, KS = Cf::KS, DB = Cf::DB, C8 = Cf::C8;
  constexpr int KROW = Cf::KROW, VROW = Cf::VROW, KI = Cf::KI, NSUB = Cf::NSUB, NBUF = Cf::NBUF;
  extern __shared__ __align__(16) unsigned char pa_smem[];
  bf16_t *Ks = (bf16_t *)pa_smem;        // [NBUF][BN][KROW]
  bf16_t *Vs = Ks + NBUF * BN * KROW;    // [NBUF][BN][VROW], row-major like K

  const int tid = threadIdx.x, wave = tid / WAVE, lane = tid % WAVE, h = lane / 32, col = lane % 32;
  const int u = blockIdx.y, lb = u / P.Mkv, kh = u % P.Mkv, b = lb % P.B;
  const int N = P.plen[b];
  // long rows first: the last workgroups to start are the short ones
  const int task0 = (int)(gridDim.x - 1 - blockIdx.x) * NWV;
  if ((task0 / G) * 32 >= N) return;  // the first task's rows are past the prompt, and so are the others'
  const int task = task0 + wave, g = task % G, qs = (task / G) * 32;
  const bool wave_on = qs < N;
  const int query = qs + col;
  const int qm = min(query, N - 1);        // rows past the prompt repeat the last row and are never stored
  const int q_lo = min(qs, N - 1), q_hi = min(qs + 31, N - 1);
  const int ntile = min(((task0 + NWV - 1) / G) * 32 + 31, N - 1) / BN + 1;  // up to the last task's last row
  const bf16_t *Kb = P.K + (size_t)u * P.Nmax * D, *Vb = P.V + (size_t)u * P.Nmax * D;
  const size_t head = (size_t)lb * P.Mq + (size_t)kh * G + g;

  // the wave's queries as B fragments: lane (h, col) holds channels 16s + 8h .. +8 of row qs + col
  pa_bf16x8 qf[KS];
  {
    const bf16_t *qrow = P.Q + (head * P.Nmax + qm) * D;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = __builtin_bit_cast(pa_bf16x8, *(const uint4 *)(qrow + 16 * s + 8 * h));
  }

  pa_f32x16 Oacc[DB];
#pragma unroll
  for (int blk = 0; blk < DB; ++blk)
#pragma unroll
    for (int v = 0; v < 16; ++v) Oacc[blk][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;  // log2 domain; l_run is this lane's share of the row sum

  // Trip t works on tile t out of LDS buffer t % NBUF while tile t + NSUB travels global -> registers (issued
  // before the arithmetic) -> its buffer (after it); the first NSUB trips only stage.  One barrier every NSUB
  // trips: between the trip that writes a buffer and the trips that read it, and between the trips that read
  // it and the next trip that overwrites it (NBUF = 2 NSUB trips apart), lies a trip that ends in a barrier.
  for (int t = -NSUB; t < ntile; ++t) {
    const int buf = (t + NBUF) % NBUF, nbuf = (t + NSUB + NBUF) % NBUF, kb = t * BN;
    const bool more = t + NSUB < ntile;
    uint4 kr[KI], vr[KI];
    if (more) {
      const int kn = kb + NSUB * BN;
#pragma unroll
      for (int i = 0; i < KI; ++i) {
        const int e = tid + i * NT;
        kr[i] = make_uint4(0u, 0u, 0u, 0u);
        if (Cf::K_ITEMS % NT == 0 || e < Cf::K_ITEMS) {
          // (32-bit offsets from the unit's base: a thread keeps no 64-bit address per piece)
          const uint32_t row = (uint32_t)min(kn + e / C8, N - 1);  // rows past the prompt are masked below
          kr[i] = *(const uint4 *)(Kb + (row * (uint32_t)D + (uint32_t)(e % C8) * 8u));
          // a value row past the prompt is taken as zero: a zero weight must not meet a NaN
          vr[i] = make_uint4(0u, 0u, 0u, 0u);
          if (kn + e / C8 < N) vr[i] = *(const uint4 *)(Vb + (row * (uint32_t)D + (uint32_t)(e % C8) * 8u));
        }
      }
    }
    if (t >= 0 && wave_on && kb <= q_hi) {
      pa_f32x16 s[2];
#pragma unroll
      for (int hk = 0; hk < 2; ++hk)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[hk][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int hk = 0; hk < 2; ++hk) {
          const pa_bf16x8 a = __builtin_bit_cast(
              pa_bf16x8, *(const uint4 *)(Ks + (buf * BN + 32 * hk + col) * KROW + 16 * ks + 8 * h));
          s[hk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[hk], 0, 0, 0);
        }
      // register v of lane (h, col): key kb + 32 hk + 8 (v / 4) + 4 h + v % 4, query qs + col
      if (kb + BN - 1 > q_lo) {
#pragma unroll
        for (int hk = 0; hk < 2; ++hk)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = kb + 32 * hk + 8 * (v / 4) + 4 * h + (v % 4);
            s[hk][v] = key <= qm ? s[hk][v] : -INFINITY;
          }
      }
      // (four partial maxima and sums: short dependency chains)
      float mx4[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
      for (int hk = 0; hk < 2; ++hk)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx4[v & 3] = fmaxf(mx4[v & 3], s[hk][v]);
      float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
      {
        // the other half-wave's maximum for the same row, by a register swap between the halves (no LDS trip):
        // afterwards the two results hold (low half's, high half's) value in every lane
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * P.scale_log2;
      }
      // The reference only moves when the row's maximum has outgrown it by 2^8 (any reference gives the same
      // quotient; the exponentials stay below 2^8, far from any overflow): the accumulators are rescaled a
      // few times per row instead of at every new maximum.  Finite from the first tile on: key 0 is visible
      // to every row.
      const float m_new = mx > m_run + 8.0f ? mx : m_run;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      float ls4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int hk = 0; hk < 2; ++hk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s[hk][v] = __builtin_amdgcn_exp2f(fmaf(s[hk][v], P.scale_log2, -m_new));
          ls4[v & 3] += s[hk][v];
        }
      l_run = l_run * alpha + ((ls4[0] + ls4[1]) + (ls4[2] + ls4[3]));
      m_run = m_new;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int blk = 0; blk < DB; ++blk)
#pragma unroll
          for (int v = 0; v < 16; ++v) Oacc[blk][v] *= alpha;
      }
      // lane a of a 16-lane group points at key a / 4 of its 4-key block and at channels 4 (a % 4) .. +3 of the
      // group's 16 channels; the second half-wave takes the keys 4 further on
      const bf16_t *vtr = Vs + (buf * BN + 4 * h + (lane % 16) / 4) * VROW + 16 * ((lane % 32) / 16) + 4 * (lane % 4);
#pragma unroll
      for (int hk = 0; hk < 2; ++hk)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          pa_bf16x8 pf;
#pragma unroll
          for (int j = 0; j < 8; j += 2) {
            const pa_f32x2 two = {s[hk][8 * m + j], s[hk][8 * m + j + 1]};
            const pa_bf16x2 r = __builtin_convertvector(two, pa_bf16x2);
            pf[j] = r[0];
            pf[j + 1] = r[1];
          }
#pragma unroll
          for (int blk = 0; blk < DB; ++blk) {
            // A fragment = V^T: channel 32 blk + lane % 32, keys 32 hk + 16 m + 8 b + 4 h + (0..3) for b = 0, 1.
            // One transposing read hands each lane of a 16-lane group one channel of a 4-key x 16-channel block.
            const bf16_t *vp = vtr + (32 * hk + 16 * m) * VROW + 32 * blk;
            const pa_s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pa_lds_s16x4 *)vp);
            const pa_s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pa_lds_s16x4 *)(vp + 8 * VROW));
            const pa_s16x8 a8 = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            const pa_bf16x8 a = __builtin_bit_cast(pa_bf16x8, a8);
            Oacc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, Oacc[blk], 0, 0, 0);
          }
        }
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < KI; ++i) {
        const int e = tid + i * NT;
        if (Cf::K_ITEMS % NT == 0 || e < Cf::K_ITEMS) {
          *(uint4 *)(Ks + (nbuf * BN + e / C8) * KROW + (e % C8) * 8) = kr[i];
          *(uint4 *)(Vs + (nbuf * BN + e / C8) * VROW + (e % C8) * 8) = vr[i];
        }
      }
    }
    if ((t + 1) % NSUB == 0) __syncthreads();
  }

  if (!wave_on) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (query >= N) return;
  const float inv = 1.0f / l_tot;
  bf16_t *orow = P.O + (head * P.Nmax + query) * D;
#pragma unroll
  for (int blk = 0; blk < DB; ++blk)
#pragma unroll
    for (int b4 = 0; b4 < 4; ++b4) {
      // registers 4 b4 .. +4 are channels 32 blk + 8 b4 + 4 h .. +4 of this lane's row
      const pa_f32x2 lo = {Oacc[blk][4 * b4] * inv, Oacc[blk][4 * b4 + 1] * inv};
      const pa_f32x2 hi = {Oacc[blk][4 * b4 + 2] * inv, Oacc[blk][4 * b4 + 3] * inv};
      uint2 w;
      w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, pa_bf16x2));
      w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, pa_bf16x2));
      *(uint2 *)(orow + 32 * blk + 8 * b4 + 4 * h) = w;
    }
  if (h == 0) {
    const float lse = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;  // log2 domain -> natural log
    if (P.lse) P.lse[head * P.Nmax + query] = lse;
    const int Rw = min(P.R, N), j = query - (N - Rw);
    if (j >= 0) P.lse_w[head * P.R + j] = lse;
  }
}

}  // namespace mkv

// Fused MorphKV decode step: one workgroup per unit (layer, sequence, KV head).
//
// Per unit and step (Eq.1, Algorithm 1, Eq.4-7):
//   K pass   : logits of the G query heads against every resident slot; waves take slot tiles from a
//              shared counter, so the pass is a wave-level split over the cache
//   softmax  : exact max / sum over slots + the token itself; fp32 weights stay in LDS
//   record   : S[j] = sum_g p_g[j] -> newest ring row; per-column running aggregate and fused score
//   V pass   : O_g = sum_j p_g[j] V_j + p_g[self] v_new
//   select   : evict argmin fused score among the tokens that are older than the window once the new one is in
//              (ties evict the higher position), while more than C of them are held
//   commit   : the new token takes the slot the eviction has freed (or the next unused one).  No token ever
//              changes its slot: "older" is decided by position, every slot is a column of the score state
//              from its occupant's birth, and rows recorded before that are masked where the column is rebuilt.
//
// Two data paths:
//   bf16 : K and V live in MFMA-operand tile order (see Layout<bf16_t, D>) so that a wave reads 1 KB
//          contiguous per load and feeds v_mfma_f32_16x16x32_bf16 directly: the matrix core makes the
//          arithmetic free next to the HBM stream -- the bound stays HBM.
//   fp32 : row-major K/V, plain fp32 FMAs (small/toy configurations).
//
// Timeline of a workgroup: the HBM stream (K tiles, then V tiles) is the critical path; some waves (the
// host says how many) spend the start of the K pass rebuilding the aggregate state of the columns whose
// turn it is; the first V tile of every wave is already in flight while the softmax runs.
#pragma once
#include "common.h"

namespace mkv {

// per unit: 0 slots in use (high-water mark: slots below it hold a token or are free again), 1 next position,
// 2 last evicted position, 3 next position mod R, 4 prompt length, 5 free slots below the mark (coarse schedule), 2 unused
constexpr int META = 8;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

struct DecodeParams {
  void *K, *V;             // per unit n_pad * D elements, layout by element type (see Layout<>)
  int32_t *pos;            // [U][n_pad]
  int32_t *meta;           // [U][META]
  float *ring;             // [U][R][n_pad]  recorded rows, row index = query position mod R
  float *sfx;              // [U][R][CsP]    old-part aggregates (see column_scan); CsP = n_pad: every slot is a column
  float *nw;               // [U][CsP]       new-part aggregates
  const void *q, *k_new, *v_new;
  float *out;
  float *dbgF;             // nullable: [U][n_pad] fused score of every eviction candidate, by slot
  long long *dbgT;         // nullable: [U][8] phase time stamps (diagnostics)
  int32_t Cs, CsP, R, n, n_pad, Mq, Mkv, fusion, cps, cpt;
  int32_t cpt_shift;       // log2(cpt) if cpt is a power of two, else -1
  int32_t C, T;            // older tokens kept by a selection; selection every T steps (Appendix A.5), Cs = C+T-1
  int32_t *evl;            // [U][T] positions evicted by the last step, -1 padded
  int32_t *holes;          // [U][T] coarse schedule: slots below the high-water mark that are free (a stack, meta[5] deep)
  int32_t zig;             // parity of the step count: direction of the walk over the cache
  // split kernel only (decode_split.h): workspace of the partial results and the arrival counters
  float *sp_part;          // [U][sp_smax][2G + G*D] local maximum, local sum, partial output per workgroup
  float *sp_w;             // [U][G][n_pad] logits of the step
  int32_t *sp_cnt;         // [U] workgroups of the unit that have finished their share (0 between launches)
  int32_t sp_bps, sp_smax; // blocks of 32 slots per workgroup; record stride of sp_part
  int32_t keep_all;        // a layer that keeps every token (Appendix A.6): nothing is recorded, fused or selected;
                           // every new token is appended
  int32_t nt_k, nt_v;      // K tile groups [0, nt_k) and V tiles [0, nt_v) of every unit are loaded with the
                           // non-temporal hint (they stream from HBM); the rest is meant to stay cache-resident
  int32_t keep_cached_blocks;  // decode_keep_kernel: a unit's newest blocks of 32 slots that are read with ordinary loads
                           // (meant to stay in the memory-side cache); older blocks stream with the non-temporal hint
  int32_t rb_gw, rb_nrw;   // fused kernel: columns per group of the rebuild (turn_group_width) and the number of waves
                           // that rebuild, worked out by the host for the launch's workgroup size
  int32_t u0;              // first unit of the launch (a launch may cover one layer's units only)
  int32_t io_u0;           // unit whose rows come first in q, k_new, v_new and out (u0 when the step's tensors
                           // are one layer's own, 0 when they cover the whole model)
  float scale_log2;        // softmax scale * log2(e)
};

// ---- cache layouts -----------------------------------------------------------------------------------
// Element offset of (slot j, channel ch) inside one unit's K or V array of n_pad slots.
template <typename T, int D> struct Layout;

// fp32: row-major [slot][channel]
template <int D> struct Layout<float, D> {
  static constexpr bool tiled = false;
  static constexpr int KB = 1, CB = 1;
  __device__ __host__ static inline size_t k_off(int j, int ch) { return (size_t)j * D + ch; }
  __device__ __host__ static inline size_t v_off(int j, int ch) { return (size_t)j * D + ch; }
};

// bf16: MFMA 16x16x32 operand order.
//  K: tiles of 16 slots; inside a tile [k-block of 32 channels][8-channel group kq][slot m][8 channels]:
//     lane l = kq*16 + m of a wave reads its A-operand fragment of k-block kb at tile + kb*512 + l*8.
//  V: tiles of 32 slots; inside a tile [16-channel block cb][8-slot group kq][channel nn][8 slots]:
//     lane l = kq*16 + nn reads its B-operand fragment of channel block cb at tile + cb*512 + l*8.
template <int D> struct Layout<bf16_t, D> {
  static constexpr bool tiled = true;
  static constexpr int KB = D / 32, CB = D / 16;
  __device__ __host__ static inline size_t k_off(int j, int ch) {
    return ((((size_t)(j >> 4) * KB + (ch >> 5)) * 4 + ((ch & 31) >> 3)) * 16 + (j & 15)) * 8 + (ch & 7);
  }
  __device__ __host__ static inline size_t v_off(int j, int ch) {
    return ((((size_t)(j >> 5) * CB + (ch >> 4)) * 4 + ((j & 31) >> 3)) * 16 + (ch & 15)) * 8 + (j & 7);
  }
};

constexpr int MAXQ = 1;  // groups of 4 columns per thread whose state is prefetched before the K pass

// columns rebuilt per step, padded the way the staging area lays them out
__host__ __device__ inline int turn_cols_padded(int cps) {
  if (cps <= 64) { int c = 1; while (c < cps) c <<= 1; return c; }
  return (cps + 63) / 64 * 64;
}

// LDS bytes of decode_fused_kernel
inline size_t decode_lds_bytes(int n_pad, int G, int D, int NT, int R, int cps, int CsP, int T) {
  const size_t lg = (size_t)G * (n_pad + 4), om = (size_t)(NT / 64) * G * D;
  const size_t cpt = (size_t)turn_cols_padded(cps);
  size_t fl = (lg > om ? lg : om) + (size_t)R * cpt /*stage*/ + cpt /*turn*/ + 16 * 8 * 2 + 16 * 3 + 16 + 8 + 16;
  if (T > 1) fl += 2 * (size_t)CsP /*scores, positions*/ + 2 * 3 * 16 /*per-wave minima, two sets*/ + (size_t)n_pad / 32 /*free-slot bits*/;
  return fl * 4;
}

// slots below the high-water mark hold a token (or, under the coarse schedule, are free again: those are masked
// through a bit map of the free slots, see free_slot_bits)
__device__ inline bool slot_valid(int j, int n_used) { return j < n_used; }

// Coarse schedule: the slots a selection has freed and no token has taken yet still hold their old keys.  Their
// logits must not take part in the softmax at all (not even in its maximum), so the workgroup keeps one bit per slot
// in LDS: thread i makes word i from the unit's list of free slots (at most T - 1 <= 63 entries, uniform loads).
// The caller puts a barrier between this and the first use.
__device__ inline void free_slot_bits(unsigned *bits, int n_pad, const int32_t *holes, int n_holes, int tid, int NT) {
  for (int i = tid; i < n_pad / 32; i += NT) {
    unsigned wbits = 0u;
    for (int k = 0; k < n_holes; ++k) {
      const int h = holes[k];
      wbits |= (h >> 5) == i ? 1u << (h & 31) : 0u;
    }
    bits[i] = wbits;
  }
}
// bit i of the result: slot j0 + i is free (j0 a multiple of 4)
__device__ inline unsigned free_bits4(const unsigned *bits, int j0) { return (bits[j0 >> 5] >> (j0 & 31)) & 15u; }

// 16-byte global load; STREAM: with the non-temporal hint (the line is not kept in the caches it passes)
template <bool STREAM> __device__ inline uint4 ldg16(const void *p) {
  if constexpr (STREAM) {
    typedef unsigned int u4v __attribute__((ext_vector_type(4)));
    const u4v t = __builtin_nontemporal_load((const u4v *)p);
    return make_uint4(t.x, t.y, t.z, t.w);
  } else {
    return *(const uint4 *)p;
  }
}

// 16-byte global store with the non-temporal hint: for data this launch does not read again (the recorded row,
// the running aggregates), so that it leaves the L2 as it is written instead of in a burst when the kernel ends
__device__ inline void stg16_stream(float *p, float4 v) {
  typedef float f4v __attribute__((ext_vector_type(4)));
  const f4v t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, (f4v *)p);
}

// workgroup barrier that orders LDS traffic only: outstanding global loads/stores stay in flight
__device__ inline void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ---- wave reductions on DPP (no LDS traffic) ---------------------------------------------------------
template <int CTRL> __device__ inline float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL> __device__ inline int dpp_mov_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;
__device__ inline float lane_bcast(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ inline float wave_sum_dpp(float v) {
  v += dpp_mov<DPP_XOR1>(v); v += dpp_mov<DPP_XOR2>(v); v += dpp_mov<DPP_HALF_MIRROR>(v); v += dpp_mov<DPP_MIRROR>(v);
  return (lane_bcast(v, 0) + lane_bcast(v, 16)) + (lane_bcast(v, 32) + lane_bcast(v, 48));
}
__device__ inline float wave_max_dpp(float v) {
  v = fmaxf(v, dpp_mov<DPP_XOR1>(v)); v = fmaxf(v, dpp_mov<DPP_XOR2>(v));
  v = fmaxf(v, dpp_mov<DPP_HALF_MIRROR>(v)); v = fmaxf(v, dpp_mov<DPP_MIRROR>(v));
  return fmaxf(fmaxf(lane_bcast(v, 0), lane_bcast(v, 16)), fmaxf(lane_bcast(v, 32), lane_bcast(v, 48)));
}
// maximum over the lanes l, l ^ 16, l ^ 32, l ^ 48 (same column of the four rows of 16), in every lane: the two
// row-swap instructions of this device give a lane its partner row's value without a trip through LDS
__device__ inline float max_over_rows(float v) {
  const int b = __builtin_bit_cast(int, v);
  const auto a = __builtin_amdgcn_permlane16_swap(b, b, false, false);   // a[0]: even row's value, a[1]: odd row's
  v = fmaxf(__builtin_bit_cast(float, (int)a[0]), __builtin_bit_cast(float, (int)a[1]));
  const int c = __builtin_bit_cast(int, v);
  const auto d = __builtin_amdgcn_permlane32_swap(c, c, false, false);   // d[0]: lower half's value, d[1]: upper's
  return fmaxf(__builtin_bit_cast(float, (int)d[0]), __builtin_bit_cast(float, (int)d[1]));
}
__device__ inline float sum_over_rows(float v) {
  const int b = __builtin_bit_cast(int, v);
  const auto a = __builtin_amdgcn_permlane16_swap(b, b, false, false);
  v = __builtin_bit_cast(float, (int)a[0]) + __builtin_bit_cast(float, (int)a[1]);
  const int c = __builtin_bit_cast(int, v);
  const auto d = __builtin_amdgcn_permlane32_swap(c, c, false, false);
  return __builtin_bit_cast(float, (int)d[0]) + __builtin_bit_cast(float, (int)d[1]);
}
constexpr int DPP_ROW_ROR8 = 0x128;  // lane l of a row of 16 reads lane (l + 8) mod 16
// eviction candidate order: does (of, op) go before (f, p)?  smaller score first, on equal score the
// higher position
__device__ inline bool cand_before(float f, int p, float of, int op) { return of < f || (of == f && op > p); }
template <int CTRL> __device__ inline void argmin_step(float &f, int &p, int &c) {
  const float of = dpp_mov<CTRL>(f);
  const int op = dpp_mov_i<CTRL>(p), oc = dpp_mov_i<CTRL>(c);
  if (cand_before(f, p, of, op)) { f = of; p = op; c = oc; }
}
// the candidate that goes first among a lane's row partners (SWAP32: the two halves of the wave, else the even and
// the odd row of each half); every lane ends up with the winner
template <bool SWAP32> __device__ inline void argmin_rows(float &f, int &p, int &c) {
  const int fb = __builtin_bit_cast(int, f);
  const auto F = SWAP32 ? __builtin_amdgcn_permlane32_swap(fb, fb, false, false) : __builtin_amdgcn_permlane16_swap(fb, fb, false, false);
  const auto Pp = SWAP32 ? __builtin_amdgcn_permlane32_swap(p, p, false, false) : __builtin_amdgcn_permlane16_swap(p, p, false, false);
  const auto Cc = SWAP32 ? __builtin_amdgcn_permlane32_swap(c, c, false, false) : __builtin_amdgcn_permlane16_swap(c, c, false, false);
  const float f0 = __builtin_bit_cast(float, (int)F[0]), f1 = __builtin_bit_cast(float, (int)F[1]);
  const bool second = cand_before(f0, (int)Pp[0], f1, (int)Pp[1]);
  f = second ? f1 : f0;
  p = second ? (int)Pp[1] : (int)Pp[0];
  c = second ? (int)Cc[1] : (int)Cc[0];
}
__device__ inline void wave_argmin(float &f, int &p, int &c) {
  argmin_step<DPP_XOR1>(f, p, c); argmin_step<DPP_XOR2>(f, p, c);
  argmin_step<DPP_HALF_MIRROR>(f, p, c); argmin_step<DPP_MIRROR>(f, p, c);
  argmin_rows<false>(f, p, c);
  argmin_rows<true>(f, p, c);
}

// A wave rebuilds the aggregate state of some of the columns whose turn it is at the start of step p
// (phase (p-1) mod R) from the R-1 rows of steps p-R+1 .. p-1, of which those up to the step at which the column's
// present token was born (its own position) count as zero: they hold weights of the slot's former occupant.
// Results stay in LDS:
//   stage[i*cpt + cc] = f(rows of steps p-1-i .. p-1) of column c0+cc   (i = 0..R-2), to be stored to
//                       sfx row (p-2-i) mod R by the whole workgroup later;
//   turn[cc]          = f(all R-1 rows): the old part of this step's score for that column.
// The columns are dealt out in groups of gw to the rebuilding waves (group k to wave k mod nrw).  Within
// a group lanes are (column cc, row chunk q): a lane owns the contiguous rows [q*Lc, (q+1)*Lc), which it
// loads as one batch and scans on their way into LDS; the chunks' totals are then carried over by lane shuffles.
// gw is chosen (a) so that a chunk fits one batch (R - 1 <= 64 batches always does) and (b), in the fused kernel, so
// small that each of the waves meant to rebuild (DecodeParams::rb_nrw) gets a group: the rebuild is a chain of
// dependent steps that the rest of the workgroup waits for at the end of the K pass.  Many waves with short chunks
// shorten the chain; but every wave that takes part runs the whole of this code, and the four waves of a SIMD
// share its issue slots, so a unit with little else to do is better off with two waves.
constexpr int RB = 8;  // rows per lane and batch in the fused kernel
// columns per group: 64 lanes / gw columns = row chunks, each at most `rows` rows
__host__ __device__ inline int turn_group_width(int R, int rows) {
  int gw = WAVE;
  while (gw > 1 && (R - 1 + WAVE / gw - 1) / (WAVE / gw) > rows) gw >>= 1;
  return gw;
}
// ... and narrow enough that cps columns make a group for each of NW waves, if there are that many columns
__host__ __device__ inline int turn_group_width(int R, int rows, int cps, int NW) {
  int gw = turn_group_width(R, rows);
  while (gw > 1 && (cps + gw - 1) / gw < NW) gw >>= 1;
  return gw;
}
template <int RBT> struct TurnRebuildT {
  int lane, p, R, rs, cpt, fusion, c0, ncol, r_top, gw, gstride, g0;
  const float *ringu;
  const int32_t *posu;
  // current column group
  int cg, CP, lg2, Q, cc, q, c, Lc, i0, i1;
  int age;  // rows 0 .. age-1 (steps p-1 .. p-age) are the present token's; 0 for a free slot
  bool colok;

  // k-th of nrw rebuilding waves
  __device__ inline void init(int lane_, int p_, int wm1, int n_used, int R_, int rs_, int cps, int cpt_,
                              int fusion_, const float *ringu_, const int32_t *posu_, int k, int nrw, int gw_) {
    lane = lane_; p = p_; R = R_; rs = rs_; cpt = cpt_; fusion = fusion_; ringu = ringu_; posu = posu_;
    r_top = wm1;  // (p-1) mod R: ring row of row i = 0
    c0 = wm1 * cps;
    ncol = n_used - c0;
    ncol = ncol < 0 ? 0 : (ncol > cps ? cps : ncol);
    gw = gw_;
    g0 = k * gw;
    gstride = nrw * gw;
  }
  __device__ inline void group(int cg_) {
    cg = cg_;
    const int nc = ncol - cg < gw ? ncol - cg : gw;
    lg2 = nc <= 1 ? 0 : 32 - __builtin_clz(nc - 1);
    CP = 1 << lg2;
    Q = WAVE >> lg2;
    cc = lane & (CP - 1); q = lane >> lg2;
    colok = cc < nc;
    c = c0 + cg + cc;
    Lc = (R - 1 + Q - 1) >> (6 - lg2);  // Q = 64 >> lg2
    i0 = min(q * Lc, R - 1); i1 = min(i0 + Lc, R - 1);
  }
  // rows i0+b .. i0+b+RBT-1 of this lane's chunk (a chunk is shorter than R rows: one wrap at most)
  __device__ inline void load(int b, float (&v)[RBT]) {
    // every load is in bounds (row taken mod R, column clamped); what lies outside the chunk is ignored
    // when the batch is consumed, so issuing it is straight-line code that waits for nothing.  Past the end of
    // a short chunk the chunk's last row is asked for again: the same cache line, no new request to memory.
    if (b == 0) {
      const int pc = posu[colok ? c : c0];
      age = pc < 0 ? 0 : p - 1 - pc;
    }
    const int ib = i0 + b;
    int r0 = r_top - ib;  // ib < R
    r0 += r0 < 0 ? R : 0;
    const unsigned coff = (unsigned)(colok ? c : c0);
    const int klast = Lc - 1 - b > 0 ? Lc - 1 - b : 0;
#pragma unroll
    for (int k = 0; k < RBT; ++k) {
      int r = r0 - (k < klast ? k : klast);
      r += r < 0 ? R : 0;
      r = r < 0 ? 0 : r;
      v[k] = ringu[(unsigned)(r * rs) + coff];
    }
  }
  __device__ inline void begin(float (&v)[RBT]) {
    if (ncol > g0) { group(g0); load(0, v); }
  }
  __device__ inline void finish(float (&v)[RBT], float *stage, float *turn) {
    if (ncol <= g0) return;
    while (true) {
      // the lane's chunk, scanned.  A chunk of one short batch waits in registers for its carry; a longer one
      // (RBT > 8, or R - 1 > 64 batches: several batches a chunk) goes to LDS as it is scanned
      const int nv = i1 - i0;
      const bool inreg = RBT <= 8 && Lc <= RBT;  // the same for all lanes
      float *st = stage + cg + cc + i0 * cpt;
      float acc = 0.f;
      if (inreg) {
#pragma unroll
        for (int k = 0; k < RBT; ++k)
          if (k < nv) {
            acc = fuse2(fusion, acc, i0 + k < age ? v[k] : 0.f);
            v[k] = acc;
          }
      } else {
        for (int b = 0;;) {
#pragma unroll
          for (int k = 0; k < RBT; ++k)
            if (b + k < nv) {
              acc = fuse2(fusion, acc, i0 + b + k < age ? v[k] : 0.f);
              st[(b + k) * cpt] = acc;
            }
          b += RBT;
          if (b >= Lc) break;
          load(b, v);
        }
      }
      // chunk totals -> carry into each chunk (exclusive scan over q), and the total over all rows
      float incl = acc;
      for (int s = CP; s < WAVE; s <<= 1) {
        const float o = __shfl_up(incl, s);
        if (lane >= s) incl = fuse2(fusion, incl, o);
      }
      float carry = __shfl_up(incl, CP);
      if (q == 0) carry = 0.f;
      if (q == Q - 1) turn[cg + cc] = incl;
      if (inreg) {
#pragma unroll
        for (int k = 0; k < RBT; ++k)
          if (k < nv) st[k * cpt] = fuse2(fusion, v[k], carry);
      } else if (q > 0) {
        // eight values are read back before any is written: one LDS round trip for the eight, not one each
        for (int kb = 0; kb < nv; kb += 8) {
          float t[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) t[j] = kb + j < nv ? st[(kb + j) * cpt] : 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (kb + j < nv) st[(kb + j) * cpt] = fuse2(fusion, t[j], carry);
        }
      }
      if (cg + gstride >= ncol) break;
      group(cg + gstride);
      load(0, v);
    }
  }
};
using TurnRebuild = TurnRebuildT<RB>;

// ---- the end of a step, shared by the fused kernel, the merging workgroup of the split kernel and the kernel of
// the layers that keep every token ---------------------------------------------------------------------------
// Everything the two functions below need of a workgroup's state.  LDS arrays (see the carve-up in the kernels):
//   sh  [16] 2: slot of the new token (-1: the first slot the selection below frees), 3: evicted position,
//            4: new number of slots in use, 5: tokens a selection under the coarse schedule has to evict (0: none),
//            6: new number of free slots below the mark
//   Fl, Pl [CsP] fused score (+inf: not a candidate) and position per slot, best2 [2][3][16] (T > 1 only)
template <typename T> struct StepTail {
  const DecodeParams &P;
  int u, tid, NT, NW, wave, lane, n_pad, n_used, p, w, Tev;
  int *sh;
  float *Fl;
  int *Pl;
  float *best2, *nwu;
  int32_t *posu;
  const T *knew, *vnew;
};

// Selection of the C best of up to C+T older tokens (Eq.7 with the coarse schedule of Appendix A.5): the sh[5]
// candidates with the smallest scores go (ties: the higher position goes).  Their slots become free: the new token
// takes the first, the others wait on the unit's stack of free slots for the tokens of the next steps.
template <typename T, int D>
__device__ __forceinline__ void coarse_select(const StepTail<T> &c) {
  const DecodeParams &P = c.P;
  const int u = c.u, tid = c.tid, NT = c.NT, NW = c.NW, wave = c.wave, lane = c.lane, n_used = c.n_used, Tev = c.Tev;
  int *sh = c.sh;
  float *Fl = c.Fl, *best2 = c.best2;
  int *Pl = c.Pl;
  int32_t *posu = c.posu;
  if (Tev > 1) {
    int32_t *evl = P.evl + (size_t)u * Tev, *holes = P.holes + (size_t)u * Tev;
    const int n_ev = sh[5];  // 1..T at a selection step
    if (tid >= n_ev && tid < Tev) evl[tid] = -1;
    // n_ev rounds, each taking out the candidate that goes first.  Every wave works the round's result out
    // for itself from the per-wave minima (two sets, used in turn: one barrier per round); slot j is read
    // and, once taken, struck out by thread j mod NT only.
    for (int it = 0; it < n_ev; ++it) {
      float f = INFINITY;
      int bp = -1, bc = -1;
      for (int j = tid; j < n_used; j += NT) {
        const float F = Fl[j];
        const int pj = Pl[j];
        if (cand_before(f, bp, F, pj)) { f = F; bp = pj; bc = j; }
      }
      wave_argmin(f, bp, bc);
      float *bF = best2 + (it & 1) * 48;
      int *bPp = (int *)bF + 16, *bCc = (int *)bF + 32;
      if (lane == 0) { bF[wave] = f; bPp[wave] = bp; bCc[wave] = bc; }
      lds_barrier();
      f = INFINITY; bp = -1; bc = -1;
      if (lane < NW) { f = bF[lane]; bp = bPp[lane]; bc = bCc[lane]; }
      wave_argmin(f, bp, bc);
      if (bc >= 0 && bc % NT == tid) { Fl[bc] = INFINITY; Pl[bc] = -1; }
      if (tid == 0 && bc >= 0) {
        evl[it] = bp;
        posu[bc] = -1;
        if (it == 0) { sh[3] = bp; sh[2] = bc; }
        else holes[it - 1] = bc;
      }
    }
    if (n_ev > 0) __syncthreads();  // the new token's slot is known to everybody
  }
}

// The new token takes its slot: K, V, position (the slot's aggregates are the former occupant's: record4 ignores
// the new part at the next step and the old part until the column's next turn); the unit's counters move on.
// PRE: the caller has already loaded this thread's piece of the new token's key (kpre: threads 0 .. D/EPL-1) and of its
// value (vpre; bf16 caches: the element of channel NT-1-tid in .x; fp32: the piece of threads 64 .. 64+D/EPL-1)
template <typename T, int D, bool CLK, bool PRE = false>
__device__ __forceinline__ void commit_step(const StepTail<T> &c, uint4 kpre = uint4{0u, 0u, 0u, 0u},
                                            uint4 vpre = uint4{0u, 0u, 0u, 0u}) {
  const DecodeParams &P = c.P;
  const int u = c.u, tid = c.tid, NT = c.NT, n_pad = c.n_pad, p = c.p, w = c.w;
  int *sh = c.sh;
  using L = Layout<T, D>;
  constexpr int EPL = Elem<T>::EPL;
  const int dest = sh[2];
  const bool okd = (unsigned)dest < (unsigned)n_pad;  // (always; nothing is ever written outside the unit's slots)
  T *Kw_ = (T *)P.K + (size_t)u * n_pad * D;
  T *Vw_ = (T *)P.V + (size_t)u * n_pad * D;
  constexpr int PCS = D / EPL;  // 16-byte pieces per row
  if (okd && tid < PCS)         // K: 16-byte pieces exist in both layouts (8 or 4 consecutive channels)
    *(uint4 *)(Kw_ + L::k_off(dest, tid * EPL)) = PRE ? kpre : ((const uint4 *)c.knew)[tid];
  if constexpr (L::tiled) {
    // V: one element per (slot, channel) in tile order; starts with the last threads, the K pieces took the first
    // (workgroups have at least D threads: one element a thread)
    for (int ch = NT - 1 - tid; okd && ch < D; ch += NT)
      ((uint16_t *)Vw_)[L::v_off(dest, ch)] = PRE ? (uint16_t)vpre.x : ((const uint16_t *)c.vnew)[ch];
  } else {
    if (okd && tid >= 64 && tid < 64 + PCS)
      *(uint4 *)(Vw_ + L::v_off(dest, (tid - 64) * EPL)) = PRE ? vpre : ((const uint4 *)c.vnew)[tid - 64];
  }
  if (tid == 0) {
    if (okd) c.posu[dest] = p;
    int32_t *m = P.meta + (size_t)u * META;
    m[0] = sh[4];
    m[1] = p + 1;
    m[2] = sh[3];
    const int R = P.R;
    m[3] = w + 1 == R ? 0 : w + 1;
    m[5] = sh[6];
    if (CLK && P.dbgT) P.dbgT[(size_t)u * 8 + 4] = wall_clock64();
  }
}

// CLK: the diagnostics build that stores phase time stamps to P.dbgT; the product build carries none of it.
// COARSE: the build for selection every T > 1 steps (Appendix A.5).  The every-step build carries none of that code:
// its scalars alone cost the kernel fifty registers that the compiler then keeps in vector lanes, and every wave
// pays for moving them there and back.
template <typename T, int D, int G, bool CLK, bool COARSE>
__device__ __forceinline__ void decode_fused_body(const DecodeParams &P) {
  using L = Layout<T, D>;
  constexpr int EPL = Elem<T>::EPL;
  // tile groups (K) and tiles (V) a wave keeps in flight.  Two of each was measured on 512-thread groups and
  // brought nothing (the passes are not bound by the depth of a wave's request queue); at 1024 threads two K
  // groups do not fit the 128 registers (the head_dim 128 builds spill), so it stays at one.
  constexpr int KBUF = 1, VBUF = 1;
  extern __shared__ __align__(16) float smem[];

  const int u = blockIdx.x + P.u0, tid = threadIdx.x, NT = blockDim.x, NW = NT / WAVE;
  // (the wave's index stays a per-lane value: as a scalar it turns the waves' branches into jumps, which was
  // measured slower by a microsecond per launch although it saves vector instructions)
  const int wave = tid / WAVE, lane = tid % WAVE;
  const int Cs = P.Cs, CsP = P.CsP, R = P.R, n_pad = P.n_pad, cps = P.cps, cpt = P.cpt;
  // Running-sum policy (fusion 2, the accumulated score of H2O): a column's score is the sum of everything recorded
  // for it since it entered the cache.  That is the sum fusion with a rebuild point that never comes: the new-part
  // aggregate is all there is, no column ever takes a turn, the old part is not read.
  const bool cum = P.fusion == 2;
  const int fusion = cum ? 0 : P.fusion;

  // ---- LDS carve-up
  // rows of the weight array are n_pad + 4 floats apart: the heads then start 4 banks apart and the 16-byte
  // accesses of the MFMA passes (4 heads x 4 slot groups) spread over all 32 banks
  const int lgs = n_pad + 4;
  const size_t lgsz = max((size_t)G * lgs, (size_t)NW * G * D);
  float *lg = smem;                       // [G][lgs] logits -> exp -> weights; later [NW][G][D] output partials
  float *stage = lg + lgsz;               // [R][cpt] rebuilt aggregates on their way to the sfx rows
  float *turn = stage + (size_t)R * cpt;  // [cpt] old-part aggregate of the columns rebuilt this step
  float *red = turn + cpt;                // [16][8]
  float *red2 = red + 16 * 8;             // [16][8]
  float *bestF = red2 + 16 * 8;           // [16]
  int *bestC = (int *)(bestF + 16);       // [16]
  int *bestP = bestC + 16;                // [16]
  int *sh = bestP + 16;                   // [16] 0: K tile counter; 2..6: see StepTail
  float *shf = (float *)(sh + 16);        // [16] 1..8: logits of the token against its own key
  // selection every T > 1 steps only:
  const int Tev = COARSE ? P.T : 1;
  float *Fl = shf + 16;                   // [CsP] fused score per slot (+inf: not a candidate)
  int *Pl = (int *)(Fl + (Tev > 1 ? CsP : 0));            // [CsP] its position
  float *best2 = (float *)(Pl + (Tev > 1 ? CsP : 0));     // [2][3][16] per-wave minima of the selection rounds
  [[maybe_unused]] unsigned *hbits = (unsigned *)(best2 + 2 * 3 * 16);  // [n_pad / 32] one bit per free slot

  const T *Kb = (const T *)P.K + (size_t)u * n_pad * D;
  const T *Vb = (const T *)P.V + (size_t)u * n_pad * D;
  const int uio = u - P.io_u0;                          // the unit's index within the step's tensors
  const T *qb = (const T *)P.q + (size_t)uio * G * D;   // query heads of the unit are rows uio*G .. uio*G+G-1
  // The cache is walked forwards on even steps and backwards on odd ones: what the previous step read
  // last is read first, so the part of K/V that still sits in the memory-side cache is hit instead of
  // being pushed out by the stream just ahead of its use.
  const bool zig = P.zig != 0;

  // the unit's state is asked for first and looked at only after the first K loads are on their way
  const int32_t *meta = P.meta + (size_t)u * META;
  const int n_used = meta[0], p = meta[1], w = meta[3];  // w = p mod R, kept by the kernel itself
  const int gen_step = p - meta[4] + 1;                  // the new token is this sequence's gen_step-th generated one
  const int n_holes = COARSE ? meta[5] : 0;              // free slots below n_used (left by a selection that took several)
  const bool sel_step = COARSE && P.T > 1 && gen_step % P.T == 0;  // coarse schedule: a step at which a selection may run

  // ---- bf16 path: the first K tiles of every wave and the query fragments go out before anything that
  // depends on the unit's state (the addresses do not)
  constexpr int KBc = L::KB, TU = 2;  // TU tiles in flight per wave
  [[maybe_unused]] uint4 ka[KBUF][TU][KBc];
  [[maybe_unused]] bf16x8_t qfr[KBc];
  [[maybe_unused]] const int kntile = n_pad / 16, kngrp = (kntile + TU - 1) / TU;
  auto load_kgroup = [&](uint4 (&dst)[TU][KBc], int grp) {
    const int gidx = zig ? kngrp - 1 - grp : grp;
    if (gidx < P.nt_k) {
#pragma unroll
      for (int t = 0; t < TU; ++t) {
        const int tile = gidx * TU + t;
        if (tile < kntile) {
#pragma unroll
          for (int kb = 0; kb < KBc; ++kb) dst[t][kb] = ldg16<true>(Kb + ((size_t)tile * KBc + kb) * 512 + lane * 8);
        }
      }
    } else {
#pragma unroll
      for (int t = 0; t < TU; ++t) {
        const int tile = gidx * TU + t;
        if (tile < kntile) {
#pragma unroll
          for (int kb = 0; kb < KBc; ++kb) dst[t][kb] = ldg16<false>(Kb + ((size_t)tile * KBc + kb) * 512 + lane * 8);
        }
      }
    }
  };
  if constexpr (L::tiled) {
    if (wave < kngrp) load_kgroup(ka[0], wave);
    const int head = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int kb = 0; kb < KBc; ++kb) {
      uint4 r = {0u, 0u, 0u, 0u};
      if (head < G) r = *(const uint4 *)(qb + (size_t)head * D + kb * 32 + kq * 8);
      qfr[kb] = __builtin_bit_cast(bf16x8_t, r);
    }
  }

  const int wm1 = w == 0 ? R - 1 : w - 1;  // (p-1) mod R
  const int turn0 = wm1 * cps;             // first column rebuilt this step
  int turn_n = n_used - turn0;             // how many of them exist
  turn_n = turn_n < 0 || cum ? 0 : (turn_n > cps ? cps : turn_n);

  float *ringu = P.ring + (size_t)u * R * n_pad;
  float *sfxu = P.sfx + (size_t)u * R * CsP;
  float *nwu = P.nw + (size_t)u * CsP;
  int32_t *posu = P.pos + (size_t)u * n_pad;
  const T *knew = (const T *)P.k_new + (size_t)uio * D;
  const T *vnew = (const T *)P.v_new + (size_t)uio * D;

  if (tid == 0) sh[0] = 2 * NW;  // every wave starts on the tile groups wave and wave + NW
  if (CLK && P.dbgT && tid == 0) P.dbgT[(size_t)u * 8 + 0] = wall_clock64();

  // ---- prefetch of the per-column state this thread will update after the softmax (4 columns a group)
  const int nq = n_pad / 4;
  float4 pn[MAXQ], ps[MAXQ];
  int4 pp[MAXQ];
#pragma unroll
  for (int i = 0; i < MAXQ; ++i) {
    const int j0 = 4 * (tid + i * NT);
    pn[i] = make_float4(0.f, 0.f, 0.f, 0.f); ps[i] = pn[i]; pp[i] = make_int4(-1, -1, -1, -1);
    if (j0 < n_used) {
      pn[i] = *(const float4 *)(nwu + j0);
      ps[i] = *(const float4 *)(sfxu + (size_t)w * CsP + j0);
      pp[i] = *(const int4 *)(posu + j0);
    }
  }
  // the slot a free-slot stack hands to the new token, if there is one (coarse schedule)
  int hole_top = -1;
  if constexpr (COARSE) {
    if (n_holes > 0) {  // (the same for the whole workgroup)
      hole_top = P.holes[(size_t)u * Tev + n_holes - 1];
      free_slot_bits(hbits, n_pad, P.holes + (size_t)u * Tev, n_holes, tid, NT);
      lds_barrier();
    }
  }
  // ---- what the end of the step needs of the new token: this thread's pieces of its key and value for the commit,
  // and the value element of the first output element it sums -- asked for now, not behind the V pass
  constexpr int PCSp = D / EPL;
  uint4 kpre = {0u, 0u, 0u, 0u}, vpre = kpre;
  float vn_pre = 0.f;
  {
    if (tid < PCSp) kpre = ((const uint4 *)knew)[tid];
    if constexpr (L::tiled) {
      if (NT - 1 - tid < D) vpre.x = ((const uint16_t *)vnew)[NT - 1 - tid];
    } else {
      if (tid >= 64 && tid < 64 + PCSp) vpre = ((const uint4 *)vnew)[tid - 64];
    }
    if (tid < G * D) {
      const int ch = tid % D;
      if constexpr (sizeof(T) == 4) vn_pre = ((const float *)vnew)[ch];
      else vn_pre = __uint_as_float(((uint32_t)((const uint16_t *)vnew)[ch]) << 16);
    }
  }
  // ---- the waves rebuild the columns whose turn it is, a group of columns each
  TurnRebuild tr;
  float rbv[RB];
  const int tgw = P.rb_gw, nrw = P.rb_nrw;
  if (wave >= NW - nrw) {
    tr.init(lane, p, wm1, cum ? 0 : n_used, R, n_pad, cps, cpt, fusion, ringu, posu, NW - 1 - wave, nrw, tgw);
    tr.begin(rbv);  // its rows are on their way while the wave works off its first tile group
  }

  // ---- self logit (every lane ends up with all G values)
  float selfl[G];
  if constexpr (!L::tiled) {
    constexpr int LPR = D / EPL;
    const int chunk = lane % LPR;
    uint4 r = ((const uint4 *)knew)[chunk];
    float kf[EPL];
    Elem<T>::unpack(r, kf);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint4 rq = ((const uint4 *)(qb + (size_t)g * D))[chunk];
      float qf[EPL];
      Elem<T>::unpack(rq, qf);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kf[e], d);
#pragma unroll
      for (int m = 1; m < LPR; m <<= 1) d += __shfl_xor(d, m);
      selfl[g] = d * P.scale_log2;
    }
  }
  // ---- K pass, first part: each wave works off the tile group it asked for at the very start and asks
  // for a second one, all before the workgroup's first barrier (late waves do not hold the others up)
  // running maximum of the logits: per head on the FMA path (a lane sees every head of its rows); on the MFMA
  // path a lane only ever sees the head lane & 15, so one value does
  float mx[L::tiled ? 1 : G];
#pragma unroll
  for (int g = 0; g < (L::tiled ? 1 : G); ++g) mx[g] = -INFINITY;
  [[maybe_unused]] const int head = lane & 15, kq = lane >> 4;
  auto process_kgroup = [&](const uint4 (&src)[TU][KBc], int grp) {
    const int gidx = zig ? kngrp - 1 - grp : grp;
#pragma unroll
    for (int t = 0; t < TU; ++t) {
      const int tile = gidx * TU + t;
      if (tile < kntile) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < KBc; ++kb)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, src[t][kb]), qfr[kb], acc, 0, 0, 0);
        // acc[i] = logit of slot tile*16 + 4*kq + i for head `head`
        if (head < G) {
          float l4[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int j = tile * 16 + 4 * kq + i;
            l4[i] = slot_valid(j, n_used) ? acc[i] * P.scale_log2 : -INFINITY;
          }
          if constexpr (COARSE) {
            if (n_holes > 0) {
              const unsigned fb = free_bits4(hbits, tile * 16 + 4 * kq);
#pragma unroll
              for (int i = 0; i < 4; ++i) l4[i] = (fb >> i) & 1u ? -INFINITY : l4[i];
            }
          }
          mx[0] = fmaxf(fmaxf(mx[0], fmaxf(l4[0], l4[1])), fmaxf(l4[2], l4[3]));
          *(float4 *)(lg + (size_t)head * lgs + tile * 16 + 4 * kq) = make_float4(l4[0], l4[1], l4[2], l4[3]);
        }
      }
    }
  };
  if constexpr (L::tiled) {
    if (wave < kngrp) process_kgroup(ka[0], wave);
    if (wave + NW < kngrp) load_kgroup(ka[0], wave + NW);
  }
  if (CLK && P.dbgT && tid == 0) P.dbgT[(size_t)u * 8 + 6] = wall_clock64();
  if (CLK && P.dbgT && tid == NT - 64) P.dbgT[(size_t)u * 8 + 5] = wall_clock64();
  lds_barrier();  // the tile counter is initialised
  if (CLK && P.dbgT && tid == 0) P.dbgT[(size_t)u * 8 + 7] = wall_clock64();

  // ---- rebuild of the columns whose turn it is, then the rest of the K pass
  if (wave >= NW - nrw) tr.finish(rbv, stage, turn);

  // ---- K pass, the rest
  if constexpr (L::tiled) {
    // MFMA: A = 16 slots x 32 channels of K, B = 32 channels x 16 heads of q (heads >= G are zero)
    constexpr int KB = L::KB;
    // wave 0: the token's own key as slot 0 of one more tile (other slots zero): its logits come out of
    // the same MFMA and are handed to everybody through LDS
    if (wave == 0) {
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        uint4 a = {0u, 0u, 0u, 0u};
        if (head == 0) a = *(const uint4 *)(knew + kb * 32 + kq * 8);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), qfr[kb], acc, 0, 0, 0);
      }
      if (lane < G) shf[1 + lane] = acc[0] * P.scale_log2;  // lanes 0..15 (kq = 0): slot 0, head = lane
    }
    const int ngrp = kngrp;
    // each buffer of the wave holds one group in flight; the first came with the wave's index, the
    // others and all later ones are drawn from the shared counter
    int gq[KBUF];
    gq[0] = wave + NW;  // in flight since before the barrier
#pragma unroll
    for (int b = 1; b < KBUF; ++b) {
      int x = 0;
      if (lane == 0) x = atomicAdd(&sh[0], 1);
      gq[b] = __builtin_amdgcn_readfirstlane(x);
      if (gq[b] < ngrp) load_kgroup(ka[b], gq[b]);
    }
    bool more = true;
    while (more) {
      more = false;
#pragma unroll
      for (int b = 0; b < KBUF; ++b) {
        if (gq[b] < ngrp) {
          int nxt = 0;
          if (lane == 0) nxt = atomicAdd(&sh[0], 1);
          process_kgroup(ka[b], gq[b]);
          gq[b] = __builtin_amdgcn_readfirstlane(nxt);
          if (gq[b] < ngrp) load_kgroup(ka[b], gq[b]);
          more = true;
        }
      }
    }
  } else {
    // plain FMAs on row-major K: LPR lanes share a row
    constexpr int LPR = D / EPL, RPL = WAVE / LPR, UNR = 4, RPT = RPL * UNR;
    const int chunk = lane % LPR, rowsub = lane / LPR;
    float qf[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint4 r = ((const uint4 *)(qb + (size_t)g * D))[chunk];
      Elem<T>::unpack(r, qf[g]);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qf[g][e] *= P.scale_log2;
    }
    const int ntile = (n_pad + RPT - 1) / RPT;
    int tile = wave;
    bool first = true;  // tiles wave and wave + NW are this wave's by right, the rest come from the counter
    while (tile < ntile) {
      int nxt = wave + NW;
      if (!first && lane == 0) nxt = atomicAdd(&sh[0], 1);
      uint4 r[UNR];
      bool ok[UNR];
#pragma unroll
      for (int i = 0; i < UNR; ++i) {
        const int j = tile * RPT + i * RPL + rowsub;
        ok[i] = slot_valid(j, n_used);
        if constexpr (COARSE) {
          if (n_holes > 0 && ok[i]) ok[i] = !((hbits[j >> 5] >> (j & 31)) & 1u);
        }
        if (ok[i]) r[i] = ((const uint4 *)(Kb + (size_t)j * D))[chunk];
      }
#pragma unroll
      for (int i = 0; i < UNR; ++i) {
        const int j = tile * RPT + i * RPL + rowsub;
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
          const float l = ok[i] ? d : -INFINITY;
          mx[g] = fmaxf(mx[g], l);
          if (chunk == 0 && j < n_pad) lg[(size_t)g * lgs + j] = l;
        }
      }
      tile = first ? nxt : __builtin_amdgcn_readfirstlane(nxt);
      first = false;
    }
  }
  // a lane saw only some heads / rows: combine across the wave
  if constexpr (L::tiled) {
    // lanes l, l + 16, l + 32, l + 48 hold the same head
    const float v = max_over_rows(mx[0]);
    if (lane < G) red[wave * 8 + lane] = v;
  } else {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float v = wave_max_dpp(mx[g]);
      if (lane == 0) red[wave * 8 + g] = v;
    }
  }

  // ---- first V tile of this wave goes in flight now: it does not depend on the softmax
  [[maybe_unused]] uint4 vbuf[VBUF][L::CB];
  auto load_vtile = [&](uint4 (&dst)[L::CB], int ti) {
    const int tile = zig ? n_pad / 32 - 1 - ti : ti;
    if (tile < P.nt_v) {
#pragma unroll
      for (int cb = 0; cb < L::CB; ++cb) dst[cb] = ldg16<true>(Vb + ((size_t)tile * L::CB + cb) * 512 + lane * 8);
    } else {
#pragma unroll
      for (int cb = 0; cb < L::CB; ++cb) dst[cb] = ldg16<false>(Vb + ((size_t)tile * L::CB + cb) * 512 + lane * 8);
    }
  };
  if constexpr (L::tiled) {
#pragma unroll
    for (int b = 0; b < VBUF; ++b)
      if (wave + b * NW < n_pad / 32) load_vtile(vbuf[b], wave + b * NW);
  }
  lds_barrier();
  if (CLK && P.dbgT && tid == 0) P.dbgT[(size_t)u * 8 + 1] = wall_clock64();

  if constexpr (L::tiled) {
#pragma unroll
    for (int g = 0; g < G; ++g) selfl[g] = shf[1 + g];
  }
  // ---- the rebuilt aggregates of this step's turn columns (complete in LDS since the barrier above) go out to
  // their sfx rows: by the waves that have no slots to take in the softmax and record phases below, beside those
  // phases, if there are such waves; else by everybody after them.  Threads t0, t0 + nthr, .. of the caller's.
  auto store_turn_columns = [&](int t0, int nthr) {
    const int rz = wm1, r0 = wm1 == 0 ? R - 1 : wm1 - 1;  // (p-1) mod R, (p-2) mod R
    // row R-1 of the staging area stands for the zeroed row (p-1) mod R
    if (((cpt | turn_n | turn0) & 3) == 0) {
      // whole groups of four columns: 16-byte stores (CsP is a multiple of 32, the staging area starts 16-byte aligned)
      const int q4 = cpt >> 2, total = R * q4, csh = P.cpt_shift;
      for (int idx = t0; idx < total; idx += nthr) {
        const int i = csh >= 2 ? idx >> (csh - 2) : idx / q4, c4 = (idx - i * q4) * 4;
        if (c4 < turn_n) {
          int r = r0 - i;
          if (r < 0) r += R;
          const bool last = i == R - 1;
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (!last) v = *(const float4 *)(stage + (size_t)i * cpt + c4);
          *(float4 *)(sfxu + (size_t)(last ? rz : r) * CsP + turn0 + c4) = v;
        }
      }
    } else {
      const int total = R * cpt, csh = P.cpt_shift;
      for (int idx = t0; idx < total; idx += nthr) {
        const int i = csh >= 0 ? idx >> csh : idx / cpt, cc = idx - i * cpt;
        if (cc < turn_n) {
          int r = r0 - i;
          if (r < 0) r += R;
          const bool last = i == R - 1;
          sfxu[(size_t)(last ? rz : r) * CsP + turn0 + cc] = last ? 0.f : stage[idx];
        }
      }
    }
  };
  const int busy_waves = (nq + WAVE - 1) / WAVE;  // waves that hold slots in the phases below (4 slots a thread)
  const bool helpers = turn_n > 0 && busy_waves < NW;
  if (helpers && wave >= busy_waves) store_turn_columns(tid - busy_waves * WAVE, (NW - busy_waves) * WAVE);
  // ---- softmax: exact max, sum, weights (4 slots per thread and head at a time)
  float M[G], inv[G], pself[G];
  {
    // red holds [wave][8]: lane l looks at head l%8 of waves l/8 and l/8+8, then lanes of equal head combine
    float v = -INFINITY;
    if ((lane >> 3) < NW) v = red[lane];
    if ((lane >> 3) + 8 < NW) v = fmaxf(v, red[lane + 64]);
    v = max_over_rows(fmaxf(v, dpp_mov<DPP_ROW_ROR8>(v)));  // over the lanes of equal head: l, l ^ 8, l ^ 16, l ^ 32
#pragma unroll
    for (int g = 0; g < G; ++g) M[g] = fmaxf(selfl[g], lane_bcast(v, g));
  }
  {
    float zs[G];
#pragma unroll
    for (int g = 0; g < G; ++g) zs[g] = 0.f;
    for (int jq = tid; jq < nq; jq += NT) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float4 *pl = (float4 *)(lg + (size_t)g * lgs + 4 * jq);
        float4 l = *pl;
        l.x = exp2_native(l.x - M[g]); l.y = exp2_native(l.y - M[g]); l.z = exp2_native(l.z - M[g]); l.w = exp2_native(l.w - M[g]);
        *pl = l;
        zs[g] += (l.x + l.y) + (l.z + l.w);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float s = wave_sum_dpp(zs[g]);
      if (lane == 0) red2[wave * 8 + g] = s;
    }
  }
  lds_barrier();
  {
    float v = 0.f;
    if ((lane >> 3) < NW) v = red2[lane];
    if ((lane >> 3) + 8 < NW) v += red2[lane + 64];
    v = sum_over_rows(v + dpp_mov<DPP_ROW_ROR8>(v));
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float es = exp2_native(selfl[g] - M[g]);
      const float z = es + lane_bcast(v, g);
      inv[g] = 1.0f / z;
      pself[g] = es * inv[g];
    }
  }

  // ---- record the row, update per-column aggregates, fused scores, local argmin
  float bF = INFINITY;
  int bP = -1, bC = -1;
  // Every slot in use is a column.  Its old part (the sfx row) counts only if the column has had a turn since its
  // token was born -- until then the row holds the former occupant's, and the new part alone is the whole window
  // aggregate (none of the token's rows has expired yet: every column's turn comes once in any R steps).  A token is
  // a candidate for eviction once it is older than the window that includes the new token: position <= p - R.
  // (phi, rem) = (j0 / cps, j0 % cps): the phase of column j0 and where in its group of cps columns it sits.
  auto record4 = [&](int j0, float4 nw_old, float4 sfx_old, int4 pj4, int phi, int rem) {
    float S[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float4 *pl = (float4 *)(lg + (size_t)g * lgs + j0);
      float4 l = *pl;
      l.x *= inv[g]; l.y *= inv[g]; l.z *= inv[g]; l.w *= inv[g];
      *pl = l;
      S[0] += l.x; S[1] += l.y; S[2] += l.z; S[3] += l.w;
    }
    stg16_stream(ringu + (size_t)w * n_pad + j0, make_float4(S[0], S[1], S[2], S[3]));
    if (j0 < n_used) {
      float nwo[4] = {nw_old.x, nw_old.y, nw_old.z, nw_old.w};
      const float sfo[4] = {sfx_old.x, sfx_old.y, sfx_old.z, sfx_old.w};
      const int pj[4] = {pj4.x, pj4.y, pj4.z, pj4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = j0 + i;
        // steps since the column's last turn before this step, and rows recorded since its token was born
        int d = wm1 - phi;
        d += d < 0 ? R : 0;
        const int age = p - 1 - pj[i];
        float so = (cum || pj[i] < 0 || d > age) ? 0.f : sfo[i];
        if (j >= turn0 && j < turn0 + turn_n) { nwo[i] = 0.f; so = turn[j - turn0]; }
        if (pj[i] == p - 1) nwo[i] = 0.f;  // born at the last step: what is stored is the former occupant's
        nwo[i] = fuse2(fusion, nwo[i], S[i]);
        const bool cand = j < n_used && pj[i] >= 0 && pj[i] <= p - R;
        // (a score that is not a number -- the caller's q or k were not -- counts as the largest: a candidate is
        // then still found, by position, and the cache keeps its structure)
        const float Fv = fuse2(fusion, so, nwo[i]);
        const float F = cand && Fv == Fv ? Fv : INFINITY;
        if (cand && P.dbgF) P.dbgF[(size_t)u * n_pad + j] = F;
        if (sel_step && j < n_used) { Fl[j] = F; Pl[j] = cand ? pj[i] : -1; }  // (position -1: never taken)
        if (cand && cand_before(bF, bP, F, pj[i])) { bF = F; bP = pj[i]; bC = j; }
        ++rem;
        if (rem == cps) { rem = 0; ++phi; }
      }
      stg16_stream(nwu + j0, make_float4(nwo[0], nwo[1], nwo[2], nwo[3]));
    }
  };
  // phase of this thread's first column, and how it moves from one of its groups of 4 columns to the next
  int cphi = (4 * tid) / cps, crem = (4 * tid) % cps;
  const int qstep = (4 * NT) / cps, rstep = (4 * NT) % cps;
  auto next_phase = [&]() {
    cphi += qstep;
    crem += rstep;
    if (crem >= cps) { crem -= cps; ++cphi; }
  };
#pragma unroll
  for (int i = 0; i < MAXQ; ++i) {
    const int jq = tid + i * NT;
    if (jq < nq) record4(4 * jq, pn[i], ps[i], pp[i], cphi, crem);
    next_phase();
  }
  for (int jq = tid + MAXQ * NT; jq < nq; jq += NT) {
    const int j0 = 4 * jq;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
    int4 pj = make_int4(-1, -1, -1, -1);
    if (j0 < n_used) {
      a = *(const float4 *)(nwu + j0);
      b = *(const float4 *)(sfxu + (size_t)w * CsP + j0);
      pj = *(const int4 *)(posu + j0);
    }
    record4(j0, a, b, pj, cphi, crem);
    next_phase();
  }
  wave_argmin(bF, bP, bC);
  if (lane == 0) { bestF[wave] = bF; bestP[wave] = bP; bestC[wave] = bC; }
  if (turn_n > 0 && !helpers) store_turn_columns(tid, NT);
  lds_barrier();
  if (CLK && P.dbgT && tid == 0) P.dbgT[(size_t)u * 8 + 2] = wall_clock64();

  // ---- decision (wave 0, before its share of the V pass): needs only the scores
  if (wave == 0) {
    float f = INFINITY;
    int bp = -1, bc = -1;
    if (lane < NW) { f = bestF[lane]; bp = bestP[lane]; bc = bestC[lane]; }
    wave_argmin(f, bp, bc);
    if (lane == 0) {
      // tokens older than the window once the new token is in
      const int older = n_used - n_holes + 1 - (p + 1 < R ? p + 1 : R);
      int dest = n_used, evicted = -1, nu = n_used + 1, multi = 0, nh = n_holes;
      if (Tev > 1) {
        // a selection is due at every T-th generation step, if more than C older tokens would be held; between
        // selections the new token takes a slot an earlier selection has freed, while there is one
        if (sel_step && older > P.C) {
          multi = older - P.C;  // top-C of up to C+T: done by the whole workgroup after the V pass
          dest = -1; nu = n_used; nh = multi - 1;
        } else if (n_holes > 0) {
          dest = hole_top; nu = n_used; nh = n_holes - 1;
        }
      } else if (older > Cs && bc >= 0) {
        dest = bc; evicted = bp; nu = n_used;
      }
      if (dest >= n_pad) { dest = -1; nu = n_used; }  // (a full cache with nothing to evict cannot happen: no write then)
      sh[2] = dest;
      sh[3] = evicted;
      sh[4] = nu;
      sh[5] = multi;
      sh[6] = nh;
    }
  }

  // ---- V pass
  if constexpr (L::tiled) {
    // MFMA: A = 16 heads x 32 slots of weights (bf16 hi + lo parts, so the product keeps ~16 bits of p),
    //       B = 32 slots x 16 channels of V
    constexpr int CB = L::CB;
    const int head = lane & 15, kq = lane >> 4;
    f32x4_t acc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) acc[cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int ntile = n_pad / 32;
    // tiles are dealt out statically here: the order in which a wave adds up its tiles, and with it the
    // rounding of the output, is then the same in every run
    auto process_vtile = [&](const uint4 (&src)[CB], int ti) {
      const int tile = zig ? ntile - 1 - ti : ti;
      bf16x8_t ahi, alo;
      {
        float pv[8];
        if (head < G) {
          const float4 x = *(const float4 *)(lg + (size_t)head * lgs + tile * 32 + kq * 8);
          const float4 y = *(const float4 *)(lg + (size_t)head * lgs + tile * 32 + kq * 8 + 4);
          pv[0] = x.x; pv[1] = x.y; pv[2] = x.z; pv[3] = x.w; pv[4] = y.x; pv[5] = y.y; pv[6] = y.z; pv[7] = y.w;
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) pv[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const __bf16 h = (__bf16)pv[i];
          ahi[i] = h;
          alo[i] = (__bf16)(pv[i] - (float)h);
        }
      }
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, src[cb]);
        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi, bv, acc[cb], 0, 0, 0);
        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo, bv, acc[cb], 0, 0, 0);
      }
    };
    for (int ti0 = wave; ti0 < ntile; ti0 += VBUF * NW) {
#pragma unroll
      for (int b = 0; b < VBUF; ++b) {
        const int ti = ti0 + b * NW;
        if (ti < ntile) {
          process_vtile(vbuf[b], ti);
          // the tile this buffer holds next goes into the same registers
          if (ti + VBUF * NW < ntile) load_vtile(vbuf[b], ti + VBUF * NW);
        }
      }
    }
    lds_barrier();  // every wave is done reading the weights: lg may be reused
    // acc[cb][i] = O[head 4*kq + i][channel cb*16 + (lane & 15)]
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int g = 4 * kq + i;
        if (g < G) lg[(size_t)(wave * G + g) * D + cb * 16 + head] = acc[cb][i];
      }
  } else {
    constexpr int LPR = D / EPL, RPL = WAVE / LPR, UNR = 4, RPT = RPL * UNR;
    const int chunk = lane % LPR, rowsub = lane / LPR;
    float acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    const int ntile = (n_pad + RPT - 1) / RPT;
    for (int tile = wave; tile < ntile; tile += NW) {
      uint4 r[UNR];
      bool ok[UNR];
#pragma unroll
      for (int i = 0; i < UNR; ++i) {
        const int j = tile * RPT + i * RPL + rowsub;
        ok[i] = slot_valid(j, n_used);
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
            const float pg = lg[(size_t)g * lgs + j];
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
    lds_barrier();  // every wave is done reading the weights: lg may be reused
    if (rowsub == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) lg[(size_t)(wave * G + g) * D + chunk * EPL + e] = acc[g][e];
    }
  }
  if (CLK && P.dbgT && tid == 0) P.dbgT[(size_t)u * 8 + 3] = wall_clock64();
  // the output partials are in LDS; every wave is done with K and V (the commit below writes into them).  Nothing
  // the commit stores is an address the record phase has stored to: no wait for those stores
  lds_barrier();

  // ---- output
  for (int idx = tid; idx < G * D; idx += NT) {
    const int g = idx / D, ch = idx % D;
    float o = 0.f;
    for (int x = 0; x < NW; ++x) o += lg[(size_t)(x * G + g) * D + ch];
    float vn = vn_pre;  // (the first element of every thread; the others -- small workgroups -- are fetched here)
    if (idx != tid) {
      if constexpr (sizeof(T) == 4) vn = ((const float *)vnew)[ch];
      else vn = __uint_as_float(((uint32_t)((const uint16_t *)vnew)[ch]) << 16);
    }
    float psg = 0.f;
#pragma unroll
    for (int gg = 0; gg < G; ++gg) psg = gg == g ? pself[gg] : psg;
    o = fmaf(psg, vn, o);
    P.out[((size_t)uio * G + g) * D + ch] = o;
  }

  // ---- selection among more than C+1 candidates (coarse schedule), commit: shared with the split kernel
  StepTail<T> tc{P, u, tid, NT, NW, wave, lane, n_pad, n_used, p, w, Tev, sh, Fl, Pl, best2, nwu, posu, knew, vnew};
  if constexpr (COARSE) coarse_select<T, D>(tc);
  commit_step<T, D, CLK, true>(tc, kpre, vpre);
}

// Register budgets.  The compiler version this is built with places spill stores at the top of the block
// where the lanes of a skipped branch join again, BEFORE it restores their execution mask: a value spilled
// there is lost for waves that skipped the branch (seen: the fp32 d=64 G=8 build moved only 16 of a key's 256
// bytes when it wrote a token into its slot).  So no build may spill vector registers: the bf16 builds fit 128 registers (1024-thread
// groups); the fp32 builds, which keep G x 4 products per lane in flight, get 256 (groups of at most 512).
template <typename T, int D, int G, bool CLK, bool COARSE>
__global__ __launch_bounds__(1024) void decode_fused_kernel(DecodeParams P) {
  decode_fused_body<T, D, G, CLK, COARSE>(P);
}
template <typename T, int D, int G, bool COARSE>
__global__ __launch_bounds__(512) void decode_fused_kernel_512(DecodeParams P) {
  decode_fused_body<T, D, G, false, COARSE>(P);
}

}  // namespace mkv

// C-ABI of libmorphkv (see include/morphkv.h): argument checks, buffer carve-up, kernel launches.
// Host code only enqueues work on the caller's stream; all device memory is the caller's.
#include "../../include/morphkv.h"
#include "../../include/morphkv_diag.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <vector>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "host.h"
#include "decode.h"
#include "decode_split.h"
#include "decode_keep.h"
#include "prefill.h"
#include "prompt_attn.h"
#include "misc_kernels.h"

using namespace mkv;

namespace {
thread_local char g_err[512] = "";
}  // namespace

int mkv::fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

namespace {

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- library-owned workspace for callers that cannot allocate (morphkv_prefill_select_noalloc): one array per
// GPU, part of the loaded code object, held until the process ends.  In host code the array's name is only a
// stand-in: its device address is looked up once per device and kept.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)MORPHKV_NOALLOC_SCRATCH_BYTES;
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
char *g_scratch_ptr[MAX_DEVICES] = {};
}  // namespace
static __device__ __align__(256) unsigned char scratch[(size_t)MORPHKV_NOALLOC_SCRATCH_BYTES];
namespace {

// device address of the current device's copy of `scratch`
int static_scratch(char **out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(MORPHKV_EHIP, "device index %d outside 0..%d", dev, MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(MORPHKV_EHIP, "hipGetSymbolAddress returned a null address for the library's workspace");
    g_scratch_ptr[dev] = (char *)p;
  }
  *out = g_scratch_ptr[dev];
  return MORPHKV_OK;
}

// up to 256 host integers handed to the device as kernel arguments: no copy engine, no staging buffer, no host
// synchronisation, and the launch can be captured in a HIP graph
struct IntArgs { int32_t v[256]; };
__global__ void store_ints_kernel(int32_t *dst, IntArgs a, int n) {
  if ((int)threadIdx.x < n) dst[threadIdx.x] = a.v[threadIdx.x];
}
int upload_ints(int32_t *dst, const int32_t *src, int n, hipStream_t st) {
  for (int i0 = 0; i0 < n; i0 += 256) {
    IntArgs a;
    const int m = n - i0 < 256 ? n - i0 : 256;
    for (int i = 0; i < 256; ++i) a.v[i] = i < m ? src[i0 + i] : 0;
    hipLaunchKernelGGL(store_ints_kernel, dim3(1), dim3(256), 0, st, dst + i0, a, m);
    HIP_TRY(hipGetLastError());
  }
  return MORPHKV_OK;
}

struct BufLayout {
  int U, G, Cs, CsP, n, n_pad, cps, cpt, esz;
  // cache
  size_t offK, offV, offPos, offMeta, offEvl, offHoles, cache_bytes;
  // scores_ring
  size_t offRing, offSfx, offNw, offSpW, offSpPart, offSpCnt, ring_bytes;
  int sp_smax;     // most workgroups a unit is ever split over (1: the split kernel is never used, no workspace)
  int sp_force;    // MORPHKV_SPLIT_BPS: blocks per workgroup forced (tuning / tests), 0 = never split, -1 = choose
  bool keep_all;   // layers that keep every token: no recorded rows, no aggregates; decode_keep_kernel (or, on request,
                   // the split kernel with one or more workgroups a unit)
  // scratch
  size_t offSrow, offStat, offF, offSel, offPlen, offLseW, scratch_bytes;
};

int validate(const morphkv_config *c) {
  if (!c) return fail(MORPHKV_EINVAL, "config is null");
  if (c->n_layers < 1 || c->batch < 1) return fail(MORPHKV_EINVAL, "n_layers and batch must be >= 1");
  if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads)
    return fail(MORPHKV_EINVAL, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", c->n_q_heads,
                c->n_kv_heads);
  const int G = c->n_q_heads / c->n_kv_heads;
  if (G > 8) return fail(MORPHKV_EINVAL, "group size %d not supported (1..8)", G);
  if (c->head_dim != 64 && c->head_dim != 128) return fail(MORPHKV_EINVAL, "head_dim must be 64 or 128");
  if (c->C < 1) return fail(MORPHKV_EINVAL, "C must be >= 1");
  if (c->R < 1 || c->R > 1024) return fail(MORPHKV_EINVAL, "R must be in 1..1024");
  if (c->fusion != MORPHKV_FUSION_SUM && c->fusion != MORPHKV_FUSION_MAX && c->fusion != MORPHKV_FUSION_CUMSUM)
    return fail(MORPHKV_EINVAL, "fusion must be 0 (sum), 1 (max) or 2 (running sum)");
  if (c->dtype != MORPHKV_DTYPE_F32 && c->dtype != MORPHKV_DTYPE_BF16)
    return fail(MORPHKV_EINVAL, "dtype must be 0 (f32) or 1 (bf16)");
  if (c->evict_every < 0 || c->evict_every > 64) return fail(MORPHKV_EINVAL, "evict_every must be in 0..64");
  if (c->evict_every == 0 && (c->max_new_tokens < 1 || c->max_new_tokens > (1 << 20)))
    return fail(MORPHKV_EINVAL, "evict_every == 0 (selection at the prompt only) needs max_new_tokens >= 1");
  if (c->max_prompt_len < 1) return fail(MORPHKV_EINVAL, "max_prompt_len must be >= 1");
  if (!(c->softmax_scale >= 0.0f) || !std::isfinite(c->softmax_scale))
    return fail(MORPHKV_EINVAL, "softmax_scale must be finite and >= 0");
  if (c->n_keep_all_layers < 0 || c->n_keep_all_layers > c->n_layers)
    return fail(MORPHKV_EINVAL, "n_keep_all_layers must be in 0..n_layers");
  if (c->n_keep_all_layers > 0 && c->dtype != MORPHKV_DTYPE_BF16)
    return fail(MORPHKV_EINVAL, "layers that keep every token (n_keep_all_layers) are built for bf16 caches only");
  if (c->n_keep_all_layers > 0 && (c->max_new_tokens < 1 || c->max_new_tokens > (1 << 20)))
    return fail(MORPHKV_EINVAL, "n_keep_all_layers > 0 needs max_new_tokens >= 1 (those layers hold max_prompt_len + max_new_tokens tokens)");
  const long long U = (long long)c->n_layers * c->batch * c->n_kv_heads;
  if (U > 65535) return fail(MORPHKV_EINVAL, "too many units (layers*batch*kv_heads must be <= 65535)");
  if ((long long)c->C + c->R + (c->evict_every == 0 ? c->max_new_tokens : 0) > (1 << 20)) return fail(MORPHKV_EINVAL, "C + R too large");
  if (c->n_keep_all_layers > 0 && (long long)c->max_prompt_len + c->max_new_tokens + c->R > (1 << 20))
    return fail(MORPHKV_EINVAL, "n_keep_all_layers > 0: max_prompt_len + max_new_tokens + R = %lld slots per layer that keeps every token, "
                "at most 1048576", (long long)c->max_prompt_len + c->max_new_tokens + c->R);
  return MORPHKV_OK;
}


// How a launch of n_units units is split over workgroups (decode_split.h): S workgroups per unit, each on bps
// blocks of 32 slots.  S = 1: the fused kernel.  The device is taken to have N_CU_REF compute units (MI355X), so
// that the plan -- and the workspace sized from it -- is the same wherever it is made.
constexpr int N_CU_REF = 256;
struct SplitPlan { int S, bps; };
SplitPlan plan_split(int n_pad, int G, int D, int R, int cps, int CsP, int T, bool bf16, int n_units, int force_bps,
                     bool fused_fits) {
  SplitPlan one{1, n_pad / 32};
  if (!bf16) return one;
  const int nblk = n_pad / 32;
  int bps;
  // one workgroup per unit wherever it can hold the unit: the split kernel's chain (partial results out, count in,
  // merge) was measured slower than the fused kernel even for launches of 8 and 64 units (1088 and 544 slots)
  if (force_bps <= 0 && fused_fits) return one;
  if (force_bps > 0) {
    bps = force_bps;
  } else {
    // as many workgroups per unit as fill the device once
    const int S0 = n_units >= N_CU_REF ? 1 : N_CU_REF / n_units;
    bps = (nblk + S0 - 1) / S0;
  }
  // phase A keeps the share's G x (32 bps) logits in LDS: 64 KB at most; and at most SPLIT_MAX workgroups a unit
  const int bps_lds = ((64 * 1024 / 4) / G - 4) / 32, bps_min = (nblk + SPLIT_MAX - 1) / SPLIT_MAX;
  if (bps > bps_lds) bps = bps_lds;
  if (bps < bps_min) bps = bps_min;
  if (bps < 1) bps = 1;
  SplitPlan pl{(nblk + bps - 1) / bps, bps};
  if (force_bps <= 0 && n_units < N_CU_REF && pl.S > 1) {
    // The shares' limit may have raised the number of workgroups to one that does not go evenly over the compute
    // units (64 units of 16 k slots: 5 workgroups each = 320 on 256 units, and the launch takes as long as 512
    // would): then the next number that does, if it is in reach
    int g = n_units, r = N_CU_REF;
    while (r) { const int t = g % r; g = r; r = t; }
    const int m = N_CU_REF / g, S2 = (pl.S + m - 1) / m * m;
    if (S2 != pl.S && S2 <= SPLIT_MAX && S2 <= 2 * pl.S) {
      bps = (nblk + S2 - 1) / S2;
      pl = SplitPlan{(nblk + bps - 1) / bps, bps};
    }
  }
  if (pl.S < 2 && fused_fits) return one;
  if (bps > bps_lds || decode_split_lds_bytes(bps, G, D, R, cps, CsP, T) > 160 * 1024) return SplitPlan{0, 0};  // does not fit
  return pl;
}

// Workgroups per unit of decode_keep_kernel (layers that keep every token) in a launch of n_units units: one (or two)
// from 160 units on; below that as many as give every compute unit a share, a number that goes evenly over the compute units
// where one is in reach, and shares of 16 blocks of 32 slots at least when the layer is full.
int keep_shares(int n_units, int n_pad) {
  if (const char *e = std::getenv("MORPHKV_KEEP_SHARES")) {  // (tests, tuning)
    const int v = std::atoi(e);
    if (v >= 1 && v <= SPLIT_MAX) return v;
  }
  // (about one workgroup per compute unit and long layers: two halves go over the compute units more evenly than
  // one whole, 256 units x 5.9 k tokens 138 -> 129 us; with layers of 2.9 k tokens it costs 7 %)
  if (n_units >= 160) return n_units < 2 * N_CU_REF && n_pad >= 8192 ? 2 : 1;
  int S = (N_CU_REF + n_units - 1) / n_units;
  int g = n_units, r = N_CU_REF;
  while (r) { const int t = g % r; g = r; r = t; }
  const int m = N_CU_REF / g, S2 = (S + m - 1) / m * m;
  if (S2 <= 2 * S) S = S2;
  const int cap = n_pad / 32 / 16;
  if (S > cap) S = cap;
  if (S > SPLIT_MAX) S = SPLIT_MAX;
  return S < 1 ? 1 : S;
}

BufLayout make_layout(const morphkv_config *c, bool keep_all = false) {
  BufLayout L{};
  L.keep_all = keep_all;
  L.U = c->n_layers * c->batch * c->n_kv_heads;
  L.G = c->n_q_heads / c->n_kv_heads;
  L.Cs = c->C + (c->evict_every >= 1 ? c->evict_every - 1 : c->max_new_tokens);
  L.n = L.Cs + c->R;
  L.n_pad = (L.n + 31) / 32 * 32;  // K/V slot arrays are padded to whole tiles
  L.CsP = L.n_pad;                 // row stride of the per-column state: every slot is a column
  // Columns rebuilt per step: at least ceil(Cs/R), so that every column's turn comes once in R steps.  The
  // rebuilt aggregates go out as one run of cps floats per sfx row: runs that are whole 128-byte lines (else
  // 64, 32 .. bytes) keep partial-line writes away from HBM, which cost several us per step on c3-sized
  // caches when the run was 17 floats.  Rounded up as far as the LDS staging area (R x cps floats) allows.
  const int cps0 = keep_all ? 1 : (L.n + c->R - 1) / c->R;  // (a layer that keeps every token rebuilds nothing)
  L.cps = cps0;
  for (int a = keep_all ? 1 : 32; a > 1; a >>= 1) {
    const int cand = (cps0 + a - 1) / a * a;
    const size_t stage = (size_t)c->R * turn_cols_padded(cand) * 4;
    if (stage <= 32 * 1024 &&
        decode_lds_bytes(L.n_pad, L.G, c->head_dim, 1024, c->R, cand, L.n_pad, c->evict_every) <= 160 * 1024) {
      L.cps = cand;
      break;
    }
  }
  L.cpt = turn_cols_padded(L.cps);
  L.esz = c->dtype == MORPHKV_DTYPE_F32 ? 4 : 2;
  const size_t U = (size_t)L.U, np = (size_t)L.n_pad, d = (size_t)c->head_dim, R = (size_t)c->R,
               CsP = (size_t)L.CsP;
  size_t o = 0;
  L.offK = o; o = align_up(o + U * np * d * L.esz);
  L.offV = o; o = align_up(o + U * np * d * L.esz);
  L.offPos = o; o = align_up(o + U * np * 4);
  L.offMeta = o; o = align_up(o + U * META * 4);
  L.offEvl = o; o = align_up(o + U * (size_t)(c->evict_every > 0 ? c->evict_every : 1) * 4);
  L.offHoles = o; o = align_up(o + U * (size_t)(c->evict_every > 0 ? c->evict_every : 1) * 4);
  L.cache_bytes = o;
  o = 0;
  L.offRing = o; o = align_up(o + (keep_all ? 0 : U * R * np * 4));
  L.offSfx = o; o = align_up(o + (keep_all ? 0 : U * R * CsP * 4));
  L.offNw = o; o = align_up(o + (keep_all ? 0 : U * CsP * 4));
  // workspace of the split decode kernel, sized for the launches this configuration can make: all units at once,
  // or one layer's
  L.sp_force = -1;
  if (const char *e = std::getenv("MORPHKV_SPLIT_BPS")) L.sp_force = std::atoi(e);
  L.sp_smax = 1;
  if (L.esz == 2) {
    const bool fits = !keep_all &&
                      decode_lds_bytes(L.n_pad, L.G, c->head_dim, 1024, c->R, L.cps, L.CsP, c->evict_every) <= 160 * 1024;
    for (int units : {L.U, c->batch * c->n_kv_heads}) {
      const SplitPlan pl = plan_split(L.n_pad, L.G, c->head_dim, c->R, L.cps, L.CsP, c->evict_every > 0 ? c->evict_every : 1,
                                      true, units, L.sp_force, fits);
      if (pl.S > L.sp_smax) L.sp_smax = pl.S;
      if (keep_all && keep_shares(units, L.n_pad) > L.sp_smax) L.sp_smax = keep_shares(units, L.n_pad);
    }
  }
  const bool sp = L.sp_smax > 1 || keep_all;  // (a layer that keeps every token always has the records and counters)
  L.offSpW = o; o = align_up(o + (sp && !keep_all ? U * (size_t)L.G * np * 4 : 0));
  L.offSpPart = o; o = align_up(o + (sp ? U * (size_t)L.sp_smax * split_part_floats(L.G, c->head_dim) * 4 : 0));
  L.offSpCnt = o; o = align_up(o + (sp ? U * 4 : 0));
  L.ring_bytes = o;
  o = 0;
  const size_t Nm = (size_t)c->max_prompt_len;
  // prompt-time scratch: fp32 keeps whole rows of weights; bf16 only softmax statistics per block of keys
  const size_t R16 = (R + 15) / 16 * 16, nblk = (Nm + PF_BLOCK - 1) / PF_BLOCK;
  L.offSrow = o;
  o = align_up(o + (c->dtype == MORPHKV_DTYPE_F32 ? U * R * Nm * 4 : U * nblk * (size_t)L.G * R16 * 8));
  L.offStat = o; o = align_up(o + U * (size_t)L.G * R16 * 8);
  L.offF = o; o = align_up(o + U * Nm * 4);
  L.offSel = o; o = align_up(o + U * (size_t)L.Cs * 4);
  L.offPlen = o; o = align_up(o + (size_t)c->batch * 4);
  L.offLseW = o; o = align_up(o + U * (size_t)L.G * R * 4);  // window rows' log-sum-exp from the prompt's attention pass
  L.scratch_bytes = o;
  return L;
}

}  // namespace

struct morphkv_handle {
  morphkv_config cfg;
  BufLayout L;
  char *cache, *ring, *scratch;
  float *dbgF;
  long long *dbgT;
  bool prefilled;
  unsigned steps;  // whole-model decode steps since the last prefill
  std::vector<unsigned> layer_steps;  // decode steps of each layer taken by per-layer calls
  float scale_log2;
  int n_cu;
  int force_threads;  // MORPHKV_DECODE_THREADS (multiple of 64 in 128..1024): tuning override, 0 = choose
  size_t min_lds;     // MORPHKV_DECODE_MIN_LDS (bytes): tuning override, asks for at least this much LDS per group
  int nt_k, nt_v;     // K tile groups / V tiles per unit that stream past the caches (see decode.h)
  int keep_cached_blocks;  // decode_keep_kernel: newest blocks of a unit that are read with ordinary loads
  int keep_kernel;    // MORPHKV_KEEP_KERNEL: 1 = the split kernel for layers that keep all, else the online-softmax kernel
  int rb_waves;       // waves of a workgroup that rebuild aggregates (see decode.h); MORPHKV_REBUILD_WAVES overrides
  bool keep_all;      // this handle's layers keep every token (Appendix A.6)
  // A configuration whose first layers keep every token is two handles: this one for the layers that select, and
  // `keep` for the first keep->cfg.n_layers layers; every call goes to both with its tensors split by layer
  morphkv_handle *keep;
  morphkv_config pub;  // the configuration as the caller gave it
};

namespace {

DecodeParams decode_params(const morphkv_handle *h) {
  DecodeParams P{};
  const BufLayout &L = h->L;
  P.K = h->cache + L.offK;
  P.V = h->cache + L.offV;
  P.pos = (int32_t *)(h->cache + L.offPos);
  P.meta = (int32_t *)(h->cache + L.offMeta);
  P.ring = (float *)(h->ring + L.offRing);
  P.sfx = (float *)(h->ring + L.offSfx);
  P.nw = (float *)(h->ring + L.offNw);
  P.dbgF = h->dbgF;
  P.dbgT = h->dbgT;
  // selection at the prompt only: the kernel runs its every-step schedule on a cache that never fills up
  P.C = h->cfg.C; P.T = h->cfg.evict_every > 0 ? h->cfg.evict_every : 1;
  P.evl = (int32_t *)(h->cache + L.offEvl);
  P.holes = (int32_t *)(h->cache + L.offHoles);
  P.zig = (int32_t)(h->steps & 1u);
  P.nt_k = h->nt_k;
  P.nt_v = h->nt_v;
  P.keep_cached_blocks = h->keep_cached_blocks;
  P.sp_w = (float *)(h->ring + L.offSpW);
  P.sp_part = (float *)(h->ring + L.offSpPart);
  P.sp_cnt = (int32_t *)(h->ring + L.offSpCnt);
  P.sp_smax = L.sp_smax;
  P.sp_bps = 0;
  P.keep_all = h->keep_all ? 1 : 0;
  P.cpt_shift = -1;
  for (int sft = 0; sft < 16; ++sft)
    if ((1 << sft) == L.cpt) P.cpt_shift = sft;
  P.Cs = L.Cs; P.CsP = L.CsP; P.R = h->cfg.R; P.n = L.n; P.n_pad = L.n_pad; P.Mq = h->cfg.n_q_heads;
  P.Mkv = h->cfg.n_kv_heads; P.fusion = h->cfg.fusion; P.cps = L.cps; P.cpt = L.cpt; P.scale_log2 = h->scale_log2;
  return P;
}

// scratch: the workspace the prompt-time kernels use (the caller's, or the library's own), carved up as L says
PrefillParams prefill_params(const morphkv_handle *h, char *scratch_base, const BufLayout &L) {
  PrefillParams P{};
  P.plen = (const int32_t *)(scratch_base + L.offPlen);
  P.Srow = (float *)(scratch_base + L.offSrow);
  P.Spart = (float2 *)(scratch_base + L.offSrow);
  P.Sfin = (float2 *)(scratch_base + L.offStat);
  P.F = (float *)(scratch_base + L.offF);
  P.sel = (int32_t *)(scratch_base + L.offSel);
  P.Kc = h->cache + L.offK;
  P.Vc = h->cache + L.offV;
  P.pos = (int32_t *)(h->cache + L.offPos);
  P.meta = (int32_t *)(h->cache + L.offMeta);
  P.evl = (int32_t *)(h->cache + L.offEvl);
  P.sp_cnt = (h->L.sp_smax > 1 || h->keep_all) ? (int32_t *)(h->ring + h->L.offSpCnt) : nullptr;
  P.keep_all = h->keep_all ? 1 : 0;
  P.T = h->cfg.evict_every > 0 ? h->cfg.evict_every : 1;
  P.ring = (float *)(h->ring + L.offRing);
  P.sfx = (float *)(h->ring + L.offSfx);
  P.nw = (float *)(h->ring + L.offNw);
  P.B = h->cfg.batch; P.Mq = h->cfg.n_q_heads; P.Mkv = h->cfg.n_kv_heads; P.C = h->cfg.C; P.Cs = L.Cs; P.CsP = L.CsP;
  P.R = h->cfg.R; P.n = L.n; P.n_pad = L.n_pad; P.fusion = h->cfg.fusion; P.cps = L.cps;
  P.scale_log2 = h->scale_log2;
  P.q_rows = h->cfg.R;
  P.q_prompt = 0;
  return P;
}

// threads per workgroup of the fused decode kernel: enough workgroups to cover the CUs several times
// over -> small groups (several co-resident per CU); about one unit per CU -> one large group.
int decode_threads(const morphkv_handle *h, int U) {
  if (h->force_threads) return h->force_threads;
  const int cu = h->n_cu > 0 ? h->n_cu : 256;
  if (U >= 8 * cu) return 128;
  if (U >= 4 * cu) return 256;
  if (U >= 2 * cu) return 512;
  // few units: the launch is a chain of latencies and of instructions that every wave issues (the four waves of a
  // SIMD share its issue slots), so: as few waves as take the cache's tile groups of 32 slots in the same number of
  // rounds as 16 waves would (c4 layer by layer, 17 groups: 9 waves, 515 -> 483 us per step; c2, 34 groups: 12
  // waves, 14.1 -> 13.7 us).  Long caches stream: all 16 waves.
  const int groups = h->L.n_pad / 32;
  if (h->cfg.dtype != MORPHKV_DTYPE_BF16) return h->L.n_pad < 1024 ? 512 : 1024;
  if (groups > 48) return 1024;
  const int rounds = (groups + 15) / 16;
  int nw = 4;
  while ((groups + nw - 1) / nw > rounds) ++nw;
  return 64 * nw;
}

// does the fused kernel's LDS-resident weight array fit (priced for its largest workgroup)?
bool fused_fits(const morphkv_handle *h) {
  return !h->keep_all && decode_lds_bytes(h->L.n_pad, h->L.G, h->cfg.head_dim, 1024, h->cfg.R, h->L.cps, h->L.CsP,
                          h->cfg.evict_every) <= 160 * 1024;
}
SplitPlan handle_plan(const morphkv_handle *h, int n_units) {
  return plan_split(h->L.n_pad, h->L.G, h->cfg.head_dim, h->cfg.R, h->L.cps, h->L.CsP,
                    h->cfg.evict_every > 0 ? h->cfg.evict_every : 1, h->cfg.dtype == MORPHKV_DTYPE_BF16, n_units,
                    h->L.sp_force, fused_fits(h));
}

int dispatch_decode(const morphkv_handle *h, const DecodeParams &P, int n_units, hipStream_t st) {
  const bool f32 = h->cfg.dtype == MORPHKV_DTYPE_F32;
  const int G = h->L.G, D = h->cfg.head_dim;
  DecodeLaunch L{};
  L.n_units = n_units;
  L.clocks = P.dbgT != nullptr;
  L.coarse = P.T > 1;
  L.stream = st;
  // (the kernels' dynamic-LDS limits were raised when the handle was made, on the device current then)
  // a layer that keeps every token runs in the kernel made for it (online softmax; one or two workgroups per unit
  // from 160 units on, several with a merge below that)
  if (h->keep_all && h->L.sp_force <= 0 && h->keep_kernel != 1) {
    if (L.clocks) return fail(MORPHKV_EINVAL, "phase clocks are built for the fused kernel only");
    // (workgroups of 256 threads, three to a compute unit, were measured even with one of 512 on launches of many
    // units: the override is for tests)
    L.threads = h->force_threads == 256 || h->force_threads == 512 ? h->force_threads : KEEP_NT;
    int S = keep_shares(n_units, P.n_pad);
    if (S > h->L.sp_smax) S = h->L.sp_smax;
    return launch_decode_keep(D, G, P, L, S);
  }
  const SplitPlan pl = handle_plan(h, n_units);
  if (pl.S == 0) return fail(MORPHKV_EINVAL, "C + R = %d is too large for the decode kernels' LDS", P.n);
  if (pl.S > 1 || h->keep_all) {
    // a cache beyond the fused kernel's LDS, or on request: the split kernel
    if (L.clocks) return fail(MORPHKV_EINVAL, "phase clocks are built for the fused kernel only");
    DecodeParams PS = P;
    PS.sp_bps = pl.bps;
    L.threads = SPLIT_NT;
    L.lds = decode_split_lds_bytes(pl.bps, G, D, P.R, P.cps, P.CsP, P.T);
    return launch_decode_split(D, G, PS, L, pl.S);
  }
  L.threads = decode_threads(h, n_units);
  if (f32 && L.threads > 512) L.threads = 512;  // fp32 builds: 256 registers a lane, groups of at most 512 threads
  L.lds = decode_lds_bytes(P.n_pad, G, D, L.threads, P.R, P.cps, P.CsP, P.T);
  if (L.lds > 160 * 1024) return fail(MORPHKV_EINVAL, "C + R = %d needs %zu bytes of LDS (limit 163840)", P.n, L.lds);
  // the rebuild's shape for this workgroup size: columns per group, waves that take part
  DecodeParams PF = P;
  {
    const int NW = L.threads / WAVE, rbw = h->rb_waves < NW ? h->rb_waves : NW;
    PF.rb_gw = turn_group_width(P.R, RB, P.cps, rbw);
    const int groups = (P.cps + PF.rb_gw - 1) / PF.rb_gw;
    PF.rb_nrw = groups < rbw ? groups : rbw;
  }
  if (h->min_lds > L.lds && h->min_lds <= 160 * 1024) L.lds = h->min_lds;
  if (f32) {
    if (L.clocks) return fail(MORPHKV_EINVAL, "phase clocks are built for bf16 caches with head_dim 128 only");
    return L.coarse ? launch_decode_f32_coarse(D, G, PF, L) : launch_decode_f32(D, G, PF, L);
  }
  if (L.clocks) return launch_decode_bf16_clocks(D, G, PF, L);
  return L.coarse ? launch_decode_bf16_coarse(D, G, PF, L) : launch_decode_bf16_product(D, G, PF, L);
}

// raises the decode kernels' dynamic-LDS limit for this handle's configuration on the current device (once, at
// creation: not inside a launch, which may be under stream capture); only ever raised, since another handle on
// the same device may need the larger value
int dispatch_lds_limit(const morphkv_handle *h, size_t lds, size_t lds_split) {
  static size_t limit[MAX_DEVICES][2][2][9] = {};  // [device][f32?][d == 128?][G]
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(MORPHKV_EHIP, "device index %d outside 0..%d", dev, MAX_DEVICES - 1);
  const bool f32 = h->cfg.dtype == MORPHKV_DTYPE_F32;
  const int G = h->L.G, D = h->cfg.head_dim;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  static size_t limit_split[MAX_DEVICES][2][9] = {};
  if (!f32 && lds_split > limit_split[dev][D == 128 ? 1 : 0][G]) {
    if (const int rc = decode_lds_limit_split(D, G, lds_split)) return rc;
    limit_split[dev][D == 128 ? 1 : 0][G] = lds_split;
  }
  size_t &cur = limit[dev][f32 ? 1 : 0][D == 128 ? 1 : 0][G];
  if (lds <= cur) return MORPHKV_OK;
  if (f32) {
    if (const int rc = decode_lds_limit_f32(D, G, lds)) return rc;
    if (const int rc = decode_lds_limit_f32_coarse(D, G, lds)) return rc;
  } else {
    if (const int rc = decode_lds_limit_bf16_product(D, G, lds)) return rc;
    if (const int rc = decode_lds_limit_bf16_coarse(D, G, lds)) return rc;
    if (const int rc = decode_lds_limit_bf16_clocks(D, G, lds)) return rc;
  }
  cur = lds;
  return MORPHKV_OK;
}

int dispatch_prefill(const morphkv_handle *h, const PrefillParams &P, hipStream_t st) {
  return h->cfg.dtype == MORPHKV_DTYPE_F32 ? launch_prefill_f32(h->cfg.head_dim, h->L.G, P, h->L.U, st)
                                           : launch_prefill_bf16(h->cfg.head_dim, h->L.G, P, h->L.U, st);
}

// A configuration with n_keep_all_layers = k > 0 is served by two handles: `keep` for the first k layers, which
// hold every token (prompt and response: C = max_prompt_len older slots filled at the prompt plus max_new_tokens
// more, nothing ever selected), and `sel` for the others.  Returns k.
int split_config(const morphkv_config *c, morphkv_config *keep, morphkv_config *sel) {
  const int k = c->n_keep_all_layers;
  *keep = *c;
  keep->n_layers = k;
  keep->n_keep_all_layers = 0;
  keep->C = c->max_prompt_len;
  keep->evict_every = 0;
  *sel = *c;
  sel->n_layers = c->n_layers - k;
  sel->n_keep_all_layers = 0;
  return k;
}

// bytes per layer of the tensors the calls take
struct LayerStrides { size_t q_win, kv_prompt, lse_win, q_prompt, lse_prompt, q_step, kv_step, out_step; };
LayerStrides layer_strides(const morphkv_config *c, int Nmax) {
  const size_t e = c->dtype == MORPHKV_DTYPE_F32 ? 4 : 2, B = (size_t)c->batch, M = (size_t)c->n_q_heads,
               Mk = (size_t)c->n_kv_heads, d = (size_t)c->head_dim, R = (size_t)c->R, N = (size_t)Nmax;
  return LayerStrides{B * M * R * d * e, B * Mk * N * d * e, B * M * R * 4, B * M * N * d * e, B * M * N * 4,
                      B * M * d * e,     B * Mk * d * e,     B * M * d * 4};
}
const void *adv(const void *p, size_t bytes) { return p ? (const char *)p + bytes : nullptr; }
void *adv(void *p, size_t bytes) { return p ? (char *)p + bytes : nullptr; }

// selection over the prompt from the window queries (all three window entries end up here)
int prefill_window(morphkv_handle *h, const void *Q_window, const void *K, const void *V, const float *lse_window,
                   const int32_t *prompt_len, int32_t Nmax, hipStream_t st, char *scratch_base, const BufLayout &Ls) {
  if (!Q_window || !K || !V || !prompt_len) return fail(MORPHKV_EINVAL, "null input pointer");
  if (Nmax < 1 || Nmax > h->cfg.max_prompt_len)
    return fail(MORPHKV_EINVAL, "Nmax %d outside 1..max_prompt_len (%d)", Nmax, h->cfg.max_prompt_len);
  for (int b = 0; b < h->cfg.batch; ++b)
    if (prompt_len[b] < 1 || prompt_len[b] > Nmax)
      return fail(MORPHKV_EINVAL, "prompt_len[%d] = %d outside 1..Nmax (%d)", b, prompt_len[b], Nmax);
  PrefillParams P = prefill_params(h, scratch_base, Ls);
  P.Qw = Q_window; P.K = K; P.V = V; P.Nmax = Nmax; P.lse = lse_window;
  if (const int rc = upload_ints((int32_t *)P.plen, prompt_len, h->cfg.batch, st)) return rc;
  const int rc = dispatch_prefill(h, P, st);
  if (rc) return rc;
  h->prefilled = true;
  h->steps = 0;
  std::fill(h->layer_steps.begin(), h->layer_steps.end(), 0u);
  return MORPHKV_OK;
}

}  // namespace

extern "C" {

const char *morphkv_last_error(void) { return g_err; }

int morphkv_sizes(const morphkv_config *cfg, size_t *cache_bytes, size_t *ring_bytes, size_t *scratch_bytes) {
  int rc = validate(cfg);
  if (rc) return rc;
  morphkv_config ck, cs;
  const int k = split_config(cfg, &ck, &cs);
  size_t cb = 0, rb = 0, sb = 0;
  if (k > 0) {
    const BufLayout L = make_layout(&ck, true);
    cb += L.cache_bytes; rb += L.ring_bytes; sb = std::max(sb, L.scratch_bytes);
  }
  if (k < cfg->n_layers) {
    const BufLayout L = make_layout(&cs, false);
    cb += L.cache_bytes; rb += L.ring_bytes; sb = std::max(sb, L.scratch_bytes);
  }
  if (cache_bytes) *cache_bytes = cb;
  if (ring_bytes) *ring_bytes = std::max<size_t>(rb, 256);
  if (scratch_bytes) *scratch_bytes = sb;
  return MORPHKV_OK;
}

// one handle over layers that all behave alike: cfg is the configuration of those layers alone
// budget_share: this segment's part of the memory-side cache budget (the segments of a handle share it by layers)
static int create_segment(morphkv_handle **out, const morphkv_config *cfg, bool keep_all, void *cache, void *scores_ring,
                          void *scratch, double budget_share) {
  *out = nullptr;
  morphkv_handle *h = new (std::nothrow) morphkv_handle();
  if (!h) return fail(MORPHKV_EINVAL, "out of host memory");
  h->cfg = *cfg;
  h->pub = *cfg;
  h->keep_all = keep_all;
  h->keep = nullptr;
  h->L = make_layout(cfg, keep_all);
  h->cache = (char *)cache;
  h->ring = (char *)scores_ring;
  h->scratch = (char *)scratch;
  h->dbgF = nullptr;
  h->dbgT = nullptr;
  h->prefilled = false;
  h->steps = 0;
  try {
    h->layer_steps.assign((size_t)cfg->n_layers, 0u);
  } catch (...) {
    delete h;
    return fail(MORPHKV_EINVAL, "out of host memory");
  }
  const double scale = cfg->softmax_scale != 0.0f ? (double)cfg->softmax_scale : 1.0 / std::sqrt((double)cfg->head_dim);
  h->scale_log2 = (float)(scale * 1.4426950408889634074);
  h->n_cu = 0;
  h->force_threads = 0;
  h->min_lds = 0;
  if (const char *e = std::getenv("MORPHKV_DECODE_MIN_LDS")) h->min_lds = (size_t)std::atol(e);
  // Which part of K/V streams past the caches.  The device has a 256 MB memory-side cache in front of HBM: a
  // step that reads more than that through ordinary loads evicts everything before the next step can reuse
  // it.  So only `budget` bytes of the handle's K/V are read with ordinary loads (V first, then the end of K:
  // they stay resident from step to step), the rest with the non-temporal hint, which neither displaces the
  // resident part nor pays for being inserted.
  h->nt_k = 0; h->nt_v = 0;
  if (cfg->dtype == MORPHKV_DTYPE_BF16) {
    double budget_mb = 208.0;
    if (const char *e = std::getenv("MORPHKV_CACHE_BUDGET_MB")) budget_mb = std::atof(e);
    budget_mb *= budget_share;
    // (a layer that keeps every token is mostly headroom: its kernel applies the budget to what is resident --
    // the newest keep_cached_blocks blocks of 32 slots of every unit are read with ordinary loads)
    h->keep_cached_blocks = (int)std::min(1.0e9, budget_mb * 1048576.0 / ((double)h->L.U * 32.0 * cfg->head_dim * 4.0));
    const double half = (double)h->L.U * h->L.n_pad * cfg->head_dim * 2.0;  // bytes of K (= bytes of V) of the handle
    const double stream = 2.0 * half - budget_mb * 1048576.0;              // bytes that have to stream
    const int kgroups = (h->L.n_pad / 16 + 1) / 2, vtiles = h->L.n_pad / 32;
    if (stream > 0.0) {
      const double fk = stream >= half ? 1.0 : stream / half, fv = stream > half ? (stream - half) / half : 0.0;
      h->nt_k = (int)(fk * kgroups + 0.5);
      h->nt_v = (int)((fv > 1.0 ? 1.0 : fv) * vtiles + 0.5);
    }
  }
  // How many waves of a workgroup rebuild aggregates (any number is correct; measured on this device): all of
  // them where the K pass is long enough to hide that every wave then runs the rebuild's code, few where it is not
  {
    const int kgroups = (h->L.n_pad / 16 + 1) / 2;
    h->rb_waves = kgroups >= 64 ? (cfg->R <= 128 ? 16 : 8) : kgroups >= 32 ? 4 : 2;
  }
  h->keep_kernel = 0;
  if (const char *e = std::getenv("MORPHKV_KEEP_KERNEL")) h->keep_kernel = !std::strcmp(e, "split") ? 1 : !std::strcmp(e, "stream") ? 2 : 0;
  if (const char *e = std::getenv("MORPHKV_REBUILD_WAVES")) {
    const int v = std::atoi(e);
    if (v >= 1 && v <= 16) h->rb_waves = v;
  }
  if (const char *e = std::getenv("MORPHKV_DECODE_THREADS")) {
    const int v = std::atoi(e);
    if (v >= 128 && v <= 1024 && v % 64 == 0) h->force_threads = v;
  }
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
    h->n_cu = prop.multiProcessorCount;
  else
    (void)hipGetLastError();
  // the fused decode kernel keeps one weight per (head, slot) in LDS; a cache too large for that runs in the split
  // kernel (bf16), whose shares are bounded instead: say so now if neither can take C + R
  const int upl = cfg->batch * cfg->n_kv_heads;
  size_t lds_max = 0, lds_split = 0;
  for (int units : {h->L.U, upl}) {
    const SplitPlan pl = handle_plan(h, units);
    if (pl.S == 0 && h->keep_all) continue;  // (beyond the split kernel's shares: decode_keep_kernel has no such bound)
    if (pl.S == 0) {
      const int n = h->L.n;
      delete h;
      return fail(MORPHKV_EINVAL, "C + R = %d needs more LDS than the decode kernels have (limit 163840 bytes)", n);
    }
    if (pl.S > 1 || h->keep_all) {
      const size_t lds = decode_split_lds_bytes(pl.bps, h->L.G, cfg->head_dim, cfg->R, h->L.cps, h->L.CsP,
                                                cfg->evict_every > 0 ? cfg->evict_every : 1);
      lds_split = lds > lds_split ? lds : lds_split;
      continue;
    }
    const size_t lds = decode_lds_bytes(h->L.n_pad, h->L.G, cfg->head_dim,
                                        cfg->dtype == MORPHKV_DTYPE_F32 ? std::min(decode_threads(h, units), 512)
                                                                        : decode_threads(h, units),
                                        cfg->R, h->L.cps, h->L.CsP, cfg->evict_every);
    if (lds > 160 * 1024) {
      const int n = h->L.n;
      delete h;
      return fail(MORPHKV_EINVAL, "C + R = %d needs %zu bytes of LDS in the decode kernel (limit 163840)", n, lds);
    }
    lds_max = lds > lds_max ? lds : lds_max;
  }
  if (h->min_lds > lds_max && h->min_lds <= 160 * 1024) lds_max = h->min_lds;
  if (const int rc = dispatch_lds_limit(h, lds_max, lds_split)) {
    delete h;
    return rc;
  }
  // set-up for morphkv_prefill_select_noalloc: the address of this device's copy of the library's workspace
  // is looked up here, once per device, not inside a call that may be under stream capture
  char *ws = nullptr;
  if (const int rc = static_scratch(&ws)) {
    delete h;
    return rc;
  }
  *out = h;
  return MORPHKV_OK;
}

int morphkv_create(morphkv_handle **out, const morphkv_config *cfg, void *cache, void *scores_ring, void *scratch) {
  if (!out) return fail(MORPHKV_EINVAL, "handle pointer is null");
  *out = nullptr;
  if (const int rc = validate(cfg)) return rc;
  if (!cache || !scores_ring || !scratch) return fail(MORPHKV_EINVAL, "cache, scores_ring and scratch must be non-null");
  if (((uintptr_t)cache | (uintptr_t)scores_ring | (uintptr_t)scratch) & 255)
    return fail(MORPHKV_EINVAL, "buffers must be 256-byte aligned");
  morphkv_config ck, cs;
  const int k = split_config(cfg, &ck, &cs);
  morphkv_handle *hk = nullptr, *hs = nullptr;
  size_t cache_k = 0, ring_k = 0;
  if (k > 0) {
    // the layers that keep every token come first in both buffers; the prompt-time workspace is shared (the two
    // parts of a call run one after the other on the caller's stream)
    if (const int rc = create_segment(&hk, &ck, true, cache, scores_ring, scratch, (double)k / cfg->n_layers)) return rc;
    cache_k = hk->L.cache_bytes;
    ring_k = hk->L.ring_bytes;
    if (k == cfg->n_layers) {
      hk->pub = *cfg;
      *out = hk;
      return MORPHKV_OK;
    }
  }
  if (const int rc = create_segment(&hs, &cs, false, (char *)cache + cache_k, (char *)scores_ring + ring_k, scratch,
                                    (double)(cfg->n_layers - k) / cfg->n_layers)) {
    delete hk;
    return rc;
  }
  hs->keep = hk;
  hs->pub = *cfg;
  *out = hs;
  return MORPHKV_OK;
}

int morphkv_destroy(morphkv_handle *h) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  delete h->keep;
  delete h;
  return MORPHKV_OK;
}

int morphkv_prefill_select(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                           const int32_t *prompt_len, int32_t Nmax, void *stream) {
  return morphkv_prefill_select_lse(h, Q_window, K, V, nullptr, prompt_len, Nmax, stream);
}

int morphkv_prefill_select_lse(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                               const float *lse_window, const int32_t *prompt_len, int32_t Nmax, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (h->keep) {  // the first layers keep every token: their part of the tensors comes first
    morphkv_handle *k = h->keep;
    if (const int rc = prefill_window(k, Q_window, K, V, lse_window, prompt_len, Nmax, (hipStream_t)stream, k->scratch, k->L))
      return rc;
    const LayerStrides ls = layer_strides(&h->pub, Nmax);
    const size_t nk = (size_t)k->cfg.n_layers;
    Q_window = adv(Q_window, nk * ls.q_win); K = adv(K, nk * ls.kv_prompt); V = adv(V, nk * ls.kv_prompt);
    lse_window = (const float *)adv((const void *)lse_window, nk * ls.lse_win);
  }
  return prefill_window(h, Q_window, K, V, lse_window, prompt_len, Nmax, (hipStream_t)stream, h->scratch, h->L);
}

static int prefill_noalloc_segment(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                                   const int32_t *prompt_len, int32_t Nmax, void *stream) {
  if (Nmax < 1 || Nmax > h->cfg.max_prompt_len)
    return fail(MORPHKV_EINVAL, "Nmax %d outside 1..max_prompt_len (%d)", Nmax, h->cfg.max_prompt_len);
  // the workspace is laid out for this call's Nmax, not for the handle's max_prompt_len
  morphkv_config c = h->cfg;
  c.max_prompt_len = Nmax;
  const BufLayout Ls = make_layout(&c, h->keep_all);
  if (Ls.scratch_bytes > STATIC_SCRATCH_BYTES)
    return fail(MORPHKV_EINVAL,
                "prefill_select_noalloc: this configuration with Nmax = %d needs %zu bytes of workspace, the library's "
                "own holds %zu (MORPHKV_NOALLOC_SCRATCH_BYTES); use morphkv_prefill_select with a caller-provided scratch",
                Nmax, Ls.scratch_bytes, STATIC_SCRATCH_BYTES);
  char *ws = nullptr;
  if (const int rc = static_scratch(&ws)) return rc;
  return prefill_window(h, Q_window, K, V, nullptr, prompt_len, Nmax, (hipStream_t)stream, ws, Ls);
}

int morphkv_prefill_select_noalloc(morphkv_handle *h, const void *Q_window, const void *K, const void *V,
                                   const int32_t *prompt_len, int32_t Nmax, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (h->keep) {
    if (const int rc = prefill_noalloc_segment(h->keep, Q_window, K, V, prompt_len, Nmax, stream)) return rc;
    const LayerStrides ls = layer_strides(&h->pub, Nmax);
    const size_t nk = (size_t)h->keep->cfg.n_layers;
    Q_window = adv(Q_window, nk * ls.q_win); K = adv(K, nk * ls.kv_prompt); V = adv(V, nk * ls.kv_prompt);
  }
  return prefill_noalloc_segment(h, Q_window, K, V, prompt_len, Nmax, stream);
}

static int attend_select_segment(morphkv_handle *h, const void *Q, const void *K, const void *V, void *O, float *lse,
                                 const int32_t *prompt_len, int32_t Nmax, void *stream) {
  if (!Q || !K || !V || !O || !prompt_len) return fail(MORPHKV_EINVAL, "null input pointer");
  if (h->cfg.dtype != MORPHKV_DTYPE_BF16)
    return fail(MORPHKV_EINVAL, "prefill_attend_select is built for bf16 only");
  if (Nmax < 1 || Nmax > h->cfg.max_prompt_len)
    return fail(MORPHKV_EINVAL, "Nmax %d outside 1..max_prompt_len (%d)", Nmax, h->cfg.max_prompt_len);
  for (int b = 0; b < h->cfg.batch; ++b)
    if (prompt_len[b] < 1 || prompt_len[b] > Nmax)
      return fail(MORPHKV_EINVAL, "prompt_len[%d] = %d outside 1..Nmax (%d)", b, prompt_len[b], Nmax);
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15)
    return fail(MORPHKV_EINVAL, "Q, K, V and O must be 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  PrefillParams P = prefill_params(h, h->scratch, h->L);
  if (const int rc = upload_ints((int32_t *)P.plen, prompt_len, h->cfg.batch, st)) return rc;
  PromptAttnParams A{};
  A.Q = (const bf16_t *)Q; A.K = (const bf16_t *)K; A.V = (const bf16_t *)V; A.O = (bf16_t *)O;
  A.lse = lse;
  A.lse_w = (float *)(h->scratch + h->L.offLseW);
  A.plen = P.plen;
  A.B = h->cfg.batch; A.Mq = h->cfg.n_q_heads; A.Mkv = h->cfg.n_kv_heads; A.R = h->cfg.R; A.Nmax = Nmax;
  A.scale_log2 = h->scale_log2;
  int rc = launch_prompt_attn(h->cfg.head_dim, h->L.G, A, h->L.U, st);
  if (rc) return rc;
  // selection over the prompt, with the window queries read in place and their normalisers from the pass above
  P.Qw = Q; P.q_rows = Nmax; P.q_prompt = 1;
  P.K = K; P.V = V; P.Nmax = Nmax; P.lse = A.lse_w;
  rc = dispatch_prefill(h, P, st);
  if (rc) return rc;
  h->prefilled = true;
  h->steps = 0;
  std::fill(h->layer_steps.begin(), h->layer_steps.end(), 0u);
  return MORPHKV_OK;
}

int morphkv_prefill_attend_select(morphkv_handle *h, const void *Q, const void *K, const void *V, void *O, float *lse,
                                  const int32_t *prompt_len, int32_t Nmax, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (h->keep) {
    if (const int rc = attend_select_segment(h->keep, Q, K, V, O, lse, prompt_len, Nmax, stream)) return rc;
    const LayerStrides ls = layer_strides(&h->pub, Nmax);
    const size_t nk = (size_t)h->keep->cfg.n_layers;
    Q = adv(Q, nk * ls.q_prompt); K = adv(K, nk * ls.kv_prompt); V = adv(V, nk * ls.kv_prompt);
    O = adv(O, nk * ls.q_prompt);
    lse = (float *)adv((void *)lse, nk * ls.lse_prompt);
  }
  return attend_select_segment(h, Q, K, V, O, lse, prompt_len, Nmax, stream);
}

static int decode_step_segment(morphkv_handle *h, const void *q, const void *k_new, const void *v_new, float *out,
                               void *stream) {
  if (!q || !k_new || !v_new || !out) return fail(MORPHKV_EINVAL, "null pointer");
  if (!h->prefilled) return fail(MORPHKV_ESTATE, "decode_step before prefill_select");
  if (h->cfg.evict_every == 0 &&
      h->steps + *std::max_element(h->layer_steps.begin(), h->layer_steps.end()) >= (unsigned)h->cfg.max_new_tokens)
    return fail(MORPHKV_ESTATE, "the cache has room for max_new_tokens = %d decode steps only", h->cfg.max_new_tokens);
  DecodeParams P = decode_params(h);
  P.q = q; P.k_new = k_new; P.v_new = v_new; P.out = out;
  const int rc = dispatch_decode(h, P, h->L.U, (hipStream_t)stream);
  if (rc == MORPHKV_OK) ++h->steps;
  return rc;
}

int morphkv_decode_step(morphkv_handle *h, const void *q, const void *k_new, const void *v_new, float *out,
                        void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (h->keep) {
    if (const int rc = decode_step_segment(h->keep, q, k_new, v_new, out, stream)) return rc;
    const LayerStrides ls = layer_strides(&h->pub, 1);
    const size_t nk = (size_t)h->keep->cfg.n_layers;
    q = adv(q, nk * ls.q_step); k_new = adv(k_new, nk * ls.kv_step); v_new = adv(v_new, nk * ls.kv_step);
    out = (float *)adv((void *)out, nk * ls.out_step);
  }
  return decode_step_segment(h, q, k_new, v_new, out, stream);
}

int morphkv_decode_step_layer(morphkv_handle *h, int32_t layer, const void *q, const void *k_new, const void *v_new,
                              float *out, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (h->keep) {  // the first layers live in the handle of the layers that keep every token
    if (layer >= 0 && layer < h->keep->cfg.n_layers)
      return morphkv_decode_step_layer(h->keep, layer, q, k_new, v_new, out, stream);
    if (layer < 0 || layer >= h->pub.n_layers)
      return fail(MORPHKV_EINVAL, "layer %d outside 0..%d", layer, h->pub.n_layers - 1);
    layer -= h->keep->cfg.n_layers;
  }
  if (!q || !k_new || !v_new || !out) return fail(MORPHKV_EINVAL, "null pointer");
  if (layer < 0 || layer >= h->cfg.n_layers)
    return fail(MORPHKV_EINVAL, "layer %d outside 0..%d", layer, h->cfg.n_layers - 1);
  if (!h->prefilled) return fail(MORPHKV_ESTATE, "decode_step_layer before prefill_select");
  if (h->cfg.evict_every == 0 && h->layer_steps[layer] + h->steps >= (unsigned)h->cfg.max_new_tokens)
    return fail(MORPHKV_ESTATE, "the cache has room for max_new_tokens = %d decode steps only", h->cfg.max_new_tokens);
  const int upl = h->cfg.batch * h->cfg.n_kv_heads;  // units per layer
  DecodeParams P = decode_params(h);
  P.u0 = layer * upl;
  P.io_u0 = P.u0;  // q, k_new, v_new and out are this layer's own tensors
  P.zig = (int32_t)(h->layer_steps[layer] & 1u);
  P.q = q; P.k_new = k_new; P.v_new = v_new; P.out = out;
  const int rc = dispatch_decode(h, P, upl, (hipStream_t)stream);
  if (rc == MORPHKV_OK) ++h->layer_steps[layer];
  return rc;
}

int morphkv_export_positions(morphkv_handle *h, int32_t *pos, int32_t *n_snap, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (!pos) return fail(MORPHKV_EINVAL, "pos is null");
  if (!h->prefilled) return fail(MORPHKV_ESTATE, "export before prefill_select");
  // rows are as long as the longest layer's; each layer's slots come first in its rows, -1 after them
  const int row = h->keep ? std::max(h->L.n, h->keep->L.n) : h->L.n;
  for (morphkv_handle *g : {h->keep, h}) {
    if (!g) continue;
    const BufLayout &L = g->L;
    hipLaunchKernelGGL(export_positions_kernel, dim3((row + 255) / 256, L.U), dim3(256), 0, (hipStream_t)stream,
                       (const int32_t *)(g->cache + L.offPos), (const int32_t *)(g->cache + L.offMeta), pos, n_snap,
                       L.n, L.n_pad, row, g->cfg.R);
    HIP_TRY(hipGetLastError());
    pos += (size_t)L.U * row;
    if (n_snap) n_snap += L.U;
  }
  return MORPHKV_OK;
}

int morphkv_export_evicted(morphkv_handle *h, int32_t *evicted, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (!evicted) return fail(MORPHKV_EINVAL, "evicted is null");
  if (!h->prefilled) return fail(MORPHKV_ESTATE, "export before prefill_select");
  for (morphkv_handle *g : {h->keep, h}) {
    if (!g) continue;
    const BufLayout &L = g->L;
    hipLaunchKernelGGL(export_evicted_kernel, dim3((L.U + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       (const int32_t *)(g->cache + L.offMeta), evicted, L.U);
    HIP_TRY(hipGetLastError());
    evicted += L.U;
  }
  return MORPHKV_OK;
}

int morphkv_export_evicted_list(morphkv_handle *h, int32_t *evicted, void *stream) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (!evicted) return fail(MORPHKV_EINVAL, "evicted is null");
  if (!h->prefilled) return fail(MORPHKV_ESTATE, "export before prefill_select");
  const int T = h->cfg.evict_every;
  if (T <= 1) return morphkv_export_evicted(h, evicted, stream);
  if (h->keep) {  // layers that keep every token evict nothing
    const size_t n = (size_t)h->keep->L.U * T;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, evicted, n, -1);
    HIP_TRY(hipGetLastError());
    evicted += n;
  }
  const BufLayout &L = h->L;
  HIP_TRY(hipMemcpyAsync(evicted, h->cache + L.offEvl, (size_t)L.U * T * 4, hipMemcpyDeviceToDevice,
                         (hipStream_t)stream));
  return MORPHKV_OK;
}

int morphkv_capture_scores(morphkv_handle *h, float *F) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  // rows of layers that keep every token are left untouched (they never score anything)
  h->dbgF = (F && h->keep) ? F + (size_t)h->keep->L.U * h->L.n_pad : F;
  return MORPHKV_OK;
}

int morphkv_calib_copy(void *dst, const void *src, size_t bytes, void *stream) {
  if (!dst || !src || (bytes & 15)) return fail(MORPHKV_EINVAL, "calib_copy needs non-null pointers and a multiple of 16 bytes");
  const size_t nvec = bytes / 16;
  if (nvec == 0) return MORPHKV_OK;
  const unsigned blocks = (unsigned)((nvec + 1023) / 1024 > 65535u * 16u ? 65535u * 16u : (nvec + 1023) / 1024);
  hipLaunchKernelGGL(calib_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (uint4 *)dst,
                     (const uint4 *)src, nvec);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}

int morphkv_calib_read(uint32_t *sink, const void *src, size_t bytes, void *stream) {
  if (!sink || !src || (bytes & 15)) return fail(MORPHKV_EINVAL, "calib_read needs non-null pointers and a multiple of 16 bytes");
  const size_t nvec = bytes / 16;
  if (nvec == 0) return MORPHKV_OK;
  // one 1024-thread group per CU (as the decode kernel runs c3), each on its own contiguous share
  int dev = 0, n_cu = 256;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
  else (void)hipGetLastError();
  const size_t per_block = (nvec + (size_t)n_cu - 1) / (size_t)n_cu;
  // beyond what the decode kernels would keep cache-resident the read streams with non-temporal loads, as they do
  if (bytes > ((size_t)208 << 20))
    hipLaunchKernelGGL(calib_read_kernel<true>, dim3(n_cu), dim3(1024), 0, (hipStream_t)stream, sink, (const uint4 *)src,
                       nvec, per_block);
  else
    hipLaunchKernelGGL(calib_read_kernel<false>, dim3(n_cu), dim3(1024), 0, (hipStream_t)stream, sink, (const uint4 *)src,
                       nvec, per_block);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}

int morphkv_decode_plan(morphkv_handle *h, int32_t n_units, int32_t *workgroups_per_unit, int32_t *blocks_per_workgroup) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  if (n_units < 1 || n_units > h->L.U) return fail(MORPHKV_EINVAL, "n_units %d outside 1..%d", n_units, h->L.U);
  SplitPlan pl = handle_plan(h, n_units);
  if (h->keep_all && h->L.sp_force <= 0 && h->keep_kernel != 1) {  // decode_keep_kernel: shares interleaved block by block
    pl.S = std::min(keep_shares(n_units, h->L.n_pad), h->L.sp_smax);
    pl.bps = (h->L.n_pad / 32 + pl.S - 1) / pl.S;
  }
  if (workgroups_per_unit) *workgroups_per_unit = pl.S;
  if (blocks_per_workgroup) *blocks_per_workgroup = pl.bps;
  return MORPHKV_OK;
}

int morphkv_capture_phase_clocks(morphkv_handle *h, long long *clocks) {
  if (!h) return fail(MORPHKV_EINVAL, "handle is null");
  h->dbgT = (clocks && h->keep) ? clocks + (size_t)h->keep->L.U * 8 : clocks;
  return MORPHKV_OK;
}

}  // extern "C"

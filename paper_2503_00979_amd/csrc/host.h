// Host-side declarations shared by the translation units of libmorphkv: error reporting and the launchers
// each unit exports for the kernels it holds (device code never crosses a unit's boundary).
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/morphkv.h"
#include "common.h"

namespace mkv {

struct DecodeParams;
struct PrefillParams;
struct PromptAttnParams;

// records the text morphkv_last_error() returns on this thread; returns `code`
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

#define HIP_TRY(expr)                                                                            \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) return mkv::fail(MORPHKV_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#define MKV_SWITCH_G(G, CALL)                                                          \
  switch (G) {                                                                         \
    case 1: { constexpr int G_ = 1; return CALL; }                                     \
    case 2: { constexpr int G_ = 2; return CALL; }                                     \
    case 3: { constexpr int G_ = 3; return CALL; }                                     \
    case 4: { constexpr int G_ = 4; return CALL; }                                     \
    case 5: { constexpr int G_ = 5; return CALL; }                                     \
    case 6: { constexpr int G_ = 6; return CALL; }                                     \
    case 7: { constexpr int G_ = 7; return CALL; }                                     \
    case 8: { constexpr int G_ = 8; return CALL; }                                     \
    default: return mkv::fail(MORPHKV_EINVAL, "group size %d not supported (1..8)", G); \
  }

struct DecodeLaunch {
  int n_units;     // workgroups
  int threads;     // per workgroup
  size_t lds;      // dynamic LDS bytes
  bool clocks;     // the build that stores phase time stamps (diagnostics)
  bool coarse;     // the build for selection every T > 1 steps
  hipStream_t stream;
};

// fused decode step, one workgroup per unit (decode_bf16.hip, decode_bf16_coarse.hip, decode_bf16_clk.hip,
// decode_f32.hip, decode_f32_coarse.hip); the clocks build takes any selection schedule
int launch_decode_bf16_product(int D, int G, const DecodeParams &P, const DecodeLaunch &L);
int launch_decode_bf16_coarse(int D, int G, const DecodeParams &P, const DecodeLaunch &L);
int launch_decode_bf16_clocks(int D, int G, const DecodeParams &P, const DecodeLaunch &L);
int launch_decode_f32(int D, int G, const DecodeParams &P, const DecodeLaunch &L);
int launch_decode_f32_coarse(int D, int G, const DecodeParams &P, const DecodeLaunch &L);
// the same step with S workgroups per unit (decode_split.hip); L.threads is ignored (fixed by the kernel)
int launch_decode_split(int D, int G, const DecodeParams &P, const DecodeLaunch &L, int S);
int decode_lds_limit_split(int D, int G, size_t lds);
// the step of layers that keep every token, S workgroups of L.threads (256 or 512) per unit, online softmax
// (decode_keep.hip); L.lds is ignored (follows from the threads)
int launch_decode_keep(int D, int G, const DecodeParams &P, const DecodeLaunch &L, int S);
// raise the kernels' dynamic-LDS limit on the current device
int decode_lds_limit_bf16_product(int D, int G, size_t lds);
int decode_lds_limit_bf16_coarse(int D, int G, size_t lds);
int decode_lds_limit_bf16_clocks(int D, int G, size_t lds);
int decode_lds_limit_f32(int D, int G, size_t lds);
int decode_lds_limit_f32_coarse(int D, int G, size_t lds);

// selection over the prompt (prefill_bf16.hip, prefill_f32.hip); the two steps both element types share
// (top-C select, aggregate state of the columns) live in prefill_f32.hip
int launch_prefill_bf16(int D, int G, const PrefillParams &P, int U, hipStream_t st);
int launch_prefill_f32(int D, int G, const PrefillParams &P, int U, hipStream_t st);
int launch_prefill_select(const PrefillParams &P, int U, hipStream_t st);
int launch_prefill_state(const PrefillParams &P, int U, hipStream_t st);

// causal attention over the prompt, bf16 (prompt_attn.hip)
int launch_prompt_attn(int D, int G, const PromptAttnParams &P, int U, hipStream_t st);

}  // namespace mkv

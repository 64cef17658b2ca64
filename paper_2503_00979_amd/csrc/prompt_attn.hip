// Causal attention over the prompt, bf16: head_dim 64 / 128, group sizes 1..8.
#include "host.h"
#include "prompt_attn.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const PromptAttnParams &P, int U, hipStream_t st) {
  using Cf = PromptAttnCfg<D, G>;
  // more LDS than a launch gets by default; asked for at every call (a call lasts milliseconds, and the
  // attribute belongs to the current device)
  HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&prompt_attn_kernel<D, G>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cf::lds_bytes));
  const int ntask = (P.Nmax + 31) / 32 * G;  // (32-row block, head) pairs of one KV head
  hipLaunchKernelGGL((prompt_attn_kernel<D, G>), dim3((ntask + Cf::NWV - 1) / Cf::NWV, U), dim3(Cf::NT), Cf::lds_bytes,
                     st, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
}  // namespace

int launch_prompt_attn(int D, int G, const PromptAttnParams &P, int U, hipStream_t st) {
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, U, st))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, U, st)))
}
}  // namespace mkv

// Diagnostics builds of the fused decode step (bf16, head_dim 128; one per selection schedule, like the product's):
// the same kernel with the phase time stamps of morphkv_capture_phase_clocks compiled in.  The product builds carry none of that code.
#include "host.h"
#include "decode.h"

namespace mkv {
namespace {
template <int G>
int launch(const DecodeParams &P, const DecodeLaunch &L) {
  if (L.coarse)
    hipLaunchKernelGGL((decode_fused_kernel<bf16_t, 128, G, true, true>), dim3(L.n_units), dim3(L.threads), L.lds, L.stream, P);
  else
    hipLaunchKernelGGL((decode_fused_kernel<bf16_t, 128, G, true, false>), dim3(L.n_units), dim3(L.threads), L.lds, L.stream, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
template <int G>
int lds_limit(size_t lds) {
  HIP_TRY(hipFuncSetAttribute((const void *)decode_fused_kernel<bf16_t, 128, G, true, true>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  HIP_TRY(hipFuncSetAttribute((const void *)decode_fused_kernel<bf16_t, 128, G, true, false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  return MORPHKV_OK;
}
}  // namespace

int launch_decode_bf16_clocks(int D, int G, const DecodeParams &P, const DecodeLaunch &L) {
  if (D != 128) return fail(MORPHKV_EINVAL, "phase clocks are built for bf16 caches with head_dim 128 only");
  MKV_SWITCH_G(G, (launch<G_>(P, L)))
}
int decode_lds_limit_bf16_clocks(int D, int G, size_t lds) {
  if (D != 128) return MORPHKV_OK;
  MKV_SWITCH_G(G, (lds_limit<G_>(lds)))
}
}  // namespace mkv

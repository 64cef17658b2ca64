// Fused decode step, bf16 caches (MFMA path), selection at every step: the product builds for head_dim 64 / 128
// and group sizes 1..8.
#include "host.h"
#include "decode.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const DecodeParams &P, const DecodeLaunch &L) {
  hipLaunchKernelGGL((decode_fused_kernel<bf16_t, D, G, false, false>), dim3(L.n_units), dim3(L.threads), L.lds, L.stream, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
template <int D, int G>
int lds_limit(size_t lds) {
  HIP_TRY(hipFuncSetAttribute((const void *)decode_fused_kernel<bf16_t, D, G, false, false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  return MORPHKV_OK;
}
}  // namespace

int launch_decode_bf16_product(int D, int G, const DecodeParams &P, const DecodeLaunch &L) {
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, L))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, L)))
}
int decode_lds_limit_bf16_product(int D, int G, size_t lds) {
  if (D == 128) { MKV_SWITCH_G(G, (lds_limit<128, G_>(lds))) }
  MKV_SWITCH_G(G, (lds_limit<64, G_>(lds)))
}
}  // namespace mkv

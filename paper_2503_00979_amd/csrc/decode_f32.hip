// Fused decode step, fp32 caches (plain FMA path; small and toy configurations), selection at every step: head_dim 64 / 128,
// group sizes 1..8.  These builds keep G x 4 products per lane in flight and get 256 registers: workgroups of at most
// 512 threads.
#include "host.h"
#include "decode.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const DecodeParams &P, const DecodeLaunch &L) {
  hipLaunchKernelGGL((decode_fused_kernel_512<float, D, G, false>), dim3(L.n_units), dim3(L.threads), L.lds, L.stream, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
template <int D, int G>
int lds_limit(size_t lds) {
  HIP_TRY(hipFuncSetAttribute((const void *)decode_fused_kernel_512<float, D, G, false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  return MORPHKV_OK;
}
}  // namespace

int launch_decode_f32(int D, int G, const DecodeParams &P, const DecodeLaunch &L) {
  if (L.threads > 512) return fail(MORPHKV_EINVAL, "fp32 decode kernels run in workgroups of at most 512 threads");
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, L))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, L)))
}
int decode_lds_limit_f32(int D, int G, size_t lds) {
  if (D == 128) { MKV_SWITCH_G(G, (lds_limit<128, G_>(lds))) }
  MKV_SWITCH_G(G, (lds_limit<64, G_>(lds)))
}
}  // namespace mkv

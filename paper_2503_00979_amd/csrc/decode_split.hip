// Decode step with a unit's cache split over several workgroups (bf16 caches): head_dim 64 / 128, group sizes 1..8.
#include "host.h"
#include "decode_split.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const DecodeParams &P, const DecodeLaunch &L, int S) {
  hipLaunchKernelGGL((decode_split_kernel<D, G>), dim3(S, L.n_units), dim3(SPLIT_NT), L.lds, L.stream, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
template <int D, int G>
int lds_limit(size_t lds) {
  HIP_TRY(hipFuncSetAttribute((const void *)decode_split_kernel<D, G>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds));
  return MORPHKV_OK;
}
}  // namespace

int launch_decode_split(int D, int G, const DecodeParams &P, const DecodeLaunch &L, int S) {
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, L, S))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, L, S)))
}
int decode_lds_limit_split(int D, int G, size_t lds) {
  if (D == 128) { MKV_SWITCH_G(G, (lds_limit<128, G_>(lds))) }
  MKV_SWITCH_G(G, (lds_limit<64, G_>(lds)))
}
}  // namespace mkv

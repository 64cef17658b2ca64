// Decode step of layers that keep every token (Appendix A.6), S workgroups per unit with an online softmax
// (bf16 caches): head_dim 64 / 128, group sizes 1..8.
#include "host.h"
#include "decode_keep.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const DecodeParams &P, const DecodeLaunch &L, int S) {
  hipLaunchKernelGGL((decode_keep_kernel<D, G>), dim3(S, L.n_units), dim3(L.threads), decode_keep_lds_bytes(G, D, L.threads), L.stream, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
}  // namespace

int launch_decode_keep(int D, int G, const DecodeParams &P, const DecodeLaunch &L, int S) {
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, L, S))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, L, S)))
}
}  // namespace mkv

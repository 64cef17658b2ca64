// Selection over the prompt, bf16 (key-major MFMA passes, radix select, tiled gather): head_dim 64 / 128, group
// sizes 1..8.
#include "host.h"
#include "prefill.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const PrefillParams &P, int U, hipStream_t st) {
  const int nblk = (P.Nmax + PF_BLOCK - 1) / PF_BLOCK;
  if (P.keep_all) {
    // every prompt token is kept (the capacity covers the prompt): positions 0 .. N-R-1 in order, then the gather
    if (const int rc = launch_prefill_select(P, U, st)) return rc;
    hipLaunchKernelGGL((prefill_gather_tiled_kernel<D>), dim3(P.n_pad / 32, U), dim3(256), 0, st, P);
    HIP_TRY(hipGetLastError());
    return MORPHKV_OK;
  }
  if (P.lse) {
    hipLaunchKernelGGL((prefill_stats_from_lse_kernel<G>), dim3(U, G, (P.R + 63) / 64), dim3(64), 0, st, P);
    HIP_TRY(hipGetLastError());
  } else {
    hipLaunchKernelGGL((prefill_pass_kernel<D, G, PF_STATS>), dim3(nblk, U), dim3(256), 0, st, P);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL((prefill_stats_merge_kernel<G>), dim3(U, G, (P.R + 63) / 64), dim3(64), 0, st, P, nblk);
    HIP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL((prefill_pass_kernel<D, G, PF_FUSE>), dim3(nblk, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  if (const int rc = launch_prefill_select(P, U, st)) return rc;
  hipLaunchKernelGGL((prefill_gather_tiled_kernel<D>), dim3(P.n_pad / 32, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL((prefill_pass_kernel<D, G, PF_RING>), dim3((P.n_pad + PF_BLOCK - 1) / PF_BLOCK, U), dim3(256), 0,
                     st, P);
  HIP_TRY(hipGetLastError());
  return launch_prefill_state(P, U, st);
}
}  // namespace

int launch_prefill_bf16(int D, int G, const PrefillParams &P, int U, hipStream_t st) {
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, U, st))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, U, st)))
}
}  // namespace mkv

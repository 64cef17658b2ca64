// Selection over the prompt, fp32 (plain FMA rows; small and toy configurations): head_dim 64 / 128, group sizes
// 1..8 -- and the two steps both element types share: the top-C select and the aggregate state of the columns.
#include "host.h"
#include "prefill_shared.h"

namespace mkv {
namespace {
template <int D, int G>
int launch(const PrefillParams &P, int U, hipStream_t st) {
  hipLaunchKernelGGL((prefill_rows_kernel<float, D, G>), dim3(P.R, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(prefill_fuse_kernel, dim3((P.Nmax + 255) / 256, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  if (const int rc = launch_prefill_select(P, U, st)) return rc;
  constexpr int SPB = 256 / (2 * (D / Elem<float>::EPL));
  hipLaunchKernelGGL((prefill_gather_kernel<float, D>), dim3((P.n_pad + SPB - 1) / SPB, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(prefill_ring_kernel, dim3((P.n_pad + 255) / 256, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  return launch_prefill_state(P, U, st);
}
}  // namespace

int launch_prefill_select(const PrefillParams &P, int U, hipStream_t st) {
  hipLaunchKernelGGL(prefill_select_kernel, dim3(U), dim3(1024), 0, st, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}
int launch_prefill_state(const PrefillParams &P, int U, hipStream_t st) {
  hipLaunchKernelGGL(prefill_state_kernel, dim3((P.CsP + 255) / 256, U), dim3(256), 0, st, P);
  HIP_TRY(hipGetLastError());
  return MORPHKV_OK;
}

int launch_prefill_f32(int D, int G, const PrefillParams &P, int U, hipStream_t st) {
  if (D == 128) { MKV_SWITCH_G(G, (launch<128, G_>(P, U, st))) }
  MKV_SWITCH_G(G, (launch<64, G_>(P, U, st)))
}
}  // namespace mkv

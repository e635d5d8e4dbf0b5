// Causal prefill attention over the compact cache: the host-side plan of key ranges and the
// dispatch on the score width; the kernel is in rap_prefill_kernel.h.
#include "rap_device.h"

namespace rap {

namespace {
constexpr int kKeysPerTile = 64;     // rows of a staged tile, as in the kernel
}

hipError_t launch_prefill_kch1(const PrefillArgs& a, hipStream_t stream);
hipError_t launch_prefill_kch2(const PrefillArgs& a, hipStream_t stream);
hipError_t launch_prefill_kch3(const PrefillArgs& a, hipStream_t stream);
hipError_t launch_prefill_kch4(const PrefillArgs& a, hipStream_t stream);

PrefillPlan prefill_plan(int batch, int n_kv, int group, int d_k, int d_v, int n_new, int max_len) {
  // column blocks per wavefront as the instantiation table (launch_prefill_k and the four callers) picks them
  const int kch = (d_k + 31) / 32, nt = (d_v + 15) / 16;
  const int nq = (kch == 4 || nt >= 7) ? kPrefillBlocksWide : kPrefillBlocks;
  PrefillPlan p;
  p.tok_per_wg = (64 * nq) / group;
  p.n_qblk = (n_new + p.tok_per_wg - 1) / p.tok_per_wg;
  p.n_ksplit = 1;
  p.tiles_per_split = 0;
  const long long base = static_cast<long long>(p.n_qblk) * n_kv * batch;
  const int tiles = (max_len + kKeysPerTile - 1) / kKeysPerTile;
  if (base > 0 && base < 384 && tiles >= 8) {
    const int want = static_cast<int>((512 + base - 1) / base);
    int per = (tiles + want - 1) / want;
    if (per < 4) per = 4;
    p.tiles_per_split = per;
    p.n_ksplit = (tiles + per - 1) / per;
  }
  return p;
}

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream) {
  switch ((a.d_k + 31) / 32) {
    case 1: return launch_prefill_kch1(a, stream);
    case 2: return launch_prefill_kch2(a, stream);
    case 3: return launch_prefill_kch3(a, stream);
    case 4: return launch_prefill_kch4(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rap

// Prefill attention kernels for score widths d_k in (64, 96] (KCH = 3 fragments of 32).
#include "rap_prefill_kernel.h"

namespace rap {

hipError_t launch_prefill_kch3(const PrefillArgs& a, hipStream_t stream) { return launch_prefill_k<3, kPrefillBlocks>(a, stream); }

}  // namespace rap

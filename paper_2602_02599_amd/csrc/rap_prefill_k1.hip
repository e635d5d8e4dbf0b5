// Prefill attention kernels for score widths d_k in (0, 32] (KCH = 1 fragments of 32).
#include "rap_prefill_kernel.h"

namespace rap {

hipError_t launch_prefill_kch1(const PrefillArgs& a, hipStream_t stream) { return launch_prefill_k<1, kPrefillBlocks>(a, stream); }

}  // namespace rap

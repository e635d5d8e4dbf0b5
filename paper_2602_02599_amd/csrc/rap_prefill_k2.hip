// Prefill attention kernels for score widths d_k in (32, 64] (KCH = 2 fragments of 32).
#include "rap_prefill_kernel.h"

namespace rap {

hipError_t launch_prefill_kch2(const PrefillArgs& a, hipStream_t stream) { return launch_prefill_k<2, kPrefillBlocks>(a, stream); }

}  // namespace rap

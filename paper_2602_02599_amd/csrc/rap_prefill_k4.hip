// Prefill attention kernels for score widths d_k in (96, 128] (KCH = 4 fragments of 32).
#include "rap_prefill_kernel.h"

namespace rap {

hipError_t launch_prefill_kch4(const PrefillArgs& a, hipStream_t stream) { return launch_prefill_k<4, kPrefillBlocksWide>(a, stream); }

}  // namespace rap

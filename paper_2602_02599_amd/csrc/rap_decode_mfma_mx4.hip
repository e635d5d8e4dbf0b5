// Dispatch of the matrix-core decode kernel over 4-bit (microscaling FP4) caches: one instantiation
// per (blocks of a K row, blocks of a V row), dense caches (the kernel itself: rap_decode_kernel.h).
#include "rap_decode_kernel.h"

namespace rap {

namespace {

template <int KCH>
hipError_t launch_v(const DecodeArgs& a, hipStream_t stream) {
  switch (mx_blocks(a.d_v)) {
    case 1: return launch_inst2<KCH, 2, true, false, false, false, true>(a, stream);
    case 2: return launch_inst2<KCH, 4, true, false, false, false, true>(a, stream);
    case 3: return launch_inst2<KCH, 6, true, false, false, false, true>(a, stream);
    case 4: return launch_inst2<KCH, 8, true, false, false, false, true>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_decode_mfma_mx4(const DecodeArgs& a, hipStream_t stream) {
  switch (mx_blocks(a.d_k)) {
    case 1: return launch_v<1>(a, stream);
    case 2: return launch_v<2>(a, stream);
    case 3: return launch_v<3>(a, stream);
    case 4: return launch_v<4>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rap

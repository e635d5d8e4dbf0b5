// Dispatch of the matrix-core decode kernel over caches of one-byte E4M3 codes (the kernel itself:
// rap_decode_kernel.h).  NT is 4 or 8 (blocks of 64 V channels); AL marks row widths at which every
// fragment read is naturally aligned in LDS (d_k a multiple of 8, d_v of 4) and needs no byte shifts.
#include "rap_decode_kernel.h"

namespace rap {

namespace {

template <int KCH, int NT>
hipError_t launch_q8_inst(const DecodeArgs& a, hipStream_t stream) {
  const bool paged = a.block_table != nullptr;
  const bool aligned = (a.d_k % 8) == 0 && (a.d_v % 4) == 0;
  if (aligned) return paged ? launch_inst2<KCH, NT, false, true, true, true>(a, stream) : launch_inst2<KCH, NT, false, false, true, true>(a, stream);
  return paged ? launch_inst2<KCH, NT, false, true, true, false>(a, stream) : launch_inst2<KCH, NT, false, false, true, false>(a, stream);
}

template <int KCH>
hipError_t launch_q8_k(const DecodeArgs& a, hipStream_t stream) {
  switch (decode_v_tiles(a.d_v, true)) {
    case 4: return launch_q8_inst<KCH, 4>(a, stream);
    case 8: return launch_q8_inst<KCH, 8>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_decode_mfma_q8(const DecodeArgs& a, hipStream_t stream) {
  switch ((a.d_k + 31) / 32) {
    case 1: return launch_q8_k<1>(a, stream);
    case 2: return launch_q8_k<2>(a, stream);
    case 3: return launch_q8_k<3>(a, stream);
    case 4: return launch_q8_k<4>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rap

// Dispatch of the matrix-core decode kernel over bf16 caches (the kernel itself: rap_decode_kernel.h),
// and the LDS size both element types need.
#include "rap_decode_kernel.h"

namespace rap {

hipError_t launch_decode_mfma_q8(const DecodeArgs& a, hipStream_t stream);   // rap_decode_mfma_q8.hip
hipError_t launch_decode_mfma_mx4(const DecodeArgs& a, hipStream_t stream);  // rap_decode_mfma_mx4.hip

namespace {

template <int KCH, int NT, bool VPAIR>
hipError_t launch_inst(const DecodeArgs& a, hipStream_t stream) {
  if (a.block_table != nullptr) return launch_inst2<KCH, NT, VPAIR, true, false>(a, stream);
  return launch_inst2<KCH, NT, VPAIR, false, false>(a, stream);
}

template <int KCH>
hipError_t launch_k(const DecodeArgs& a, hipStream_t stream) {
  const int nt = decode_v_tiles(a.d_v, false);
  if ((a.d_v & 1) == 0 && (nt & 1) == 0) {   // paired 4-byte V reads
    switch (nt) {
      case 2: return launch_inst<KCH, 2, true>(a, stream);
      case 4: return launch_inst<KCH, 4, true>(a, stream);
      case 6: return launch_inst<KCH, 6, true>(a, stream);
      case 8: return launch_inst<KCH, 8, true>(a, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (nt) {
    case 1: return launch_inst<KCH, 1, false>(a, stream);
    case 2: return launch_inst<KCH, 2, false>(a, stream);
    case 3: return launch_inst<KCH, 3, false>(a, stream);
    case 4: return launch_inst<KCH, 4, false>(a, stream);
    case 5: return launch_inst<KCH, 5, false>(a, stream);
    case 6: return launch_inst<KCH, 6, false>(a, stream);
    case 7: return launch_inst<KCH, 7, false>(a, stream);
    case 8: return launch_inst<KCH, 8, false>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// LDS bytes one wavefront needs: its K tile, its V tile and slack for the fragment reads that run
// past the last row, or the hand-over area of the final fold, whichever is larger.
// (4-bit caches: the tile is widened on its way into LDS, to rows of 32 bf16 per block plus 16 bytes.)
int mfma_lds_wave_bytes(int d_k, int d_v, bool q8, int cols, bool mx4) {
  const int nt = mx4 ? 2 * mx_blocks(d_v) : decode_v_tiles(d_v, q8);
  const int tiles = mx4 ? 32 * (mx4_row_pitch(mx_blocks(d_k)) + mx4_row_pitch(nt / 2)) + 128
                        : 1024 * (k_tile_loads((d_k + 31) / 32, q8) + v_tile_loads(nt, q8)) + 128;
  const int fold = (32 + (cols > kMaxGroup ? kMaxCols : kMaxGroup) * 16 * nt) * 4;
  const int need = tiles > fold ? tiles : fold;
  return (need + 127) / 128 * 128;
}

hipError_t launch_decode_mfma(const DecodeArgs& a, hipStream_t stream) {
  if (a.k_scales4 != nullptr) return launch_decode_mfma_mx4(a, stream);
  if (a.k_scale != nullptr) return launch_decode_mfma_q8(a, stream);
  switch ((a.d_k + 31) / 32) {
    case 1: return launch_k<1>(a, stream);
    case 2: return launch_k<2>(a, stream);
    case 3: return launch_k<3>(a, stream);
    case 4: return launch_k<4>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rap

// The pieces of librap's arithmetic and indexing that are our own and can go wrong silently: the
// rounding to bf16, the sine / cosine of the rotation angle, the first (software) half of the
// rounding to E4M3, and the rule that says which 16-byte loads of a cache tile are issued.  They
// are plain functions of their arguments, compiled for the device and for the host, so that the
// CPU tests run the very code the kernels run (tests/host/rap_arith_host.hip, under the host
// sanitizers).
#ifndef RAP_ARITH_H_
#define RAP_ARITH_H_

#include <hip/hip_runtime.h>

#include <math.h>
#include <stdint.h>

namespace rap {

__host__ __device__ __forceinline__ uint32_t f32_bits(float f) { return __builtin_bit_cast(uint32_t, f); }
__host__ __device__ __forceinline__ float bits_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

// bf16 bit pattern -> fp32 (a bf16 is the upper half of a binary32)
__host__ __device__ __forceinline__ float bf16_lo(uint32_t packed) { return bits_f32(packed << 16); }
__host__ __device__ __forceinline__ float bf16_hi(uint32_t packed) { return bits_f32(packed & 0xffff0000u); }
__host__ __device__ __forceinline__ float bf16_to_f32(uint16_t b) { return bits_f32(static_cast<uint32_t>(b) << 16); }

// fp64 -> bf16 with a single round-to-nearest-even.  The conversion to fp32 (nearest even) cannot
// carry a value across a bf16 rounding boundary, because every such boundary is an fp32 number; it
// can only land ON one (low half exactly 0x8000) from either side.  In that case the fp32 is
// moved one step back towards the side x came from, after which rounding the fp32 to its upper 16
// bits gives the correctly rounded result.
__host__ __device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
  const float f = static_cast<float>(x);
  const uint32_t u0 = f32_bits(f);
  const double fd = static_cast<double>(f);
  uint32_t u = u0 + ((fabs(x) > fabs(fd)) ? 1u : 0u);               // sign-magnitude: +1 is away from zero
  u -= (fabs(x) < fabs(fd)) ? 1u : 0u;
  u = (u0 & 0xffffu) == 0x8000u ? u : u0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(x != x ? (u0 >> 16) | 0x40u : u >> 16);   // NaN stays NaN
}

// sin and cos of an fp64 angle, both within about 1.5e-16 of the true values for |phi| up to 2^31:
// the nearest multiple of pi/2 is taken off with two fused multiply-adds against a two-part pi/2
// (a fused multiply-add rounds once, after the cancellation), then Taylor polynomials up to
// r^15 / r^16 on |r| <= pi/4, whose first left-out terms are below 5e-17.  The library routine
// costs several times as much because it also covers angles beyond 2^31 with a table-driven
// reduction.  Only multiplications, fused multiply-adds and one rounding to integer: the host and
// the device compute the same bits.
__host__ __device__ __forceinline__ void sincos_f64(double phi, double* s, double* c) {
  const double k = rint(phi * 0.63661977236758134308);
  double r = fma(-k, 1.5707963267948965580e+00, phi);
  r = fma(-k, 6.1232339957367660359e-17, r);
  const double z = r * r;
  double ps = -1.0 / 1307674368000.0;                 // -1/15!
  ps = fma(ps, z, 1.0 / 6227020800.0);
  ps = fma(ps, z, -1.0 / 39916800.0);
  ps = fma(ps, z, 1.0 / 362880.0);
  ps = fma(ps, z, -1.0 / 5040.0);
  ps = fma(ps, z, 1.0 / 120.0);
  ps = fma(ps, z, -1.0 / 6.0);
  const double sr = fma(r * z, ps, r);
  double pc = 1.0 / 20922789888000.0;                 // 1/16!
  pc = fma(pc, z, -1.0 / 87178291200.0);
  pc = fma(pc, z, 1.0 / 479001600.0);
  pc = fma(pc, z, -1.0 / 3628800.0);
  pc = fma(pc, z, 1.0 / 40320.0);
  pc = fma(pc, z, -1.0 / 720.0);
  pc = fma(pc, z, 1.0 / 24.0);
  pc = fma(pc, z, -0.5);
  const double cr = fma(z, pc, 1.0);
  const long long n = static_cast<long long>(k) & 3;   // quadrant
  const double a = (n & 1) ? cr : sr, b = (n & 1) ? sr : cr;
  *s = (n & 2) ? -a : a;
  *c = ((n + 1) & 2) ? -b : b;
}

// First half of fp64 -> E4M3: the value, clamped to the largest E4M3 magnitude 448, brought to
// fp32 by ROUNDING TO ODD (truncate towards zero, then set the last mantissa bit if anything was
// cut off).  A value rounded to odd keeps every fact a later nearest-even rounding to a format at
// least two bits shorter needs, so the conversion instruction that follows on the device
// (fp32 -> E4M3, nearest even) yields the single correct rounding of the fp64 value.  NaN must be
// handled by the caller.
__host__ __device__ __forceinline__ float f64_to_f32_odd_clamped448(double y) {
  y = y > 448.0 ? 448.0 : (y < -448.0 ? -448.0 : y);
  const float f = static_cast<float>(y);            // nearest-even; repaired to round-to-odd below
  uint32_t bits = f32_bits(f);
  const double d = static_cast<double>(f);
  if (d != y) {
    if (fabs(d) > fabs(y)) bits -= 1u;              // went away from zero: step back to the truncation
    bits |= 1u;
  }
  return bits_f32(bits);
}

// Which loads of a cache tile the decode kernel issues.  A tile (32 rows of any width: a multiple
// of 64 bytes for two-byte elements, of 32 for one-byte ones, 16-byte aligned) is fetched as n_ld
// wave-wide loads of 1 KB, lane l of load j taking bytes [1024 j + 16 l, + 16).  n_ld is fixed at
// compile time from the instantiation (KCH = ceil(d_k / 32) score steps; NT output tiles of 16
// channels: ceil(d_v / 16) for bf16 caches, blocks of 64 channels, i.e. 4 or 8 tiles, for one-byte
// codes) and can exceed the number of loads the tile needs by one whole load (bf16 K tiles: 2 KCH
// against ceil(d_k / 16); one-byte V tiles: NT / 2 against ceil(d_v / 32)).  The last n_trim loads
// are therefore trimmed to the tile by lane, all earlier ones are issued whole.  In a partial tile
// (the last rows of a sequence) every load is trimmed to the bytes of the rows that exist.
// ---- 4-bit caches: microscaling FP4 (E2M1 elements, one E8M0 scale byte per block of 32) --------
// E2M1 code (S.EE.M; magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6) nearest to y, ties to the code with
// mantissa bit 0, magnitudes above 6 saturate.  The thresholds are the midpoints between
// neighbouring magnitudes, each closed on the side of its even neighbour.
__host__ __device__ __forceinline__ uint32_t f64_to_e2m1(double y) {
  const double a = y < 0 ? -y : y;
  const uint32_t c = a <= 0.25 ? 0u : a < 0.75 ? 1u : a <= 1.25 ? 2u : a < 1.75 ? 3u : a <= 2.5 ? 4u : a < 3.5 ? 5u : a <= 5.0 ? 6u : 7u;
  return c | ((__builtin_bit_cast(uint64_t, y) >> 63) != 0 ? 8u : 0u);
}

// Scale exponent of a block whose largest magnitude is amax (finite, not subnormal as a double):
// floor(log2 amax) - 2, so that amax / 2^e lies in [4, 8), the top binade of E2M1; limited to
// [-126, 127]; 0 for a block of zeros.  The scale byte is e + 127.
__host__ __device__ __forceinline__ int mx_shared_exponent(double amax) {
  if (!(amax > 0.0)) return 0;
  const int e = static_cast<int>((__builtin_bit_cast(uint64_t, amax) >> 52) & 0x7ff) - 1023 - 2;
  return e < -126 ? -126 : (e > 127 ? 127 : e);
}

// 2^(-e) for e in [-126, 127], exact
__host__ __device__ __forceinline__ double pow2_neg(int e) {
  return __builtin_bit_cast(double, static_cast<uint64_t>(1023 - e) << 52);
}

constexpr int mx_blocks(int d) { return (d + 31) / 32; }
// A widened 4-bit tile in LDS: 32 rows of nb blocks of 32 bf16 (64 bytes).  The layout is chosen so
// that, with LDS serving 128 bytes per clock, neither the 16-byte stores that fill the tile (lane c
// holds block c % nb of row c / nb) nor the 16-byte K fragment reads (16 rows, one column) nor the
// 4-byte V reads fall on the same banks: rows 16 bytes past a multiple of 32 and blocks 64 bytes
// apart for one, two and four blocks (with four, the upper two blocks of a row also store their
// four 16-byte pieces in the order 2, 3, 0, 1: blocks 0 and 2 of a row are 128 bytes apart); three
// blocks lie 80 bytes apart in rows of 240 bytes.  (One extra 16 bytes per row was measured against
// none, 32 and 48 at the time the blocks were all 64 bytes apart: cfg3 shape 298 us against 733,
// 326 and 298 us.)
constexpr int mx4_block_stride(int nb) { return nb == 3 ? 80 : 64; }
constexpr int mx4_row_pitch(int nb) { return nb == 3 ? 240 : 64 * nb + 16; }
constexpr bool mx4_rotate_upper_blocks(int nb) { return nb == 4; }

constexpr int decode_v_tiles(int d_v, bool q8) { return q8 ? 4 * ((d_v + 63) / 64) : (d_v + 15) / 16; }
constexpr int k_tile_loads(int kch, bool q8) { return q8 ? kch : 2 * kch; }
constexpr int v_tile_loads(int nt, bool q8) { return q8 ? (nt + 1) / 2 : nt; }
constexpr int k_tile_trimmed(bool q8) { return q8 ? 1 : 2; }
constexpr int v_tile_trimmed(bool q8) { return q8 ? 2 : 1; }
__host__ __device__ __forceinline__ bool tile_load_issued(int j, int lane, int n_ld, int n_trim, int bytes, bool whole_tile) {
  if (whole_tile && j < n_ld - n_trim) return true;
  return 1024 * j + 16 * lane < bytes;
}

}  // namespace rap
#endif  // RAP_ARITH_H_

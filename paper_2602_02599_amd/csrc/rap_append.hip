// rap_rope_append: index-aware RoPE of new compact K rows + write of K and V rows into the cache.
//
// Eq. (rope): pair (a, b) = (k[c], k[c + P]) is rotated by the block [[cos, -sin], [sin, cos]] with
// angle t * theta^(-2 j / D), where j = keep_pair_idx[h][c] is the ORIGINAL pair index of compact
// pair c (the index-aware rotation of Sec. "RAP").  The angle, its sine/cosine and the rotation are
// taken in fp64 so that positions up to 2^17 and beyond stay far inside one bf16 ulp; the result is
// rounded to bf16 once.
//
// Work layout: one wavefront per (token, kv head); lane c handles pairs c and c + 64, then the
// same lanes copy the V row.  A K row is 4P bytes and a V row 2 d_v bytes, so the traffic of this
// call is a few KB per token: it is latency bound and never near a roofline.
#include "rap_device.h"

namespace rap {

__global__ __launch_bounds__(256) void append_kernel(AppendArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int h = blockIdx.y;
  const long long tok = static_cast<long long>(blockIdx.x) * 4 + wave;   // b * n_new + n
  const long long n_tok = static_cast<long long>(a.batch) * a.n_new;
  if (tok >= n_tok) return;
  const int b = static_cast<int>(tok / a.n_new);
  const int t = a.pos[tok];
  if (t < 0 || t >= a.cap) return;                                        // documented: skipped

  const int P = a.n_pairs;
  const uint16_t* ksrc = a.k_new + (tok * a.n_kv + h) * (2 * P);
  uint16_t* kdst = a.k_cache + ((static_cast<long long>(b) * a.n_kv + h) * a.cap + t) * (2 * P);
  for (int c = lane; c < P; c += kWave) {
    const int j = a.keep[h * P + c];
    if (j < 0 || j >= a.d_head / 2) continue;                             // documented: skipped
    const double inv_freq = pow(a.theta, -2.0 * static_cast<double>(j) / static_cast<double>(a.d_head));
    const double phi = static_cast<double>(t) * inv_freq;
    double sn, cs;
    sincos(phi, &sn, &cs);
    const double x = static_cast<double>(bf16_to_f32(ksrc[c]));
    const double y = static_cast<double>(bf16_to_f32(ksrc[c + P]));
    kdst[c] = f64_to_bf16_rne(x * cs - y * sn);
    kdst[c + P] = f64_to_bf16_rne(x * sn + y * cs);
  }
  const uint16_t* vsrc = a.v_new + (tok * a.n_kv + h) * a.d_v;
  uint16_t* vdst = a.v_cache + ((static_cast<long long>(b) * a.n_kv + h) * a.cap + t) * a.d_v;
  for (int c = lane; c < a.d_v; c += kWave) vdst[c] = vsrc[c];
}

hipError_t launch_append(const AppendArgs& a, hipStream_t stream) {
  const long long n_tok = static_cast<long long>(a.batch) * a.n_new;
  dim3 grid(static_cast<unsigned>((n_tok + 3) / 4), static_cast<unsigned>(a.n_kv), 1);
  hipLaunchKernelGGL(append_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rap

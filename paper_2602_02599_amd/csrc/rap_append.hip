// rap_rope_append: index-aware RoPE of new compact K rows + write of K and V rows into the cache.
//
// Eq. (rope): pair (a, b) = (k[c], k[c + P]) is rotated by the block [[cos, -sin], [sin, cos]] with
// angle t * theta^(-2 j / D), where j = keep_pair_idx[h][c] is the ORIGINAL pair index of compact
// pair c (the index-aware rotation of Sec. "RAP").  The angle, its sine/cosine and the rotation are
// taken in fp64 so that positions up to 2^17 and beyond stay far inside one bf16 ulp; the result is
// rounded to bf16 once.
//
// Work layout: one wavefront per (token, kv head); lane c handles pair c and V elements c and
// c + 64.  A K row is 4P bytes and a V row 2 d_v bytes, so the traffic of this call is a few KB per
// token: it is latency bound (one round trip for all loads, then the fp64 math, then the stores)
// and never near a roofline.
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
  const int P = a.n_pairs;

  // Everything this lane will need is requested at once (one memory round trip): the position,
  // its pair's original index and two elements, and its two V elements.  P <= 64 and d_v <= 128,
  // so one pair and two V elements per lane cover the row.
  const bool has_pair = lane < P;
  const bool has_v0 = lane < a.d_v, has_v1 = lane + kWave < a.d_v;
  const uint16_t* ksrc = a.k_new + (tok * a.n_kv + h) * (2 * P);
  const uint16_t* vsrc = a.v_new + (tok * a.n_kv + h) * a.d_v;
  const int t = a.pos[tok];
  const int j = has_pair ? a.keep[h * P + lane] : 0;
  const uint16_t kx = has_pair ? ksrc[lane] : 0, ky = has_pair ? ksrc[lane + P] : 0;
  const uint16_t v0 = has_v0 ? vsrc[lane] : 0, v1 = has_v1 ? vsrc[lane + kWave] : 0;
  if (t < 0 || t >= a.cap) return;                                        // documented: skipped

  const long long row = (static_cast<long long>(b) * a.n_kv + h) * a.cap + t;
  if (has_pair && j >= 0 && j < a.d_head / 2) {                           // bad index: documented skip
    // theta^(-2j/D) = 2^(j * (-2 log2(theta) / D)); the factor is taken in fp64 on the host
    const double phi = static_cast<double>(t) * exp2(static_cast<double>(j) * a.neg2_log2_theta_over_d);
    double sn, cs;
    sincos(phi, &sn, &cs);
    const double x = static_cast<double>(bf16_to_f32(kx));
    const double y = static_cast<double>(bf16_to_f32(ky));
    uint16_t* kdst = a.k_cache + row * (2 * P);
    kdst[lane] = f64_to_bf16_rne(x * cs - y * sn);
    kdst[lane + P] = f64_to_bf16_rne(x * sn + y * cs);
  }
  uint16_t* vdst = a.v_cache + row * a.d_v;
  if (has_v0) vdst[lane] = v0;
  if (has_v1) vdst[lane + kWave] = v1;
}

hipError_t launch_append(const AppendArgs& a, hipStream_t stream) {
  const long long n_tok = static_cast<long long>(a.batch) * a.n_new;
  dim3 grid(static_cast<unsigned>((n_tok + 3) / 4), static_cast<unsigned>(a.n_kv), 1);
  hipLaunchKernelGGL(append_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rap

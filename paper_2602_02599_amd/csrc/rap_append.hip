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
  double f = 0.0;
  const bool rot = has_pair && pair_frequency(a.keep, a.pair_freq, a.neg2_log2_theta_over_d, a.d_head, h * P + lane, &f);
  const uint16_t kx = has_pair ? ksrc[lane] : 0, ky = has_pair ? ksrc[lane + P] : 0;
  const uint16_t v0 = has_v0 ? vsrc[lane] : 0, v1 = has_v1 ? vsrc[lane + kWave] : 0;
  if (t < 0 || t >= a.cap) return;                                        // documented: skipped

  const long long row = cache_row(a, b, h, t);
  if (rot) {                                                              // bad index: documented skip
    const double phi = static_cast<double>(t) * f;
    double sn, cs;
    sincos_f64(phi, &sn, &cs);
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

// The same append into an fp8 cache: the rotated K value and the V value are divided by the scale
// of their KV head (fp64) and rounded once to an E4M3 code.  One wavefront per (token, KV head) for
// any n_new.
__global__ __launch_bounds__(256) void append_q8_kernel(AppendArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int h = blockIdx.y;
  const long long tok = static_cast<long long>(blockIdx.x) * 4 + wave;   // b * n_new + n
  const long long n_tok = static_cast<long long>(a.batch) * a.n_new;
  if (tok >= n_tok) return;
  const int b = static_cast<int>(tok / a.n_new);
  const int P = a.n_pairs;
  const bool has_pair = lane < P;
  const bool has_v0 = lane < a.d_v, has_v1 = lane + kWave < a.d_v;
  const uint16_t* ksrc = a.k_new + (tok * a.n_kv + h) * (2 * P);
  const uint16_t* vsrc = a.v_new + (tok * a.n_kv + h) * a.d_v;
  const int t = a.pos[tok];
  double f = 0.0;
  const bool rot = has_pair && pair_frequency(a.keep, a.pair_freq, a.neg2_log2_theta_over_d, a.d_head, h * P + lane, &f);
  const uint16_t kx = has_pair ? ksrc[lane] : 0, ky = has_pair ? ksrc[lane + P] : 0;
  const uint16_t v0 = has_v0 ? vsrc[lane] : 0, v1 = has_v1 ? vsrc[lane + kWave] : 0;
  const double ks = static_cast<double>(a.k_scale[h]), vs = static_cast<double>(a.v_scale[h]);
  if (t < 0 || t >= a.cap) return;                                        // documented: skipped
  const long long row = cache_row(a, b, h, t);                            // dense or paged
  uint8_t* k8 = reinterpret_cast<uint8_t*>(a.k_cache) + row * (2 * P);
  uint8_t* v8 = reinterpret_cast<uint8_t*>(a.v_cache) + row * a.d_v;
  if (rot) {
    double sn, cs;
    sincos_f64(static_cast<double>(t) * f, &sn, &cs);
    const double x = static_cast<double>(bf16_to_f32(kx));
    const double y = static_cast<double>(bf16_to_f32(ky));
    k8[lane] = f64_to_e4m3((x * cs - y * sn) / ks);
    k8[lane + P] = f64_to_e4m3((x * sn + y * cs) / ks);
  }
  if (has_v0) v8[lane] = f64_to_e4m3(static_cast<double>(bf16_to_f32(v0)) / vs);
  if (has_v1) v8[lane + kWave] = f64_to_e4m3(static_cast<double>(bf16_to_f32(v1)) / vs);
}

// The same append into a 4-bit cache (microscaling FP4).  A row is quantised block by block: the
// 32 elements of a block share the scale their largest magnitude asks for (mx_shared_exponent),
// every element is divided by it (a power of two: exact) and rounded once, from fp64, to the
// nearest E2M1 code.  One wavefront per (token, KV head): lane c rotates pair c as above, the
// rotated row (then the V row) is laid out in LDS, and lane e handles elements e and e + 64 of the
// row, its block being the 32 lanes around it.  A pair whose index is out of range counts as zero
// (the row is written as a whole).  Dense caches only.
__global__ __launch_bounds__(256) void append_mx4_kernel(AppendArgs a) {
  __shared__ double s_val[4][2 * kWave];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int h = blockIdx.y;
  const long long tok = static_cast<long long>(blockIdx.x) * 4 + wave;   // b * n_new + n
  const long long n_tok = static_cast<long long>(a.batch) * a.n_new;
  if (tok >= n_tok) return;
  const int b = static_cast<int>(tok / a.n_new);
  const int P = a.n_pairs;
  const bool has_pair = lane < P;
  const bool has_v0 = lane < a.d_v, has_v1 = lane + kWave < a.d_v;
  const uint16_t* ksrc = a.k_new + (tok * a.n_kv + h) * (2 * P);
  const uint16_t* vsrc = a.v_new + (tok * a.n_kv + h) * a.d_v;
  const int t = a.pos[tok];
  double f = 0.0;
  const bool rot = has_pair && pair_frequency(a.keep, a.pair_freq, a.neg2_log2_theta_over_d, a.d_head, h * P + lane, &f);
  const uint16_t kx = has_pair ? ksrc[lane] : 0, ky = has_pair ? ksrc[lane + P] : 0;
  const uint16_t v0 = has_v0 ? vsrc[lane] : 0, v1 = has_v1 ? vsrc[lane + kWave] : 0;
  if (t < 0 || t >= a.cap) return;                                        // documented: skipped (the whole wavefront)
  const long long row = (static_cast<long long>(b) * a.n_kv + h) * a.cap + t;
  double* val = s_val[wave];

  // one row in LDS -> code blocks and scale bytes of that row
  auto quantise_row = [&](int n_blk, uint8_t* codes, uint8_t* scales) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int e = lane + kWave * half, blk = e >> 5;
      const double v = val[e];
      double amax = v < 0 ? -v : v;
#pragma unroll
      for (int o = 16; o >= 1; o >>= 1) {
        const double other = __shfl_xor(amax, o);
        amax = other > amax ? other : amax;
      }
      const int se = mx_shared_exponent(amax);
      const uint32_t code = f64_to_e2m1(v * pow2_neg(se));
      const uint32_t next = __shfl_down(code, 1);
      if (blk < n_blk && (lane & 1) == 0) codes[16 * blk + ((e & 31) >> 1)] = static_cast<uint8_t>(code | (next << 4));
      if ((lane & 31) == 0) scales[blk] = static_cast<uint8_t>(blk < n_blk ? se + 127 : 127);
    }
  };
  auto wave_sync = [] {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };

  val[lane] = 0.0;
  val[lane + kWave] = 0.0;
  wave_sync();
  if (rot) {
    double sn, cs;
    sincos_f64(static_cast<double>(t) * f, &sn, &cs);
    const double x = static_cast<double>(bf16_to_f32(kx));
    const double y = static_cast<double>(bf16_to_f32(ky));
    val[lane] = x * cs - y * sn;
    val[lane + P] = x * sn + y * cs;
  }
  wave_sync();
  const int nbk = mx_blocks(2 * P), nbv = mx_blocks(a.d_v);
  quantise_row(nbk, reinterpret_cast<uint8_t*>(a.k_cache) + row * 16 * nbk, a.k_scales4 + row * 4);
  wave_sync();
  val[lane] = has_v0 ? static_cast<double>(bf16_to_f32(v0)) : 0.0;
  val[lane + kWave] = has_v1 ? static_cast<double>(bf16_to_f32(v1)) : 0.0;
  wave_sync();
  quantise_row(nbv, reinterpret_cast<uint8_t*>(a.v_cache) + row * 16 * nbv, a.v_scales4 + row * 4);
}

// Many tokens per sequence (prefill-sized appends).  The per-token kernel above spends its time in
// fp64 exp2 and sincos (about 0.6 ms for 131072 tokens x 8 heads, four times the HBM time of the
// same rows) and in one memory round trip per token.  Here a wavefront takes runs_per_wave runs of
// kBulkRun consecutive tokens of one (sequence, KV head):
//   * all loads of a run are requested before anything is computed (one round trip per run);
//   * memory moves as 32-bit words: lane i loads and stores word i of the K row (compact elements
//     2i and 2i+1), while the arithmetic is per pair: lane c rotates pair c, whose two elements
//     (c and c + P) it picks out of other lanes' words with cross-lane reads, and the rotated
//     pairs travel back to the lanes that store them the same way;
//   * theta_j and (cos theta_j, sin theta_j) are taken once per lane, the first angle exactly,
//     and while positions go up by one the angle advances by one exact complex rotation in fp64
//     (error ~1e-16 per step, over at most runs_per_wave * kBulkRun steps).
// A run whose positions are not t0, t0+1, ... inside [0, cap) takes the general loop below it
// (exact sincos per token, rows outside the cache skipped), which is the per-token arithmetic.
constexpr int kBulkRun = 16;

__device__ __forceinline__ uint32_t lane_read(int byte_addr, uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(byte_addr, static_cast<int>(v)));
}

// QUERY: the same walk over query rows (rap_rope_queries): no V, no cache; row (b, n, head) of
// the input is rotated at pos[b][n] with the kept pairs of KV head head / G and stored at the same
// place of the output; a pair with a bad index is stored as zero.
// Q8: the caches hold E4M3 codes (rap_rope_append_q8): every rotated element and every V element is
// divided by its head's scale in fp64 and rounded once to the nearest code; a lane stores the two
// code bytes of its own pair, so nothing travels back between lanes.
template <bool VDWORD, bool QUERY, bool Q8>
__global__ __launch_bounds__(256) void append_bulk_kernel(AppendArgs a, int runs_per_wave) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = blockIdx.y;
  const int b = blockIdx.z;
  const int P = a.n_pairs;
  const int32_t* pos = a.pos + static_cast<long long>(b) * a.n_new;
  const long long kstride = static_cast<long long>(a.n_kv) * 2 * P;      // elements between tokens
  const long long vstride = static_cast<long long>(a.n_kv) * a.d_v;

  // arithmetic role: lane c < P rotates pair c
  const bool has_pair = lane < P;
  double f = 0.0;                                               // bad index: pair is skipped
  const bool rot = has_pair && pair_frequency(a.keep, a.pair_freq, a.neg2_log2_theta_over_d, a.d_head,
                                              (QUERY ? h / a.group : h) * P + lane, &f);
  double sf, cf;
  sincos_f64(f, &sf, &cf);                                           // one step of the position
  const int x_lane = has_pair ? (lane >> 1) << 2 : 0, x_half = lane & 1;
  const int y_lane = has_pair ? ((lane + P) >> 1) << 2 : 0, y_half = (lane + P) & 1;
  // memory role: lane i < P moves word i = elements 2i (pair c0) and 2i+1 (pair c1)
  const bool has_k = lane < P;
  const int e0 = 2 * lane, e1 = 2 * lane + 1;
  const bool x0 = e0 < P, x1 = e1 < P;                          // element is the x half of its pair
  const int c0 = has_k ? (x0 ? e0 : e0 - P) << 2 : 0, c1 = has_k ? (x1 ? e1 : e1 - P) << 2 : 0;
  const bool ok0 = has_k && lane_read(c0, rot) != 0, ok1 = has_k && lane_read(c1, rot) != 0;
  const bool has_v0 = !QUERY && (VDWORD ? 2 * lane < a.d_v : lane < a.d_v);
  const bool has_v1 = !QUERY && !VDWORD && lane + kWave < a.d_v;
  const int kl = has_k ? lane : 0;
  const int vl0 = has_v0 ? lane : 0, vl1 = has_v1 ? lane + kWave : 0;

  double ks8 = 1.0, vs8 = 1.0;
  if constexpr (Q8) {
    ks8 = static_cast<double>(a.k_scale[h]);
    vs8 = static_cast<double>(a.v_scale[h]);
  }
  uint8_t* const k8 = reinterpret_cast<uint8_t*>(a.k_cache);
  uint8_t* const v8 = reinterpret_cast<uint8_t*>(a.v_cache);

  double cs = 1.0, sn = 0.0;
  bool anchored = false;                                         // (cs, sn) is the angle of position t_next
  int t_next = 0;
#pragma unroll 1
  for (int r = 0; r < runs_per_wave; ++r) {
    const int n0 = ((blockIdx.x * 4 + wave) * runs_per_wave + r) * kBulkRun;
    if (n0 >= a.n_new) break;
    const int cnt = min(kBulkRun, a.n_new - n0);
    const long long tok0 = static_cast<long long>(b) * a.n_new + n0;
    const uint16_t* ksrc0 = a.k_new + (tok0 * a.n_kv + h) * (2 * P);
    const uint16_t* vsrc0 = QUERY ? nullptr : a.v_new + (tok0 * a.n_kv + h) * a.d_v;
    const int tv = lane < cnt ? pos[n0 + lane] : 0;
    const int t0 = __builtin_amdgcn_readfirstlane(tv);
    // (a last, shorter run takes the general loop: at most kBulkRun - 1 tokens per sequence and head)
    // (with paged caches a run must also stay inside one page)
    const bool in_order = cnt == kBulkRun && __all(lane >= kBulkRun || tv == t0 + lane) &&
                          (QUERY || (t0 >= 0 && static_cast<long long>(t0) + kBulkRun <= a.cap &&
                                     (a.block_table == nullptr ||
                                      (t0 & ((1 << a.page_shift) - 1)) + kBulkRun <= (1 << a.page_shift))));

    if (in_order) {
      // Loads are unconditional (straight-line code, all in flight together): lanes with nothing
      // to fetch re-read an element that exists and never store what they got.
      uint32_t kw[kBulkRun], vw[kBulkRun];
#pragma unroll
      for (int i = 0; i < kBulkRun; ++i) {
        kw[i] = reinterpret_cast<const uint32_t*>(ksrc0 + i * kstride)[kl];
        if (QUERY) {
          vw[i] = 0;
        } else if (VDWORD) {
          vw[i] = reinterpret_cast<const uint32_t*>(vsrc0 + i * vstride)[vl0];
        } else {
          vw[i] = static_cast<uint32_t>((vsrc0 + i * vstride)[vl0]) |
                  static_cast<uint32_t>((vsrc0 + i * vstride)[vl1]) << 16;
        }
      }
      if (!(anchored && t0 == t_next)) sincos_f64(static_cast<double>(t0) * f, &sn, &cs);   // exact
      const long long row0 = QUERY ? 0 : cache_row(a, b, h, t0);
      uint16_t* kdst0 = QUERY ? a.k_cache + (tok0 * a.n_kv + h) * (2 * P) : a.k_cache + row0 * (2 * P);
      const long long kdstride = QUERY ? kstride : 2 * P;          // consecutive cache rows, or the input's layout
      uint16_t* vdst0 = QUERY ? nullptr : a.v_cache + row0 * a.d_v;
#pragma unroll
      for (int i = 0; i < kBulkRun; ++i) {
        {
          const uint32_t xw = lane_read(x_lane, kw[i]), yw = lane_read(y_lane, kw[i]);
          const double x = static_cast<double>(bf16_to_f32(static_cast<uint16_t>(x_half ? xw >> 16 : xw & 0xffffu)));
          const double y = static_cast<double>(bf16_to_f32(static_cast<uint16_t>(y_half ? yw >> 16 : yw & 0xffffu)));
          const double xr = x * cs - y * sn, yr = x * sn + y * cs;
          const double c2 = cs * cf - sn * sf;                   // angle advances by theta_j
          sn = sn * cf + cs * sf;
          cs = c2;
          if constexpr (Q8) {
            const long long row = row0 + i;                      // the run lies in one slab (or page)
            if (rot) {
              k8[row * (2 * P) + lane] = f64_to_e4m3(xr / ks8);
              k8[row * (2 * P) + lane + P] = f64_to_e4m3(yr / ks8);
            }
            const double v0 = static_cast<double>(bf16_to_f32(static_cast<uint16_t>(vw[i] & 0xffffu)));
            const double v1 = static_cast<double>(bf16_to_f32(static_cast<uint16_t>(vw[i] >> 16)));
            const uint8_t q0 = f64_to_e4m3(v0 / vs8), q1 = f64_to_e4m3(v1 / vs8);
            if (VDWORD) {
              if (has_v0) reinterpret_cast<uint16_t*>(v8 + row * a.d_v)[lane] = static_cast<uint16_t>(q0 | (q1 << 8));
            } else {
              if (has_v0) v8[row * a.d_v + lane] = q0;
              if (has_v1) v8[row * a.d_v + lane + kWave] = q1;
            }
            continue;
          }
          const uint32_t o = static_cast<uint32_t>(f64_to_bf16_rne(xr)) | static_cast<uint32_t>(f64_to_bf16_rne(yr)) << 16;
          const uint32_t p0 = lane_read(c0, o), p1 = lane_read(c1, o);
          const uint32_t o0 = x0 ? p0 & 0xffffu : p0 >> 16, o1 = x1 ? p1 & 0xffffu : p1 >> 16;
          uint16_t* kdst = kdst0 + i * kdstride;
          if (QUERY) {
            if (has_k) reinterpret_cast<uint32_t*>(kdst)[lane] = (ok0 ? o0 : 0u) | ((ok1 ? o1 : 0u) << 16);
          } else if (ok0 && ok1) {
            reinterpret_cast<uint32_t*>(kdst)[lane] = o0 | (o1 << 16);
          } else {
            if (ok0) kdst[e0] = static_cast<uint16_t>(o0);
            if (ok1) kdst[e1] = static_cast<uint16_t>(o1);
          }
          uint16_t* vdst = vdst0 + static_cast<long long>(i) * a.d_v;
          if (QUERY) {
          } else if (VDWORD) {
            if (has_v0) reinterpret_cast<uint32_t*>(vdst)[lane] = vw[i];
          } else {
            if (has_v0) vdst[lane] = static_cast<uint16_t>(vw[i]);
            if (has_v1) vdst[lane + kWave] = static_cast<uint16_t>(vw[i] >> 16);
          }
        }
      }
      anchored = true;
      t_next = t0 + kBulkRun;
      continue;
    }

    // general positions: lane c on pair c, one token at a time
    anchored = false;
    for (int i = 0; i < cnt; ++i) {
      const int t = pos[n0 + i];
      const uint16_t* ksrc = ksrc0 + i * kstride;
      if (QUERY) {
        uint16_t r0 = 0, r1 = 0;
        if (rot) {
          double s1, c1d;
          sincos_f64(static_cast<double>(t) * f, &s1, &c1d);
          const double x = static_cast<double>(bf16_to_f32(ksrc[lane]));
          const double y = static_cast<double>(bf16_to_f32(ksrc[lane + P]));
          r0 = f64_to_bf16_rne(x * c1d - y * s1);
          r1 = f64_to_bf16_rne(x * s1 + y * c1d);
        }
        if (has_pair) {
          uint16_t* qdst = a.k_cache + ((tok0 + i) * a.n_kv + h) * (2 * P);
          qdst[lane] = r0;
          qdst[lane + P] = r1;
        }
        continue;
      }
      if (t < 0 || t >= a.cap) continue;                         // documented: skipped
      const uint16_t* vsrc = vsrc0 + i * vstride;
      const long long row = cache_row(a, b, h, t);
      if constexpr (Q8) {
        if (rot) {
          double s1, c1d;
          sincos_f64(static_cast<double>(t) * f, &s1, &c1d);
          const double x = static_cast<double>(bf16_to_f32(ksrc[lane]));
          const double y = static_cast<double>(bf16_to_f32(ksrc[lane + P]));
          k8[row * (2 * P) + lane] = f64_to_e4m3((x * c1d - y * s1) / ks8);
          k8[row * (2 * P) + lane + P] = f64_to_e4m3((x * s1 + y * c1d) / ks8);
        }
        if (lane < a.d_v) v8[row * a.d_v + lane] = f64_to_e4m3(static_cast<double>(bf16_to_f32(vsrc[lane])) / vs8);
        if (lane + kWave < a.d_v)
          v8[row * a.d_v + lane + kWave] = f64_to_e4m3(static_cast<double>(bf16_to_f32(vsrc[lane + kWave])) / vs8);
        continue;
      }
      if (rot) {
        double s1, c1d;
        sincos_f64(static_cast<double>(t) * f, &s1, &c1d);
        const double x = static_cast<double>(bf16_to_f32(ksrc[lane]));
        const double y = static_cast<double>(bf16_to_f32(ksrc[lane + P]));
        uint16_t* kdst = a.k_cache + row * (2 * P);
        kdst[lane] = f64_to_bf16_rne(x * c1d - y * s1);
        kdst[lane + P] = f64_to_bf16_rne(x * s1 + y * c1d);
      }
      uint16_t* vdst = a.v_cache + row * a.d_v;
      if (lane < a.d_v) vdst[lane] = vsrc[lane];
      if (lane + kWave < a.d_v) vdst[lane + kWave] = vsrc[lane + kWave];
    }
  }
}

hipError_t launch_append(const AppendArgs& a, hipStream_t stream) {
  if (a.k_scales4 != nullptr) {
    const long long n_tok4 = static_cast<long long>(a.batch) * a.n_new;
    dim3 grid4(static_cast<unsigned>((n_tok4 + 3) / 4), static_cast<unsigned>(a.n_kv), 1);
    hipLaunchKernelGGL(append_mx4_kernel, grid4, dim3(256), 0, stream, a);
    return hipGetLastError();
  }
  if (a.k_scale != nullptr && a.n_new >= kBulkRun) {
    const long long runs = static_cast<long long>((a.n_new + kBulkRun - 1) / kBulkRun) * a.n_kv * a.batch;
    const int rpw = runs >= 32768 ? 4 : runs >= 16384 ? 2 : 1;
    const int per_wg = 4 * rpw * kBulkRun;
    dim3 grid(static_cast<unsigned>((a.n_new + per_wg - 1) / per_wg), static_cast<unsigned>(a.n_kv),
              static_cast<unsigned>(a.batch));
    if ((a.d_v & 1) == 0) hipLaunchKernelGGL((append_bulk_kernel<true, false, true>), grid, dim3(256), 0, stream, a, rpw);
    else hipLaunchKernelGGL((append_bulk_kernel<false, false, true>), grid, dim3(256), 0, stream, a, rpw);
    return hipGetLastError();
  }
  if (a.k_scale != nullptr) {
    const long long n_tok8 = static_cast<long long>(a.batch) * a.n_new;
    dim3 grid8(static_cast<unsigned>((n_tok8 + 3) / 4), static_cast<unsigned>(a.n_kv), 1);
    hipLaunchKernelGGL(append_q8_kernel, grid8, dim3(256), 0, stream, a);
    return hipGetLastError();
  }
  if (a.n_new >= kBulkRun) {
    // longer walks per wavefront share the per-lane set-up; short jobs keep one run per wavefront
    // so that the chip still gets enough wavefronts
    const long long runs = static_cast<long long>((a.n_new + kBulkRun - 1) / kBulkRun) * a.n_kv * a.batch;
    const int rpw = runs >= 32768 ? 4 : runs >= 16384 ? 2 : 1;
    const int per_wg = 4 * rpw * kBulkRun;
    dim3 grid(static_cast<unsigned>((a.n_new + per_wg - 1) / per_wg), static_cast<unsigned>(a.n_kv),
              static_cast<unsigned>(a.batch));
    if ((a.d_v & 1) == 0) hipLaunchKernelGGL((append_bulk_kernel<true, false, false>), grid, dim3(256), 0, stream, a, rpw);
    else hipLaunchKernelGGL((append_bulk_kernel<false, false, false>), grid, dim3(256), 0, stream, a, rpw);
    return hipGetLastError();
  }
  const long long n_tok = static_cast<long long>(a.batch) * a.n_new;
  dim3 grid(static_cast<unsigned>((n_tok + 3) / 4), static_cast<unsigned>(a.n_kv), 1);
  hipLaunchKernelGGL(append_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

// Query rows: k_new = input, k_cache = output (same layout), n_kv = number of query heads, group = G.
hipError_t launch_rope_queries(const AppendArgs& a, hipStream_t stream) {
  const long long runs = static_cast<long long>((a.n_new + kBulkRun - 1) / kBulkRun) * a.n_kv * a.batch;
  const int rpw = runs >= 32768 ? 4 : runs >= 16384 ? 2 : 1;
  const int per_wg = 4 * rpw * kBulkRun;
  dim3 grid(static_cast<unsigned>((a.n_new + per_wg - 1) / per_wg), static_cast<unsigned>(a.n_kv),
            static_cast<unsigned>(a.batch));
  hipLaunchKernelGGL((append_bulk_kernel<true, true, false>), grid, dim3(256), 0, stream, a, rpw);
  return hipGetLastError();
}

}  // namespace rap

// Matrix-core decode attention over the compact cache: the default kernel of rap_decode_attn
// (compiled by rap_decode_mfma.hip for bf16 caches and by rap_decode_mfma_q8.hip for one-byte codes,
// so that the two sets of instantiations build side by side).
//
// Eq. (attn) with the GQA remark, evaluated as online softmax over tiles of 32 cache rows.
// The path is bound by HBM: every K and V byte is needed exactly once per decode step, and the
// arithmetic (G flop per cache byte) is small.  The design therefore serves one goal, keeping many
// large, perfectly coalesced reads in flight per compute unit with as few instructions as possible
// around them:
//
//  * Each wavefront is autonomous.  It owns every fourth 32-row tile of its workgroup's row range,
//    streams the tile's K bytes and V bytes as two flat, 16-byte-aligned runs (row widths such as
//    180, 232 or 230 bytes are not multiples of 16, but 8 rows of any width are), holds the next
//    tile in registers while it works on the current one, and parks the current one in its private
//    slice of LDS.  There is no barrier in the main loop.
//  * Scores: S^T[row][g] = K_tile[row][:] . q[g][:] on v_mfma_f32_16x16x32_bf16 with the K tile as
//    the A operand (a lane reads 16 bytes of one row from LDS) and the G query rows, zero-padded to
//    16, resident in registers as the B operand.  bf16 products are exact in fp32.
//  * In the result layout of that instruction a lane (query head g, lane group lg) holds the scores
//    of eight rows of the tile.  P.V runs on the same instruction with the contraction slots
//    numbered so that a lane's eight slots are exactly those eight rows: the probabilities go from
//    the exponential into the A operand without leaving the lane, as a bf16 head plus a bf16
//    remainder (16 significant bits).  The V operand a lane needs (its channel, eight rows) is
//    gathered from LDS with 4-byte reads of two adjacent channels and a byte permute per row pair:
//    the "transpose" a row-major V needs costs LDS address bits and one ALU instruction per pair.
//  * The vector ALU only scales, exponentiates, sums and packs eight scores per lane per tile;
//    the accumulators are rescaled only when a score outgrows the reference by 2^64.
//
// Garbage safety: rows at or beyond the sequence length may hold any bits.  Their scores are
// replaced by -inf (a select, not arithmetic), their V reads are redirected to the last valid row
// of the tile, and the part of a K fragment beyond d_k is masked to zero, so nothing read outside
// the valid rows can reach a result.
#ifndef RAP_DECODE_KERNEL_H_
#define RAP_DECODE_KERNEL_H_

#include "rap_device.h"

namespace rap {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;


constexpr int kTileRows = 32;

// Rows of one-byte codes have any width, so a fragment in LDS starts at any byte.  Wide LDS reads
// at such addresses are served, but slowly (the 8- and 4-byte reads below, issued unaligned, made
// the kernel a third slower at 90- and 115-byte rows and nearly twice as fast at 64-byte rows);
// so the reads are issued dword-aligned, one dword more than needed, and the bytes are moved into
// place with v_alignbyte_b32, which shifts a 64-bit pair right by the low two bits of its third
// operand times eight: the byte address itself serves as that operand.
__device__ __forceinline__ uint32_t lds_u32_at(const unsigned char* base, int byte_off) {
  const uint32_t* p = reinterpret_cast<const uint32_t*>(base + (byte_off & ~3));
  return __builtin_amdgcn_alignbyte(p[1], p[0], static_cast<uint32_t>(byte_off));
}
__device__ __forceinline__ void lds_u64_at(const unsigned char* base, int byte_off, uint32_t* lo, uint32_t* hi) {
  const uint32_t* p = reinterpret_cast<const uint32_t*>(base + (byte_off & ~3));
  const uint32_t d0 = p[0], d1 = p[1], d2 = p[2];
  *lo = __builtin_amdgcn_alignbyte(d1, d0, static_cast<uint32_t>(byte_off));
  *hi = __builtin_amdgcn_alignbyte(d2, d1, static_cast<uint32_t>(byte_off));
}

// 16-byte load of cache bytes that are used once: the non-temporal form (global_load_dwordx4 ... nt)
// tells the caches not to keep the line.  Every K and V byte of a decode step is such a byte, and
// the hint alone takes a tenth off the kernel's time (cfg2 shape: 72.2 -> 64.5 us per call, cfg3
// shape 677 -> 616 us, same bits), presumably because the L2s and the memory-side cache no longer
// spend work on allocating and evicting lines nobody returns to.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
__device__ __forceinline__ uint4 ld_stream(const unsigned char* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ void wave_lds_sync() {
  // LDS operations of one wavefront execute in order; this only stops the compiler from moving
  // LDS accesses of different lanes across the hand-over point.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Headroom, in log2 units, by which a score may exceed the reference of its running softmax
// before the accumulators are rescaled: 2^64 * (rows of a range) * |v| stays far below fp32 max.
constexpr float kHeadroom = 64.f;

// One-call decode step: the new token, handled by one wavefront of a workgroup of its own per
// (b, h) (grid index n_split, next to the workgroups that scan the ranges), so that nobody who
// streams rows waits for it.  Lane c < P rotates pair c of the
// new K row exactly as the append kernel does (Eq. (rope) at the pair's original index, fp64, one
// rounding to bf16) and writes it into the cache, the lanes copy the V row, and the rotated row,
// still in registers, is scored against the G query rows (s_q: rotated query rows in LDS, or null
// when the query arrived rotated).  The token is left as (m = score, l = 1, acc = V row) in the
// slot behind the ranges, with m = -inf when row t is not among the attended ones.  All values
// are those a separate append followed by reading the cache would have produced.  The loads are
// a step of their own so that they can be requested together with the workgroup's other first loads.
struct TokenRegs {
  double f;
  bool rot;
  uint16_t kx, ky, v0, v1;
  uint16_t qx[kMaxGroup], qy[kMaxGroup];
};

__device__ __forceinline__ void token_load(const DecodeArgs& a, int b, int h, int lane, bool rope_q, TokenRegs& r) {
  const int P = a.n_pairs;
  const long long nrow = static_cast<long long>(b) * a.n_kv + h;
  const bool hp = lane < P;
  r.f = 0.0;
  r.rot = hp && pair_frequency(a.keep, a.pair_freq, a.neg2_log2_theta_over_d, a.d_head, h * P + lane, &r.f);
  r.kx = hp ? a.k_new[nrow * 2 * P + lane] : 0;
  r.ky = hp ? a.k_new[nrow * 2 * P + lane + P] : 0;
  r.v0 = lane < a.d_v ? a.v_new[nrow * a.d_v + lane] : 0;
  r.v1 = lane + kWave < a.d_v ? a.v_new[nrow * a.d_v + lane + kWave] : 0;
#pragma unroll
  for (int g = 0; g < kMaxGroup; ++g) {
    const bool have = !rope_q && hp && g < a.group;
    const uint16_t* qrow = a.q + (static_cast<long long>(b) * a.n_q + h * a.group + (g < a.group ? g : 0)) * 2 * P;
    r.qx[g] = have ? qrow[lane] : 0;
    r.qy[g] = have ? qrow[lane + P] : 0;
  }
}

__device__ __forceinline__ void token_finish(const DecodeArgs& a, int b, int h, int lane, int t, bool attended,
                                             const uint16_t* s_q, const TokenRegs& r) {
  const int P = a.n_pairs;
  const bool stored = t >= 0 && t < a.cap;
  const bool q8 = a.k_scale != nullptr;             // caches of E4M3 codes: value = code value x scale of the head
  // row of the cache (dense) or of the pool (paged) that holds position t
  long long row = (static_cast<long long>(b) * a.n_kv + h) * a.cap + t;
  if (a.block_table != nullptr && stored) {
    int pg = a.block_table[static_cast<long long>(b) * a.max_pages + (t >> a.page_shift)];
    pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);
    row = ((static_cast<long long>(pg) * a.n_kv + h) << a.page_shift) + (t & ((1 << a.page_shift) - 1));
  }
  uint8_t* k8 = reinterpret_cast<uint8_t*>(a.k_cache_w) + row * 2 * P;
  uint8_t* v8 = reinterpret_cast<uint8_t*>(a.v_cache_w) + row * a.d_v;
  // the new K pair and V elements as the scan would read them back from the cache (fp32, exact)
  float kxf = 0.f, kyf = 0.f, v0f = bf16_to_f32(r.v0), v1f = bf16_to_f32(r.v1);
  if (lane < P && stored) {
    if (r.rot) {
      const double phi = static_cast<double>(t) * r.f;
      double sn, cs;
      sincos_f64(phi, &sn, &cs);
      const double x = static_cast<double>(bf16_to_f32(r.kx)), y = static_cast<double>(bf16_to_f32(r.ky));
      if (q8) {
        const double ks = static_cast<double>(a.k_scale[h]);
        const uint8_t cx = f64_to_e4m3((x * cs - y * sn) / ks), cy = f64_to_e4m3((x * sn + y * cs) / ks);
        k8[lane] = cx;
        k8[lane + P] = cy;
        kxf = e4m3_to_f32(cx);
        kyf = e4m3_to_f32(cy);
      } else {
        const uint16_t kxr = f64_to_bf16_rne(x * cs - y * sn), kyr = f64_to_bf16_rne(x * sn + y * cs);
        a.k_cache_w[row * 2 * P + lane] = kxr;
        a.k_cache_w[row * 2 * P + lane + P] = kyr;
        kxf = bf16_to_f32(kxr);
        kyf = bf16_to_f32(kyr);
      }
    } else if (q8) {   // bad pair index: the append leaves these two elements as they are
      kxf = e4m3_to_f32(k8[lane]);
      kyf = e4m3_to_f32(k8[lane + P]);
    } else {
      kxf = bf16_to_f32(a.k_cache_w[row * 2 * P + lane]);
      kyf = bf16_to_f32(a.k_cache_w[row * 2 * P + lane + P]);
    }
  }
  if (q8) {
    const double vs = static_cast<double>(a.v_scale[h]);
    const uint8_t c0 = f64_to_e4m3(static_cast<double>(v0f) / vs), c1 = f64_to_e4m3(static_cast<double>(v1f) / vs);
    if (stored && lane < a.d_v) v8[lane] = c0;
    if (stored && lane + kWave < a.d_v) v8[lane + kWave] = c1;
    v0f = e4m3_to_f32(c0) * a.v_scale[h];
    v1f = e4m3_to_f32(c1) * a.v_scale[h];
  } else if (stored) {
    if (lane < a.d_v) a.v_cache_w[row * a.d_v + lane] = r.v0;
    if (lane + kWave < a.d_v) a.v_cache_w[row * a.d_v + lane + kWave] = r.v1;
  }
  const float score_scale = q8 ? a.scale_log2e * a.k_scale[h] : a.scale_log2e;
#pragma unroll
  for (int g = 0; g < kMaxGroup; ++g) {
    if (g < a.group) {
      uint16_t qx = r.qx[g], qy = r.qy[g];
      if (s_q != nullptr && lane < P) {
        qx = s_q[g * 2 * P + lane];
        qy = s_q[g * 2 * P + lane + P];
      }
      float part = lane < P ? fmaf(bf16_to_f32(qx), kxf, bf16_to_f32(qy) * kyf) : 0.f;
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o);
      const long long slot = (static_cast<long long>(b) * a.n_q + h * a.group + g) * a.n_slots + a.n_split;
      if (lane == 0) {
        a.part_ml[slot * 2 + 0] = attended ? part * score_scale : -INFINITY;
        a.part_ml[slot * 2 + 1] = attended ? 1.f : 0.f;
      }
      if (lane < a.d_v) a.part_acc[slot * a.d_v + lane] = attended ? v0f : 0.f;
      if (lane + kWave < a.d_v) a.part_acc[slot * a.d_v + lane + kWave] = attended ? v1f : 0.f;
    }
  }
}

constexpr int kMaxCols = 16;   // columns of the matrix instruction: query rows of one (b, h) with several tokens

// KCH = ceil(d_k / 32) score k-steps, NT = 16-channel output tiles.  VPAIR (even d_v): a lane
// reads two adjacent V channels with one 4-byte LDS read and tile nt holds channels
// 32 (nt / 2) + 2 l16 + (nt & 1); otherwise 2-byte reads and tile nt holds channels 16 nt + l16.
// PAGED: the caches are pools of pages [n_pages, H_kv, page_rows, d] and row r of sequence b lives
// in page block_table[b][r / page_rows]; page_rows is a power of two >= 32, so a 32-row tile never
// straddles two pages and only the start address of a tile changes.
// Q8: the caches hold one-byte E4M3 codes (value = code value x the scale of the KV head).  Rows
// are half as long, tiles take half the loads and half the LDS, and a fragment is widened to bf16
// (exactly: every E4M3 value is a bf16 number) on its way from LDS into the matrix instruction;
// the two scales fold into the softmax scale and into the partial sums.  LDS instructions, not
// bytes, are what this variant runs out of (counters: the LDS address unit 80 % busy with 1- and
// 2-byte reads), so it reads wide: a K fragment is three aligned dwords shifted into place, and a
// lane takes FOUR adjacent V channels of a row with two aligned dwords (NT is 4 or 8, tile nt
// holds channels 64 (nt / 4) + 4 l16 + (nt & 3)) and sorts the bytes of eight rows into the four
// operands with byte permutes.
// MX4: the caches hold 4-bit codes (microscaling FP4: E2M1 elements, one E8M0 scale byte per block
// of 32 elements; a row is KCH, respectively NT / 2, blocks of 16 code bytes, its scale bytes sit in
// a second array, four per row).  A tile of 32 rows is a flat run of 16-byte blocks: a lane
// fetches whole blocks with the scale byte of each, widens a block to 32 bf16 (exactly:
// v_cvt_scalef32_pk_bf16_fp4 multiplies the two codes of a byte by the scale it is given; compared
// on the device with the format's table for every byte value and scales from 2^-126 to 2^127) on
// the way into LDS, and from there on the tile is a bf16 tile of 32 KCH x 16 NT elements (rows and
// blocks placed so that neither the stores nor the fragment reads collide on LDS banks, see
// mx4_row_pitch): scores, softmax and P.V are the bf16 path's, instruction for instruction.
template <int KCH, int NT, bool VPAIR, bool PAGED, bool Q8, bool AL, bool MX4 = false>
__global__ __launch_bounds__(256, (KCH <= 3 ? 3 : 2)) void decode_mfma_kernel(DecodeArgs a) {
  // 1 KB wave-loads covering a K tile (d_k <= 32 KCH); MX4: 16-byte blocks of the tile per lane
  constexpr int NLD_K = MX4 ? (kTileRows * KCH + 63) / 64 : k_tile_loads(KCH, Q8);
  constexpr int NLD_V = MX4 ? (kTileRows * (NT / 2) + 63) / 64 : v_tile_loads(NT, Q8);   // same for a V tile (d_v <= 16 NT)
  static_assert(!MX4 || (VPAIR && !PAGED && !Q8 && !AL && NT % 2 == 0), "4-bit caches: dense, blocks of 32 channels");
  constexpr int TRIM_K = k_tile_trimmed(Q8), TRIM_V = v_tile_trimmed(Q8);   // trailing loads trimmed by lane
  constexpr int EB = Q8 ? 1 : 2;                   // bytes per cache element
  constexpr int VLANE = Q8 ? 4 : (VPAIR ? 4 : 2);  // bytes of a V row one lane slot stands for
  static_assert(!Q8 || (!VPAIR && (NT == 4 || NT == 8)), "one-byte caches: blocks of 64 channels");
  static_assert(Q8 || !AL, "AL (rows of one-byte codes that keep fragments aligned) belongs to Q8");
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction
  const int l16 = lane & 15;
  const int lg = lane >> 4;
  // One-dimensional grid.  Workgroup L < n_split * H_kv * B scans a row range: consecutive L share
  // a (b, h), and the range index is rotated by the (b, h) index so that range 0 of different
  // sequences falls on different XCDs (hardware places workgroup L on XCD L mod 8; with a ragged
  // batch the low ranges are the ones that hold rows, and n_split is often a multiple of 8).
  // The workgroups after those, one per (b, h), exist in the decode step only and take the new
  // token; coming last they do not disturb the placement of the scanning workgroups.
  const int n_scan = a.n_split * a.n_kv * a.batch;
  const int wg = blockIdx.x;
  const int slab_id = wg < n_scan ? wg / a.n_split : wg - n_scan;
  const int split = wg < n_scan ? (wg - slab_id * a.n_split + slab_id) % a.n_split : a.n_split;
  const int h = slab_id % a.n_kv;
  const int b = slab_id / a.n_kv;

  int len = a.seq_lens[b];
  len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
  // One-call decode step: the new token's row is not in the cache yet.  As the last row it simply
  // shortens the sequence; anywhere else inside it, the row is masked like the rows beyond the end.
  int t_skip = -1;
  __shared__ uint16_t s_q[kMaxGroup * 2 * kMaxPairs];
  const bool rope_q = a.q_pos != nullptr;
  bool tok_attended = false;
  if (a.new_pos != nullptr) {
    t_skip = a.new_pos[b];
    tok_attended = t_skip >= 0 && t_skip < len;
    if (len > 0 && t_skip == len - 1) len -= 1;
  }
  // several query tokens: the scan stops in front of their rows; the combining kernel adds the
  // causal part among the tokens themselves
  if (a.n_tok > 1) len = len > a.n_tok ? len - a.n_tok : 0;
  if (split == a.n_split) {                            // the workgroup of the new token (decode step only)
    TokenRegs tk;
    if (wave == 0) token_load(a, b, h, lane, rope_q, tk);
    if (rope_q) {
      rotate_queries_to_lds(a, b, h, tid, 256, s_q);
      __syncthreads();
    }
    if (wave == 0) token_finish(a, b, h, lane, t_skip, tok_attended, rope_q ? s_q : nullptr, tk);
    return;
  }
  const int r0 = split * a.rows_per_split;
  if (r0 >= len) {
    // no rows for this workgroup.  With a single range nobody else writes the output row of an
    // empty sequence; with several ranges the combining kernel does.
    if (a.direct_out)
      for (int e = tid; e < a.group * a.d_v; e += 256)
        a.out[(static_cast<long long>(b) * a.n_q + h * a.group) * a.d_v + e] = 0.f;
    return;
  }
  const int r1 = min(r0 + a.rows_per_split, len);
  // rows below len8 are readable: <= cache_cap (a multiple of 8, of 16 for one-byte elements, which
  // keeps every such group of rows 16-byte aligned whatever the row width)
  const int len8 = Q8 ? (len + 15) & ~15 : (len + 7) & ~7;

  const int G = a.group;
  const int cols = G * a.n_tok;                    // query rows of this (b, h): columns of the matrix instruction
  const int dk = a.d_k, dv = a.d_v;
  const int pitch_k = MX4 ? 16 * KCH : EB * dk, pitch_v = MX4 ? 8 * NT : EB * dv;   // bytes of a cache row
  const int lpk = MX4 ? mx4_row_pitch(KCH) : pitch_k, lpv = MX4 ? mx4_row_pitch(NT / 2) : pitch_v;   // bytes of a row in LDS
  constexpr int SK = MX4 ? mx4_block_stride(KCH) : 64, SV = MX4 ? mx4_block_stride(NT / 2) : 64;    // bytes from one 32-element block of a row to the next
  // LDS slice of this wavefront: K area and V area, each a whole number of 1 KB wave-stores
  unsigned char* kt = smem + wave * a.lds_wave_bytes;
  unsigned char* vt = kt + (MX4 ? kTileRows * lpk : 1024 * NLD_K);

  const long long slab = static_cast<long long>(b) * a.n_kv + h;
  const unsigned char* kslab = reinterpret_cast<const unsigned char*>(a.k_cache) + (PAGED ? 0 : slab * a.cap * pitch_k);
  const unsigned char* vslab = reinterpret_cast<const unsigned char*>(a.v_cache) + (PAGED ? 0 : slab * a.cap * pitch_v);
  // row of the pool (paged) or of the (b, h) slab (dense) where logical row `row` starts; a page
  // number outside the pool is clamped into it, so that a bad table cannot send a load astray
  auto tile_row = [&](int row) -> long long {
    if constexpr (PAGED) {
      int pg = a.block_table[static_cast<long long>(b) * a.max_pages + (row >> a.page_shift)];
      pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);
      return ((static_cast<long long>(pg) * a.n_kv + h) << a.page_shift) + (row & ((1 << a.page_shift) - 1));
    } else {
      return row;
    }
  };

  f32x4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY;
  float l_run = 0.f;

  uint4 kst[NLD_K], vst[NLD_V];
#pragma unroll
  for (int j = 0; j < NLD_K; ++j) kst[j] = make_uint4(0, 0, 0, 0);
#pragma unroll
  for (int j = 0; j < NLD_V; ++j) vst[j] = make_uint4(0, 0, 0, 0);
  // MX4: the scale byte that goes with each staged block, where the block lands in LDS, and the
  // slabs of the scale bytes.  Block c = lane + 64 j of a tile is block c % KCH of row c / KCH.
  uint32_t kss[MX4 ? NLD_K : 1], vss[MX4 ? NLD_V : 1];
  int k_lds[MX4 ? NLD_K : 1], v_lds[MX4 ? NLD_V : 1];
  bool k_rot[MX4 ? NLD_K : 1], v_rot[MX4 ? NLD_V : 1];     // this block stores its pieces in the order 2, 3, 0, 1
  const unsigned char* ksslab = nullptr;
  const unsigned char* vsslab = nullptr;
  if constexpr (MX4) {
    ksslab = a.k_scales4 + slab * a.cap * 4;
    vsslab = a.v_scales4 + slab * a.cap * 4;
#pragma unroll
    for (int j = 0; j < NLD_K; ++j) {
      const int c = lane + 64 * j, row = c / KCH;
      kss[j] = 127;
      k_lds[j] = row * lpk + (c - row * KCH) * SK;
      k_rot[j] = mx4_rotate_upper_blocks(KCH) && ((c - row * KCH) & 2) != 0;
    }
#pragma unroll
    for (int j = 0; j < NLD_V; ++j) {
      const int c = lane + 64 * j, row = c / (NT / 2);
      vss[j] = 127;
      v_lds[j] = row * lpv + (c - row * (NT / 2)) * SV;
      v_rot[j] = mx4_rotate_upper_blocks(NT / 2) && ((c - row * (NT / 2)) & 2) != 0;
    }
  }

  // A full tile is fetched with whole-KB loads except the last one or two of each run, which are
  // trimmed to the tile's own bytes (tile_load_issued): nothing is fetched twice, nothing beyond
  // the tile is touched.
  bool k_tail[TRIM_K], v_tail[TRIM_V];
#pragma unroll
  for (int u = 0; u < TRIM_K; ++u) k_tail[u] = tile_load_issued(NLD_K - TRIM_K + u, lane, NLD_K, TRIM_K, kTileRows * pitch_k, true);
#pragma unroll
  for (int u = 0; u < TRIM_V; ++u) v_tail[u] = tile_load_issued(NLD_V - TRIM_V + u, lane, NLD_V, TRIM_V, kTileRows * pitch_v, true);
  auto issue_loads = [&](int base, long long trow) {
    const unsigned char* kg = kslab + trow * pitch_k + 16 * lane;
    const unsigned char* vg = vslab + trow * pitch_v + 16 * lane;
    if constexpr (MX4) {
      // whole blocks of the rows below len8 (<= cache_cap), each with its scale byte: block c of the
      // tile is 16 c bytes into it, its scale byte 4 (c / KCH) + c % KCH bytes into the tile's scales
      const int rows = min(kTileRows, len8 - base);
#pragma unroll
      for (int j = 0; j < NLD_K; ++j) {
        const int c = lane + 64 * j, row = c / KCH;
        if (c < rows * KCH) {
          kst[j] = ld_stream(kg + 1024 * j);
          kss[j] = ksslab[(trow + row) * 4 + (c - row * KCH)];
        }
      }
#pragma unroll
      for (int j = 0; j < NLD_V; ++j) {
        const int c = lane + 64 * j, row = c / (NT / 2);
        if (c < rows * (NT / 2)) {
          vst[j] = ld_stream(vg + 1024 * j);
          vss[j] = vsslab[(trow + row) * 4 + (c - row * (NT / 2))];
        }
      }
      return;
    }
    if (base + kTileRows <= len8) {
      // common case, a full tile
#pragma unroll
      for (int j = 0; j < NLD_K; ++j)
        if (j < NLD_K - TRIM_K || k_tail[j < NLD_K - TRIM_K ? 0 : j - (NLD_K - TRIM_K)]) kst[j] = ld_stream(kg + 1024 * j);
#pragma unroll
      for (int j = 0; j < NLD_V; ++j)
        if (j < NLD_V - TRIM_V || v_tail[j < NLD_V - TRIM_V ? 0 : j - (NLD_V - TRIM_V)]) vst[j] = ld_stream(vg + 1024 * j);
    } else {
      // last tiles of a sequence: read only rows [base, len8), chunk by chunk
      const int rows = min(kTileRows, len8 - base);   // multiple of 8
      const int kval = rows * pitch_k, vval = rows * pitch_v;
#pragma unroll
      for (int j = 0; j < NLD_K; ++j)
        if (tile_load_issued(j, lane, NLD_K, TRIM_K, kval, false)) kst[j] = ld_stream(kg + 1024 * j);
#pragma unroll
      for (int j = 0; j < NLD_V; ++j)
        if (tile_load_issued(j, lane, NLD_V, TRIM_V, vval, false)) vst[j] = ld_stream(vg + 1024 * j);
    }
  };

  // first tile on its way before anything else is fetched
  const int first = r0 + kTileRows * wave;
  if (first < r1) issue_loads(first, tile_row(first));
  // paged: the page of the tile after next is looked up one iteration before its loads are issued
  long long trow1 = (PAGED && first + 4 * kTileRows < r1) ? tile_row(first + 4 * kTileRows) : 0;

  // ---- query rows as the B operand: lane (l16 = head slot, lg = k sub-chunk).  With q_pos the
  // rows arrive un-rotated: the workgroup rotates them into LDS first, while its first tile flies.
  if (rope_q) {
    rotate_queries_to_lds(a, b, h, tid, 256, s_q);
    __syncthreads();
  }
  bf16x8 qf[KCH];
  {
    // column c = token * G + head of the group (one token: c = head)
    // (wave-uniform base, 32-bit lane offset)
    const int qc = l16 < cols ? l16 : 0, qt = (qc * a.group_inv16) >> 16;   // qc / G, exact below 16
    const uint32_t* qbase = reinterpret_cast<const uint32_t*>(a.q) +
                            (static_cast<long long>(b) * a.n_tok * a.n_q + h * G) * a.n_pairs;
    const uint32_t* qrow = rope_q ? reinterpret_cast<const uint32_t*>(s_q) + qc * a.n_pairs
                                  : qbase + (qt * a.n_q + (qc - qt * G)) * a.n_pairs;
#pragma unroll
    for (int kk = 0; kk < KCH; ++kk) {
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = 32 * kk + 8 * lg + 2 * i;
        w[i] = (l16 < cols && e < dk) ? qrow[e >> 1] : 0u;
      }
      qf[kk] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
  }
  // mask of the last K fragment (elements at or beyond d_k belong to the next row)
  uint32_t kmask[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) kmask[i] = (32 * (KCH - 1) + 8 * lg + 2 * i) < dk ? 0xffffffffu : 0u;
  // one-byte elements: the same limit as byte masks of the fragment's two words (d_k is even)
  uint32_t kmask8[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int left = dk - (32 * (KCH - 1) + 8 * lg + 4 * i);      // elements of word i that exist
    kmask8[i] = left >= 4 ? 0xffffffffu : (left >= 2 ? 0x0000ffffu : 0u);
  }

  const float scale_log2e = Q8 ? a.scale_log2e * a.k_scale[h] : a.scale_log2e;
  // LDS byte offsets of this lane's operands inside a tile
  int koff[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) koff[rt] = (16 * rt + l16) * lpk + 8 * EB * lg;
  int vo_laid[8];   // V rows of the lane's eight contraction slots as laid out: j = 4 rt + r is row 16 rt + 4 lg + r
#pragma unroll
  for (int j = 0; j < 8; ++j) vo_laid[j] = (16 * (j >> 2) + 4 * lg + (j & 3)) * lpv + VLANE * l16;
  // MX4: a staged block of 32 codes becomes 32 bf16 (64 bytes) of its row in LDS
  // (rot: the block's 16-byte pieces are stored in the order 2, 3, 0, 1, each at its own place)
  auto park_mx4 = [&](unsigned char* area, int off, const uint4& blk, uint32_t scale_byte, bool rot, bool may_rot) {
    const float sc = bits_f32((scale_byte & 0xffu) << 23);       // 2^(e - 127), e >= 1
    const uint32_t w[4] = {blk.x, blk.y, blk.z, blk.w};
    const int off_lo = may_rot && rot ? off + 32 : off, off_hi = may_rot && rot ? off - 32 : off;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t src = may_rot && rot ? w[i ^ 2] : w[i];
      uint4 o;
      o.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(src, sc, 0));
      o.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(src, sc, 1));
      o.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(src, sc, 2));
      o.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(src, sc, 3));
      *reinterpret_cast<uint4*>(area + (i < 2 ? off_lo : off_hi) + 16 * i) = o;
    }
  };


  for (int base = first; base < r1; base += 4 * kTileRows) {
    // ---- park the staged tile in LDS, start fetching the next one
    wave_lds_sync();
    if constexpr (MX4) {
#pragma unroll
      for (int j = 0; j < NLD_K; ++j)
        if (lane + 64 * j < kTileRows * KCH) park_mx4(kt, k_lds[j], kst[j], kss[j], k_rot[j], mx4_rotate_upper_blocks(KCH));
#pragma unroll
      for (int j = 0; j < NLD_V; ++j)
        if (lane + 64 * j < kTileRows * (NT / 2)) park_mx4(vt, v_lds[j], vst[j], vss[j], v_rot[j], mx4_rotate_upper_blocks(NT / 2));
    } else {
#pragma unroll
      for (int j = 0; j < NLD_K; ++j) *reinterpret_cast<uint4*>(kt + 1024 * j + 16 * lane) = kst[j];
#pragma unroll
      for (int j = 0; j < NLD_V; ++j) *reinterpret_cast<uint4*>(vt + 1024 * j + 16 * lane) = vst[j];
    }
    wave_lds_sync();
    if (base + 4 * kTileRows < r1) issue_loads(base + 4 * kTileRows, PAGED ? trow1 : base + 4 * kTileRows);
    if (PAGED && base + 8 * kTileRows < r1) trow1 = tile_row(base + 8 * kTileRows);


    // ---- scores: sc[rt][r] = q[g = l16] . K[base + 16 rt + 4 lg + r]
    f32x4 sc[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      sc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KCH; ++kk) {
        uint4 w;
        if constexpr (Q8) {
          uint32_t c0, c1;
          if constexpr (AL) {
            const uint2 c = *reinterpret_cast<const uint2*>(kt + koff[rt] + 32 * kk);
            c0 = c.x;
            c1 = c.y;
          } else {
            lds_u64_at(kt, koff[rt] + 32 * kk, &c0, &c1);
          }
          if (kk == KCH - 1) {
            c0 &= kmask8[0];
            c1 &= kmask8[1];
          }
          w = widen_e4m3x8(c0, c1);
        } else {
          const uint32_t* p = reinterpret_cast<const uint32_t*>(kt + koff[rt] + SK * kk);
          w = make_uint4(p[0], p[1], p[2], p[3]);
          if (kk == KCH - 1) {
            w.x &= kmask[0];
            w.y &= kmask[1];
            w.z &= kmask[2];
            w.w &= kmask[3];
          }
        }
        sc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), qf[kk], sc[rt], 0, 0, 0);
      }
    }

    // ---- softmax numerators against a reference that rarely moves (log2 units)
    // A whole tile with nothing to leave out (all but the last tile of a range, normally) needs no
    // row masks and reads V as laid out; the test is wave-uniform, and the two places that differ
    // are branches around a few instructions, not copies of the arithmetic.
    const int nv = min(kTileRows, r1 - base);       // valid rows in this tile, >= 1
    const int skip_rel = t_skip - base;             // the one row to leave out, if it is in this tile
    const bool plain = nv == kTileRows && static_cast<unsigned>(skip_rel) >= static_cast<unsigned>(kTileRows);
    float x[2][4];
    float tmax = -INFINITY;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float s = sc[rt][r] * scale_log2e;
        x[rt][r] = (Q8 || ((16 * rt + 4 * lg + r) < nv && (16 * rt + 4 * lg + r) != skip_rel)) ? s : -INFINITY;
      }
    if (Q8 && !plain) {
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          x[rt][r] = ((16 * rt + 4 * lg + r) < nv && (16 * rt + 4 * lg + r) != skip_rel) ? x[rt][r] : -INFINITY;
    }
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 4; ++r) tmax = fmaxf(tmax, x[rt][r]);
    if (__any(tmax > m_run + kHeadroom)) {
      // first tile of the wavefront (m_run = -inf), or a score far above the reference: take
      // the true maximum over the four lane groups and rescale what has been accumulated
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);      // first tile: 2^-inf = 0
      l_run *= alpha;
#pragma unroll
      for (int reg = 0; reg < 4; ++reg) {
        const float at = __shfl(alpha, 4 * lg + reg);   // the head this accumulator register holds
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt][reg] *= at;
      }
      m_run = m_new;
    }
    float pr[2][4];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        pr[rt][r] = __builtin_amdgcn_exp2f(x[rt][r] - m_run);
        l_run += pr[rt][r];
      }

    // ---- P.V on the bf16 matrix instruction: acc[nt][reg] (head 4 lg + reg, channel slot l16 of
    // tile nt) += sum over the tile's 32 rows.  Contraction slot k = 8 lg + j of that instruction
    // is row 16 (j / 4) + 4 lg + (j % 4): exactly the rows whose probabilities this lane already
    // holds (j = 4 rt + r), so the A operand is built in-lane.  p is split into a bf16 head and a
    // bf16 remainder (two instructions), which keeps 16 significant bits of every probability.
    uint4 p_hi, p_lo;
    {
      uint32_t* ph = reinterpret_cast<uint32_t*>(&p_hi);
      uint32_t* pl = reinterpret_cast<uint32_t*>(&p_lo);
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const float a0 = pr[d >> 1][2 * (d & 1)], a1 = pr[d >> 1][2 * (d & 1) + 1];
        const uint32_t h = pack_bf16(a0, a1);
        ph[d] = h;
        pl[d] = pack_bf16(a0 - bf16_lo(h), a1 - bf16_hi(h));
      }
    }
    const bf16x8 pa_hi = __builtin_bit_cast(bf16x8, p_hi), pa_lo = __builtin_bit_cast(bf16x8, p_lo);
    // V rows: as laid out, unless the tile is partial or holds the row that is left out.  Rows
    // beyond the valid ones read the last valid row, the left-out row reads a valid neighbour
    // (there is one: a left-out LAST row has shortened the sequence instead): their
    // probabilities are 0, and 0 x (whatever bits such a row holds) must not reach the sums.
    int vo[8];
    if constexpr (Q8) {
      // kept between tiles as laid out; rewritten around the rare tile that differs (no selects
      // on the common path: this variant is bound by instruction issue)
      if (!plain) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          int row = min(16 * (j >> 2) + 4 * lg + (j & 3), nv - 1);
          row = row == skip_rel ? (skip_rel == 0 ? min(1, nv - 1) : skip_rel - 1) : row;
          vo_laid[j] = row * lpv + VLANE * l16;
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) vo[j] = vo_laid[j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        int row = min(16 * (j >> 2) + 4 * lg + (j & 3), nv - 1);
        row = row == skip_rel ? (skip_rel == 0 ? min(1, nv - 1) : skip_rel - 1) : row;
        vo[j] = plain ? vo_laid[j] : row * lpv + VLANE * l16;
      }
    }
    if constexpr (Q8) {
#pragma unroll
      for (int nq = 0; nq < NT / 4; ++nq) {
        uint32_t w[8];                 // four adjacent channels of row j, lowest channel in the low byte
#pragma unroll
        for (int j = 0; j < 8; ++j)
          w[j] = AL ? *reinterpret_cast<const uint32_t*>(vt + vo[j] + 64 * nq) : lds_u32_at(vt, vo[j] + 64 * nq);
        // 4 x 4 byte transposes, rows 0..3 and rows 4..7: first rows two by two (channels 0, 1 in
        // t, channels 2, 3 in u), then the pairs of rows
        uint32_t t[4], u[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          t[d] = __builtin_amdgcn_perm(w[2 * d + 1], w[2 * d], 0x05010400u);
          u[d] = __builtin_amdgcn_perm(w[2 * d + 1], w[2 * d], 0x07030602u);
        }
        uint4 bq[4];
        bq[0] = widen_e4m3x8(__builtin_amdgcn_perm(t[1], t[0], 0x05040100u), __builtin_amdgcn_perm(t[3], t[2], 0x05040100u));
        bq[1] = widen_e4m3x8(__builtin_amdgcn_perm(t[1], t[0], 0x07060302u), __builtin_amdgcn_perm(t[3], t[2], 0x07060302u));
        bq[2] = widen_e4m3x8(__builtin_amdgcn_perm(u[1], u[0], 0x05040100u), __builtin_amdgcn_perm(u[3], u[2], 0x05040100u));
        bq[3] = widen_e4m3x8(__builtin_amdgcn_perm(u[1], u[0], 0x07060302u), __builtin_amdgcn_perm(u[3], u[2], 0x07060302u));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bf16x8 vb = __builtin_bit_cast(bf16x8, bq[i]);
          acc[4 * nq + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vb, acc[4 * nq + i], 0, 0, 0);
          acc[4 * nq + i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vb, acc[4 * nq + i], 0, 0, 0);
        }
      }
    } else if constexpr (VPAIR) {
#pragma unroll
      for (int np = 0; np < NT / 2; ++np) {
        uint4 be, bo;   // even / odd channel of the pair, rows packed two by two
        uint32_t w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = *reinterpret_cast<const uint32_t*>(vt + vo[j] + SV * np);
        be.x = __builtin_amdgcn_perm(w[1], w[0], 0x05040100u);
        be.y = __builtin_amdgcn_perm(w[3], w[2], 0x05040100u);
        be.z = __builtin_amdgcn_perm(w[5], w[4], 0x05040100u);
        be.w = __builtin_amdgcn_perm(w[7], w[6], 0x05040100u);
        bo.x = __builtin_amdgcn_perm(w[1], w[0], 0x07060302u);
        bo.y = __builtin_amdgcn_perm(w[3], w[2], 0x07060302u);
        bo.z = __builtin_amdgcn_perm(w[5], w[4], 0x07060302u);
        bo.w = __builtin_amdgcn_perm(w[7], w[6], 0x07060302u);
        const bf16x8 vbe = __builtin_bit_cast(bf16x8, be), vbo = __builtin_bit_cast(bf16x8, bo);
        acc[2 * np] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vbe, acc[2 * np], 0, 0, 0);
        acc[2 * np + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vbo, acc[2 * np + 1], 0, 0, 0);
        acc[2 * np] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vbe, acc[2 * np], 0, 0, 0);
        acc[2 * np + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vbo, acc[2 * np + 1], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        uint32_t u[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) u[j] = *reinterpret_cast<const uint16_t*>(vt + vo[j] + 32 * nt);
        const uint4 bv = make_uint4(u[0] | (u[1] << 16), u[2] | (u[3] << 16), u[4] | (u[5] << 16), u[6] | (u[7] << 16));
        const bf16x8 vb = __builtin_bit_cast(bf16x8, bv);
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vb, acc[nt], 0, 0, 0);
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vb, acc[nt], 0, 0, 0);
      }
    }
    if (Q8 && !plain) {
#pragma unroll
      for (int j = 0; j < 8; ++j) vo_laid[j] = (16 * (j >> 2) + 4 * lg + (j & 3)) * lpv + VLANE * l16;
    }
  }

  // ---- fold lane groups, then the four wavefronts, through LDS
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();                                   // every wavefront is done with its tile area
  float* wm = reinterpret_cast<float*>(smem + wave * a.lds_wave_bytes);   // [16] max, [16] sum, [8][16 NT] acc
  if (lg == 0) {
    wm[l16] = m_run;
    wm[16 + l16] = l_run;
  }
#pragma unroll
  for (int reg = 0; reg < 4; ++reg) {
    const int g = 4 * lg + reg;
    if (g < (cols > kMaxGroup ? kMaxCols : kMaxGroup)) {   // the hand-over area holds 8 columns, or all 16 when more are in use
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        wm[32 + g * (16 * NT) + (Q8 ? 64 * (nt >> 2) + 4 * l16 + (nt & 3) : VPAIR ? 32 * (nt >> 1) + 2 * l16 + (nt & 1) : 16 * nt + l16)] = acc[nt][reg];
    }
  }
  __syncthreads();
  for (int e = tid; e < cols * dv; e += 256) {
    const int g = e / dv, c = e - g * dv;             // g: column
    float mw[4], mstar = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mw[w] = reinterpret_cast<const float*>(smem + w * a.lds_wave_bytes)[g];
      mstar = fmaxf(mstar, mw[w]);
    }
    float num = 0.f, den = 0.f;
    if (mstar > -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* pw = reinterpret_cast<const float*>(smem + w * a.lds_wave_bytes);
        const float wt = exp2f(mw[w] - mstar);
        den = fmaf(wt, pw[16 + g], den);
        num = fmaf(wt, pw[32 + g * (16 * NT) + c], num);
      }
    }
    if constexpr (Q8) num *= a.v_scale[h];          // codes -> values
    const int qt = (g * a.group_inv16) >> 16;         // g / G
    const long long hq = static_cast<long long>(b) * a.n_tok * a.n_q + h * G + (qt * a.n_q + (g - qt * G));
    if (a.direct_out) {
      a.out[hq * dv + c] = den > 0.f ? num / den : 0.f;
    } else {
      a.part_acc[(hq * a.n_slots + split) * dv + c] = num;
      if (c == 0) {
        a.part_ml[(hq * a.n_slots + split) * 2 + 0] = mstar;
        a.part_ml[(hq * a.n_slots + split) * 2 + 1] = den;
      }
    }
  }
}

template <int KCH, int NT, bool VPAIR, bool PAGED, bool Q8, bool AL = false, bool MX4 = false>
hipError_t launch_inst2(const DecodeArgs& a, hipStream_t stream) {
  // scanning workgroups, then (decode step: n_slots = n_split + 1) one per (b, h) for the new token
  dim3 grid(static_cast<unsigned>(a.n_slots) * a.n_kv * a.batch), block(256);
  const size_t lds = 4 * static_cast<size_t>(a.lds_wave_bytes);
  if (lds > 64 * 1024) {
    // more than the default dynamic-LDS limit: raise it once per kernel (gfx950 has 160 KB per CU)
    const hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(&decode_mfma_kernel<KCH, NT, VPAIR, PAGED, Q8, AL, MX4>), static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((decode_mfma_kernel<KCH, NT, VPAIR, PAGED, Q8, AL, MX4>), grid, block, lds, stream, a);
  return hipGetLastError();
}

}  // namespace

}  // namespace rap

#endif  // RAP_DECODE_KERNEL_H_

// Host-side harness for the CPU tests: runs librap's own arithmetic and indexing helpers
// (paper_2602_02599_amd/csrc/rap_arith.h, the code the kernels compile) on the host, so that
// pytest can compare them with the float64 oracle and with long-double library routines, under the
// host sanitizers.  Built with hipcc's host pass only; nothing here touches a GPU.
//
//   rap_arith_host bf16      stdin: float64[n]  -> stdout: uint16[n]   f64_to_bf16_rne
//   rap_arith_host sincos    stdin: float64[n]  -> stdout: float64[2n] sincos_f64 (sin, cos)
//   rap_arith_host odd448    stdin: float64[n]  -> stdout: uint32[n]   bits of f64_to_f32_odd_clamped448
//   rap_arith_host mx4       stdin: float64[32 n] (n blocks) -> stdout: per block one byte
//                               mx_shared_exponent + 127 and 32 bytes f64_to_e2m1(x * pow2_neg(e))
//   rap_arith_host loadplan  -> text, one line per (kind, width, element size): what the decode
//                               kernel's tile loads touch; exit status 1 if any load leaves its tile,
//                               or any tile byte is fetched twice or not at all
//   rap_arith_host loadplan-trim1  the same with only the LAST load of a run trimmed (a planted
//                               mistake: bf16 K tiles whose width needs an odd number of loads
//                               then read past the tile; the tests expect this one to fail)
#include <stdio.h>
#include <string.h>

#include <vector>

#include "../../paper_2602_02599_amd/csrc/rap_arith.h"

namespace {

std::vector<double> read_doubles() {
  std::vector<double> v;
  double buf[4096];
  size_t n;
  while ((n = fread(buf, sizeof(double), 4096, stdin)) > 0) v.insert(v.end(), buf, buf + n);
  return v;
}

// One line per tile shape: the highest byte (exclusive) any issued load touches and the number of
// tile bytes no load covers, for the full tile and for every partial tile of 8 k (16 k) rows.
int loadplan(bool trim_one_only) {
  int bad = 0;
  for (int q8 = 0; q8 < 2; ++q8) {
    const int eb = q8 ? 1 : 2, row_quantum = q8 ? 16 : 8;
    for (int kind = 0; kind < 2; ++kind) {            // 0: K tile (even widths), 1: V tile
      for (int d = kind == 0 ? 2 : 1; d <= 128; d += kind == 0 ? 2 : 1) {
        const int n_ld = kind == 0 ? rap::k_tile_loads((d + 31) / 32, q8 != 0) : rap::v_tile_loads(rap::decode_v_tiles(d, q8 != 0), q8 != 0);
        const int n_trim = trim_one_only ? 1 : (kind == 0 ? rap::k_tile_trimmed(q8 != 0) : rap::v_tile_trimmed(q8 != 0));
        const int pitch = eb * d;
        for (int rows = row_quantum; rows <= 32; rows += row_quantum) {
          const bool whole = rows == 32;
          const int bytes = rows * pitch;
          std::vector<char> hit(static_cast<size_t>(1024) * n_ld + 16, 0);
          int top = 0;
          for (int j = 0; j < n_ld; ++j)
            for (int lane = 0; lane < 64; ++lane)
              if (rap::tile_load_issued(j, lane, n_ld, n_trim, bytes, whole)) {
                const int at = 1024 * j + 16 * lane;
                for (int i = 0; i < 16; ++i) hit[at + i] += 1;
                top = at + 16 > top ? at + 16 : top;
              }
          int missed = 0, twice = 0;
          for (int i = 0; i < bytes; ++i) {
            missed += hit[i] == 0;
            twice += hit[i] > 1;
          }
          printf("%s q8=%d d=%d rows=%d n_ld=%d bytes=%d top=%d missed=%d twice=%d\n", kind == 0 ? "K" : "V", q8, d, rows, n_ld,
                 bytes, top, missed, twice);
          bad += top > bytes || missed != 0 || twice != 0;
        }
      }
    }
  }
  return bad;
}

}  // namespace

int main(int argc, char** argv) {
  if (argc != 2) {
    fprintf(stderr, "usage: rap_arith_host bf16|sincos|odd448|mx4|loadplan|loadplan-trim1\n");
    return 2;
  }
  if (strcmp(argv[1], "loadplan") == 0) return loadplan(false) == 0 ? 0 : 1;
  if (strcmp(argv[1], "loadplan-trim1") == 0) return loadplan(true) == 0 ? 0 : 1;
  const std::vector<double> in = read_doubles();
  if (strcmp(argv[1], "bf16") == 0) {
    std::vector<uint16_t> out(in.size());
    for (size_t i = 0; i < in.size(); ++i) out[i] = rap::f64_to_bf16_rne(in[i]);
    fwrite(out.data(), sizeof(uint16_t), out.size(), stdout);
  } else if (strcmp(argv[1], "sincos") == 0) {
    std::vector<double> out(2 * in.size());
    for (size_t i = 0; i < in.size(); ++i) rap::sincos_f64(in[i], &out[2 * i], &out[2 * i + 1]);
    fwrite(out.data(), sizeof(double), out.size(), stdout);
  } else if (strcmp(argv[1], "odd448") == 0) {
    std::vector<uint32_t> out(in.size());
    for (size_t i = 0; i < in.size(); ++i) out[i] = rap::f32_bits(rap::f64_to_f32_odd_clamped448(in[i]));
    fwrite(out.data(), sizeof(uint32_t), out.size(), stdout);
  } else if (strcmp(argv[1], "mx4") == 0) {
    std::vector<uint8_t> out;
    for (size_t b = 0; b + 32 <= in.size(); b += 32) {
      double amax = 0.0;
      for (int i = 0; i < 32; ++i) {
        const double m = in[b + i] < 0 ? -in[b + i] : in[b + i];
        amax = m > amax ? m : amax;
      }
      const int e = rap::mx_shared_exponent(amax);
      out.push_back(static_cast<uint8_t>(e + 127));
      for (int i = 0; i < 32; ++i) out.push_back(static_cast<uint8_t>(rap::f64_to_e2m1(in[b + i] * rap::pow2_neg(e))));
    }
    fwrite(out.data(), 1, out.size(), stdout);
  } else {
    fprintf(stderr, "unknown command %s\n", argv[1]);
    return 2;
  }
  return 0;
}

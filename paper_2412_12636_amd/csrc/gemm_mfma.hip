// bf16 GEMM through the matrix cores: layout dispatch and tile choice.  The kernels live in
// gemm_mfma_impl.h and are instantiated in one translation unit per operand layout.
#include <stdio.h>
#include <stdlib.h>

#include "gemm.h"

namespace tmk {

int gemm_mfma_nt(const GemmArgs &g, hipStream_t s);  // y = x W^T         (both reduction axes contiguous)
int gemm_mfma_nn(const GemmArgs &g, hipStream_t s);  // dx = dy W         (W read along its strided axis)
int gemm_mfma_tn(const GemmArgs &g, hipStream_t s);  // dW += dy^T x      (both strided, fp32 accumulate)

bool gemm_mfma_supported(const GemmArgs &g) {
  auto operand_ok = [&](const void *ptr, int64_t rs, int64_t cs, int64_t rows) {
    if (((uintptr_t)ptr) & 15) return false;
    if (cs == 1) return rs % 8 == 0 && g.K % 8 == 0;
    if (rs == 1) return cs % 8 == 0 && rows % 8 == 0;
    return false;
  };
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
  if (g.M > 0x7fffffff || g.N > 0x7fffffff || g.K > 0x7fffffff) return false;
  if (!operand_ok(g.A, g.a_rs, g.a_cs, g.M) || !operand_ok(g.B, g.b_rs, g.b_cs, g.N)) return false;
  const bool akc = g.a_cs == 1, bkc = g.b_cs == 1;
  const int64_t a_bytes = (akc ? g.M * g.a_rs : g.K * g.a_cs) * 2, b_bytes = (bkc ? g.N * g.b_rs : g.K * g.b_cs) * 2;
  const int64_t c_bytes = g.M * g.ldc * (g.c_mode ? 4 : 2);
  if (a_bytes >= (1LL << 31) || b_bytes >= (1LL << 31) || c_bytes >= (1LL << 31)) return false;  // 32-bit offsets
  if (g.ldc % 8 || (((uintptr_t)g.C) & 15)) return false;
  return g.c_mode ? (!akc && !bkc) : akc;
}

// Block tile: the candidate with the lowest estimated time.  A compute unit holds `occ` blocks of a
// tile shape at once (LDS: two stages of (BM+BN) x 128 bytes out of 160 KB), so the chip works through
// the tiles in passes of 256*occ, each pass taking occ * BM * BN / speed, where speed is the shape's
// measured rate relative to 128x192 on the 175B-shard products.  TM_GEMM_TILE=<BM>x<BN> in the
// environment overrides the choice (tuning aid).
void gemm_pick_tile(int64_t M, int64_t N, int &bm, int &bn) {
  static const int cand[9][2] = {{128, 192}, {128, 128}, {256, 256}, {256, 192}, {192, 192},
                                 {256, 128}, {128, 256}, {192, 128}, {192, 256}};
  static const double speed[9] = {1.0, 0.97, 1.05, 0.95, 0.9, 0.87, 0.87, 0.87, 0.75};
  static const int occ[9] = {2, 2, 1, 1, 1, 1, 1, 2, 1};
  static int forced_m = -1, forced_n = -1;
  if (forced_m < 0) {
    forced_m = forced_n = 0;
    if (const char *e = getenv("TM_GEMM_TILE")) {
      int a = 0, b = 0;
      if (sscanf(e, "%dx%d", &a, &b) == 2)
        for (int c = 0; c < 9; ++c)
          if (cand[c][0] == a && cand[c][1] == b) forced_m = a, forced_n = b;
    }
  }
  if (forced_m > 0) {
    bm = forced_m;
    bn = forced_n;
    return;
  }
  double best = 1e300;
  for (int c = 0; c < 9; ++c) {
    const int64_t nb = ceil_div(M, cand[c][0]) * ceil_div(N, cand[c][1]);
    const double passes = (double)ceil_div(nb, 256 * occ[c]);
    const double cost = passes * occ[c] * cand[c][0] * cand[c][1] / speed[c];
    if (cost < best) {
      best = cost;
      bm = cand[c][0];
      bn = cand[c][1];
    }
  }
}

int gemm_mfma(const GemmArgs &g, hipStream_t s) {
  const bool akc = g.a_cs == 1, bkc = g.b_cs == 1;
  if (!g.c_mode && akc && bkc) return gemm_mfma_nt(g, s);
  if (!g.c_mode && akc && !bkc) return gemm_mfma_nn(g, s);
  if (g.c_mode && !akc && !bkc) return gemm_mfma_tn(g, s);
  return fail(TM_EINVAL, "gemm_mfma: operand layout not instantiated");
}

}  // namespace tmk

// bf16 GEMM through the matrix cores: layout dispatch and choice of the tile configuration.  The kernels
// live in gemm_mfma_impl.h and are instantiated in one translation unit per operand layout.
#include <stdio.h>
#include <stdlib.h>

#include <map>
#include <mutex>
#include <tuple>
#include <vector>

#include "gemm.h"

namespace tmk {

int gemm_mfma_nt(const GemmArgs &g, int config, hipStream_t s);  // y = x W^T       (both reduction axes contiguous)
int gemm_mfma_nn(const GemmArgs &g, int config, hipStream_t s);  // dx = dy W       (W read along its strided axis)
int gemm_mfma_tn(const GemmArgs &g, int config, hipStream_t s);  // dW (+)= dy^T x  (both strided, fp32 result)
int gemm_mfma_nn_partial(const GemmArgs &g, bool large, hipStream_t s);  // dx = dy W in k_splits fp32 parts

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

// ---- tile configurations -------------------------------------------------------------------------
// Same order as TM_GEMM_CONFIGS in gemm_mfma_impl.h.  occ: blocks a compute unit holds at once (LDS: two
// stages of (BM+BN) x 128 bytes out of 160 KB; four-wave blocks of up to 256x128 outputs leave room for
// two).  speed[layout]: measured rate per busy compute unit relative to 128x192, per operand layout (0: both
// reduction axes contiguous, 1: B strided, 2: both strided; the transposing LDS reads of the strided layouts
// favour the small four-wave tiles, the plain reads the large ones), from products of 2048 to 4096 rows.
struct TileConfig {
  int bm, bn, wgm, wgn, occ;
  double speed[3];
};
static const TileConfig kConfigs[] = {
    {128, 192, 2, 2, 2, {1.00, 1.00, 1.00}}, {128, 128, 2, 2, 2, {0.95, 0.86, 0.91}}, {192, 128, 2, 2, 2, {0.98, 0.98, 1.00}},
    {256, 192, 4, 2, 1, {1.08, 0.90, 0.88}}, {192, 256, 2, 4, 1, {1.00, 0.90, 0.90}}, {256, 256, 2, 4, 1, {1.22, 1.00, 1.00}},
    {256, 256, 4, 2, 1, {1.20, 0.98, 1.00}}, {256, 128, 4, 2, 1, {0.88, 0.78, 0.80}}, {256, 192, 2, 2, 1, {1.09, 0.80, 0.83}},
    // the alternating kernel (gemm_alt_kernel)
    {256, 256, 2, 4, 1, {1.00, 1.10, 1.06}}, {256, 256, 4, 2, 1, {1.00, 1.10, 1.06}},
    // the pipelined kernel with three LDS stages
    {256, 128, 4, 2, 1, {1.05, 0.78, 0.80}}, {128, 256, 2, 4, 1, {1.05, 0.78, 0.80}},
    // the kernel with loader waves (gemm_ldw_kernel)
    {256, 192, 4, 2, 1, {1.12, 1.17, 1.10}}, {128, 192, 2, 2, 2, {0.70, 0.80, 0.85}}, {256, 192, 4, 2, 1, {1.10, 1.10, 1.05}},
};
constexpr int kNumConfigs = sizeof(kConfigs) / sizeof(kConfigs[0]);

static int layout_of(const GemmArgs &g) { return g.c_mode ? 2 : (g.b_cs == 1 ? 0 : 1); }

// Estimated time: the chip works through the tiles in passes of 256*occ blocks, each pass taking
// occ * BM * BN / speed.
static int heuristic_config(const GemmArgs &g) {
  double best = 1e300;
  int pick = 0;
  const int layout = layout_of(g);
  for (int c = 0; c < kNumConfigs; ++c) {
    const TileConfig &t = kConfigs[c];
    const int64_t nb = ceil_div(g.M, t.bm) * ceil_div(g.N, t.bn);
    const double passes = (double)ceil_div(nb, 256 * t.occ);
    const double cost = passes * t.occ * t.bm * t.bn / t.speed[layout];
    if (cost < best) best = cost, pick = c;
  }
  return pick;
}

// TM_GEMM_TILE=<BM>x<BN>x<WGM>x<WGN> in the environment forces one configuration (tuning aid).
static int g_override_config = -1;  // tm_gemm_force_config
static int forced_config() {
  if (g_override_config >= 0) return g_override_config;
  static int forced = -2;
  if (forced == -2) {
    forced = -1;
    if (const char *e = getenv("TM_GEMM_TILE")) {
      int a = 0, b = 0, c = 0, d = 0;
      if (sscanf(e, "%dx%dx%dx%d", &a, &b, &c, &d) == 4)
        for (int i = 0; i < kNumConfigs; ++i)
          if (kConfigs[i].bm == a && kConfigs[i].bn == b && kConfigs[i].wgm == c && kConfigs[i].wgn == d) forced = i;
    }
  }
  return forced;
}

int gemm_mfma_config_count() { return kNumConfigs; }
int gemm_mfma_force_config(int index) {
  if (index < -1 || index >= kNumConfigs) return fail(TM_EINVAL, "gemm_force_config: no configuration %d", index);
  g_override_config = index;
  return TM_OK;
}

// Configurations found by gemm_mfma_tune(), keyed by (layout, M, N, K).  A weight-gradient product that also applies
// the update (c_mode 3) spends most of its time in the epilogue, streaming the optimizer state.  Where the large
// staggered form does not apply (fused_on_large_tiles below) it is faster with two small blocks per compute unit than
// with one large block whose units all stream at once, so it keeps the best of the configurations that allow two
// blocks: layout key 3.
typedef std::tuple<int, int64_t, int64_t, int64_t> TuneKey;
static std::map<TuneKey, int> g_tuned;
static std::mutex g_tuned_mutex;
constexpr int kFusedLayoutKey = 3;

static int heuristic_config_fused(const GemmArgs &g) {
  double best = 1e300;
  int pick = 0;
  for (int c = 0; c < kNumConfigs; ++c) {
    const TileConfig &t = kConfigs[c];
    if (t.occ < 2) continue;
    const int64_t nb = ceil_div(g.M, t.bm) * ceil_div(g.N, t.bn);
    const double cost = (double)ceil_div(nb, 256 * t.occ) * t.occ * t.bm * t.bn / t.speed[2];
    if (cost < best) best = cost, pick = c;
  }
  return pick;
}

// A fused-update product whose 256x192 tiles fill the chip at least twice and whose main loop is short enough for
// the update to matter (up to 4096 tokens) runs on the kernel with loader waves, one block per compute unit, with
// start offsets between the units (gemm_mfma_impl.h, stagger_by_unit): 0.53 -> 0.42 ms for the FC-sized matrices of
// the 175B shard.  TM_GEMM_FUSED_LARGE=0 switches this off, TM_GEMM_FUSED_LARGE_MAXT moves the token limit.
constexpr int kLdwLargeConfig = 13;
static bool fused_on_large_tiles(const GemmArgs &g) {
  static int on = -1;
  static int64_t max_t = 4096;
  if (on < 0) {
    const char *e = getenv("TM_GEMM_FUSED_LARGE");
    on = e ? atoi(e) != 0 : 1;
    if (const char *t = getenv("TM_GEMM_FUSED_LARGE_MAXT")) max_t = atoll(t);
  }
  const TileConfig &t = kConfigs[kLdwLargeConfig];
  return on && g.K <= max_t && g.K % 64 == 0 && ceil_div(g.M, t.bm) * ceil_div(g.N, t.bn) >= 512;
}

static int pick_config(const GemmArgs &g) {
  const int f = forced_config();
  if (f >= 0) return f;
  const bool fused = g.c_mode == 3;
  if (fused && fused_on_large_tiles(g)) return kLdwLargeConfig;
  {
    std::lock_guard<std::mutex> lock(g_tuned_mutex);
    auto it = g_tuned.find(TuneKey(fused ? kFusedLayoutKey : layout_of(g), g.M, g.N, g.K));
    if (it != g_tuned.end()) return it->second;
  }
  return fused ? heuristic_config_fused(g) : heuristic_config(g);
}

static int launch_config(const GemmArgs &g, int config, hipStream_t s) {
  const bool akc = g.a_cs == 1, bkc = g.b_cs == 1;
  if (!g.c_mode && akc && bkc) return gemm_mfma_nt(g, config, s);
  if (!g.c_mode && akc && !bkc) return gemm_mfma_nn(g, config, s);
  if (g.c_mode && !akc && !bkc) return gemm_mfma_tn(g, config, s);
  return fail(TM_EINVAL, "gemm_mfma: operand layout not instantiated");
}

// ---- split reduction --------------------------------------------------------------------------------
// dx = dy W with a long reduction and few output tiles (the out-projection's input gradient: 2048 x 1536
// over 12288) fills a fraction of the chip.  With scratch from the caller the reduction is cut into parts
// whose 128x192 tiles make one pass of 512 blocks; the fp32 parts are added in part order and rounded once.
// The choice depends on the shape only, so results stay reproducible.
// With 256x192 tiles (the kernel with loader waves, one block per compute unit) when those make one pass of at least
// 192 blocks, else with 128x192 tiles, two blocks per unit.
static int splitk_parts(const GemmArgs &g, bool *large = nullptr) {
  if (large) *large = false;
  if (g.c_mode != 0 || g.bias || g.residual || !(g.a_cs == 1 && g.b_cs != 1)) return 1;
  const int64_t tiles = ceil_div(g.M, 128) * ceil_div(g.N, 192);
  if (tiles > 256 || g.K < 4096) return 1;
  const int64_t big = ceil_div(g.M, 256) * ceil_div(g.N, 192);
  int parts = (int)(256 / big);
  if (parts > 8) parts = 8;
  while (parts > 1 && g.K % (64 * parts) != 0) --parts;
  if (parts > 1 && big * parts >= 192) {
    if (large) *large = true;
    return parts;
  }
  parts = (int)(512 / tiles);
  if (parts > 8) parts = 8;
  while (parts > 1 && g.K % (64 * parts) != 0) --parts;
  return parts;
}

int64_t gemm_mfma_splitk_bytes(const GemmArgs &g) {
  const int parts = splitk_parts(g);
  return parts > 1 ? (int64_t)parts * g.M * g.N * 4 : 0;
}

// out[m, n] (bf16, row stride ldc) = sum over parts of part[p][m][n], eight columns per thread
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int parts, int64_t M, int64_t N,
                                                            bf16 *__restrict__ out, int64_t ldc) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x, per_row = N / 8;
  if (idx >= M * per_row) return;
  const int64_t m = idx / per_row, n = (idx % per_row) * 8;
  f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = lo;
  for (int q = 0; q < parts; ++q) {
    const float *src = part + ((int64_t)q * M + m) * N + n;
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src));
    const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src) + 1);
#pragma unroll
    for (int e = 0; e < 4; ++e) lo[e] += a[e], hi[e] += b[e];
  }
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16)lo[e], o[4 + e] = (bf16)hi[e];
  *reinterpret_cast<bf16x8 *>(out + m * ldc + n) = o;
}

int gemm_mfma(const GemmArgs &g, hipStream_t s) {
  bool large = false;
  const int parts = splitk_parts(g, &large);
  if (parts > 1 && g.splitk_scratch && g.splitk_bytes >= (int64_t)parts * g.M * g.N * 4 &&
      (((uintptr_t)g.splitk_scratch) & 15) == 0 && g.M * g.N * 4 < (1LL << 31) && forced_config() < 0) {
    GemmArgs p = g;
    p.C = g.splitk_scratch;
    p.ldc = g.N;
    p.c_mode = 2;
    p.k_splits = parts;
    if (int e = gemm_mfma_nn_partial(p, large, s)) return e;
    const int64_t groups = g.M * (g.N / 8);
    splitk_reduce_kernel<<<(unsigned)ceil_div(groups, (int64_t)256), 256, 0, s>>>((const float *)g.splitk_scratch, parts, g.M, g.N,
                                                                              (bf16 *)g.C, g.ldc);
    return check_launch("splitk_reduce");
  }
  return launch_config(g, pick_config(g), s);
}

// Times every configuration and remembers the fastest for this layout and shape.  `variants` are n
// instances of the same product on different memory (say, the weights of different layers): the
// launches cycle through them, so that an operand that is cold in the real sequence is cold here too.
// The result buffers are overwritten several times; an accumulating product is timed in its
// overwriting form.  Synchronises the stream.
int gemm_mfma_tune(const GemmArgs *variants, int n, hipStream_t s) {
  if (n <= 0 || forced_config() >= 0) return TM_OK;
  std::vector<GemmArgs> v(variants, variants + n);
  for (GemmArgs &g : v) {
    if (!gemm_mfma_supported(g) || g.K % 64 != 0) return TM_OK;
    if (g.M != v[0].M || g.N != v[0].N || g.K != v[0].K || layout_of(g) != layout_of(v[0]))
      return fail(TM_EINVAL, "gemm_mfma_tune: variants differ in shape or layout");
    g.bias = nullptr;
    g.residual = nullptr;
    if (g.c_mode == 1) g.c_mode = 2;
  }
  const TuneKey key(layout_of(v[0]), v[0].M, v[0].N, v[0].K);
  {
    std::lock_guard<std::mutex> lock(g_tuned_mutex);
    if (g_tuned.count(key)) return TM_OK;
  }
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return fail(TM_ELAUNCH, "gemm_mfma_tune: cannot create events");
  float ms_of[kNumConfigs];
  int rc = TM_OK, turn = 0;
  for (int c = 0; c < kNumConfigs && rc == TM_OK; ++c) {
    ms_of[c] = 1e30f;
    rc = launch_config(v[turn++ % n], c, s);  // warm-up: code object load, clocks
    for (int r = 0; r < 3 && rc == TM_OK; ++r) {
      if (hipEventRecord(e0, s) != hipSuccess) rc = fail(TM_ELAUNCH, "gemm_mfma_tune: event record");
      if (rc == TM_OK) rc = launch_config(v[turn++ % n], c, s);
      if (rc == TM_OK && (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess))
        rc = fail(TM_ELAUNCH, "gemm_mfma_tune: event wait");
      float ms = 0.f;
      if (rc == TM_OK && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms < ms_of[c]) ms_of[c] = ms;
    }
  }
  int best = 0, best_two = -1;  // best_two: among the configurations with two blocks per compute unit
  for (int c = 0; c < kNumConfigs; ++c) {
    if (ms_of[c] < ms_of[best]) best = c;
    if (kConfigs[c].occ >= 2 && (best_two < 0 || ms_of[c] < ms_of[best_two])) best_two = c;
  }
  // the cost model's pick stays unless it loses by more than 2 %: keeps the choice stable against timer noise
  const int first = heuristic_config(v[0]);
  if (ms_of[first] <= 1.02f * ms_of[best]) best = first;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != TM_OK) return rc;
  if (getenv("TM_GEMM_TUNE_LOG")) {
    fprintf(stderr, "tune layout %d M=%lld N=%lld K=%lld:", layout_of(v[0]), (long long)v[0].M, (long long)v[0].N, (long long)v[0].K);
    for (int c = 0; c < kNumConfigs; ++c)
      fprintf(stderr, " %dx%dx%dx%d=%.4f%s", kConfigs[c].bm, kConfigs[c].bn, kConfigs[c].wgm, kConfigs[c].wgn, ms_of[c], c == best ? "*" : "");
    fprintf(stderr, "\n");
  }
  std::lock_guard<std::mutex> lock(g_tuned_mutex);
  g_tuned[key] = best;
  if (layout_of(v[0]) == 2 && best_two >= 0)
    g_tuned[TuneKey(kFusedLayoutKey, v[0].M, v[0].N, v[0].K)] = getenv("TM_GEMM_FUSED_ANY") ? best : best_two;
  return TM_OK;
}

}  // namespace tmk

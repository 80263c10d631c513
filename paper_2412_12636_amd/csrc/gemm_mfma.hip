// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One 256-thread block (four wavefronts in a 2x2 grid) owns a BM x BN output tile and walks the
// reduction axis 64 elements at a time.  Both operand tiles are staged in LDS as [row][64 k]
// (128 bytes per row, 16-byte chunks XOR-swizzled by the row so that a wavefront's fragment reads
// spread over all banks), double buffered: global loads for step k+1 are issued before the MFMAs
// of step k and written to the other LDS buffer afterwards, one barrier per step.
//
// An operand whose reduction axis is the strided one (weights in the input-gradient product, both
// operands in the weight-gradient product) is read with 16-byte loads along its contiguous axis
// and transposed in registers (4 k-rows x 8 columns per thread) on the way into LDS, so the MFMA
// side never sees the difference and no transposed copies are kept in HBM.
//
// Block index -> tile mapping: consecutive hardware block ids land on different XCDs (8 per chip,
// each with its own L2); ids are re-numbered so that every XCD works on a contiguous range of
// tiles, with the M tiles of one weight column adjacent.
#include <string>

#include "gemm.h"

namespace tmk {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;          // reduction elements per step
constexpr int ROWB = BK * 2;    // bytes per LDS row
constexpr int NXCD = 8;

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// ---- operand with contiguous reduction axis: element (r, k) at base[r*ld + k] -------------------
template <int R> struct LoaderKC {
  static constexpr int NCH = R / 32;  // 16-byte chunks per thread
  u32x4 reg[NCH];
  __device__ __forceinline__ void g2r(const bf16 *base, int64_t ld, int r_valid, int k_valid) {
    const int c = threadIdx.x & 7, r0 = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int r = r0 + 32 * i;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < r_valid && c * 8 < k_valid) v = *reinterpret_cast<const u32x4 *>(base + (int64_t)r * ld + c * 8);
      reg[i] = v;
    }
  }
  __device__ __forceinline__ void r2s(char *lds) const {
    const int c = threadIdx.x & 7, r0 = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int r = r0 + 32 * i;
      *reinterpret_cast<u32x4 *>(lds + r * ROWB + ((c ^ swz(r)) << 4)) = reg[i];
    }
  }
};

// ---- operand with strided reduction axis: element (r, k) at base[k*ld + r] -----------------------
template <int R> struct LoaderKS {
  static constexpr int RB = R / 8;          // 8-column blocks along r
  static constexpr int KG_STEP = 256 / RB;  // k-groups (of 4 rows) covered by one pass of the block
  static constexpr int NB = 16 / KG_STEP;   // passes: 16 k-groups in a 64-deep step
  u32x4 reg[NB][4];
  __device__ __forceinline__ void g2r(const bf16 *base, int64_t ld, int r_valid, int k_valid) {
    const int rb = threadIdx.x % RB, kg0 = threadIdx.x / RB;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int kg = kg0 + i * KG_STEP;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = kg * 4 + j;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (rb * 8 < r_valid && k < k_valid) v = *reinterpret_cast<const u32x4 *>(base + (int64_t)k * ld + rb * 8);
        reg[i][j] = v;
      }
    }
  }
  __device__ __forceinline__ void r2s(char *lds) const {
    const int rb = threadIdx.x % RB, kg0 = threadIdx.x / RB;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int kg = kg0 + i * KG_STEP;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int w = e >> 1;
        u32x2 o;
        if (e & 1) {
          o[0] = (reg[i][0][w] >> 16) | (reg[i][1][w] & 0xffff0000u);
          o[1] = (reg[i][2][w] >> 16) | (reg[i][3][w] & 0xffff0000u);
        } else {
          o[0] = (reg[i][0][w] & 0xffffu) | (reg[i][1][w] << 16);
          o[1] = (reg[i][2][w] & 0xffffu) | (reg[i][3][w] << 16);
        }
        const int r = rb * 8 + e;
        *reinterpret_cast<u32x2 *>(lds + r * ROWB + (((kg >> 1) ^ swz(r)) << 4) + ((kg & 1) << 3)) = o;
      }
    }
  }
};

template <int R, bool KC> struct LoaderSel { typedef LoaderKC<R> type; };
template <int R> struct LoaderSel<R, false> { typedef LoaderKS<R> type; };

struct MfmaGemmParams {
  int M, N, K;
  const bf16 *A;
  int64_t lda;  // the non-unit stride of A
  const bf16 *B;
  int64_t ldb;
  void *C;
  int64_t ldc;
  const bf16 *bias;
  const bf16 *residual;
  int tiles_m, tiles_n;
};

// EPI 0: bf16 C = acc (+bias) (+residual);  EPI 1: fp32 C += acc
template <int BM, int BN, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const MfmaGemmParams p) {
  extern __shared__ __align__(16) char lds[];
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;

  // XCD-aware tile numbering
  const int nblk = gridDim.x;
  const int pid = blockIdx.x;
  const int xcd = pid % NXCD, local = pid / NXCD;
  const int base = nblk / NXCD, rem = nblk % NXCD;
  const int lid = xcd * base + (xcd < rem ? xcd : rem) + local;
  const int tile_m = lid % p.tiles_m, tile_n = lid / p.tiles_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, hh = lane >> 5;

  typename LoaderSel<BM, A_KC>::type la;
  typename LoaderSel<BN, B_KC>::type lb;
  const bf16 *Ab = A_KC ? p.A + (int64_t)m0 * p.lda : p.A + m0;
  const bf16 *Bb = B_KC ? p.B + (int64_t)n0 * p.ldb : p.B + n0;
  const int m_valid = p.M - m0, n_valid = p.N - n0;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  la.g2r(Ab, p.lda, m_valid, p.K);
  lb.g2r(Bb, p.ldb, n_valid, p.K);
  la.r2s(lds);
  lb.r2s(lds + A_BYTES);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      const int k0 = (kt + 1) * BK;
      la.g2r(A_KC ? Ab + k0 : Ab + (int64_t)k0 * p.lda, p.lda, m_valid, p.K - k0);
      lb.g2r(B_KC ? Bb + k0 : Bb + (int64_t)k0 * p.ldb, p.ldb, n_valid, p.K - k0);
    }
    const char *As = lds + cur * STAGE;
    const char *Bs = As + A_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = wm * WM + i * 32 + l32;
        a[i] = *reinterpret_cast<const bf16x8 *>(As + r * ROWB + (((2 * ks + hh) ^ swz(r)) << 4));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = wn * WN + j * 32 + l32;
        b[j] = *reinterpret_cast<const bf16x8 *>(Bs + r * ROWB + (((2 * ks + hh) ^ swz(r)) << 4));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      char *nxt = lds + (cur ^ 1) * STAGE;
      la.r2s(nxt);
      lb.r2s(nxt + A_BYTES);
    }
    __syncthreads();
  }

  // epilogue.  Accumulator element v of a 32x32 tile: row 8*(v/4) + 4*hh + v%4, column lane%32.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * WN + j * 32 + l32;
    if (col >= p.N) continue;
    float bv = 0.f;
    if (EPI == 0 && p.bias) bv = (float)p.bias[col];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
        if (row >= p.M) continue;
        const int64_t off = (int64_t)row * p.ldc + col;
        if (EPI == 0) {
          float r = acc[i][j][v] + bv;
          if (p.residual) r += (float)p.residual[off];
          reinterpret_cast<bf16 *>(p.C)[off] = (bf16)r;
        } else {
          reinterpret_cast<float *>(p.C)[off] += acc[i][j][v];
        }
      }
    }
  }
}

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
  return g.accumulate_f32 ? (!akc && !bkc) : akc;
}

template <int BM, int BN, bool A_KC, bool B_KC, int EPI>
static int launch_tile(const GemmArgs &g, hipStream_t s) {
  MfmaGemmParams p;
  p.M = (int)g.M;
  p.N = (int)g.N;
  p.K = (int)g.K;
  p.A = (const bf16 *)g.A;
  p.lda = A_KC ? g.a_rs : g.a_cs;
  p.B = (const bf16 *)g.B;
  p.ldb = B_KC ? g.b_rs : g.b_cs;
  p.C = g.C;
  p.ldc = g.ldc;
  p.bias = (const bf16 *)g.bias;
  p.residual = (const bf16 *)g.residual;
  p.tiles_m = (int)ceil_div(g.M, BM);
  p.tiles_n = (int)ceil_div(g.N, BN);
  constexpr int lds_bytes = 2 * (BM + BN) * ROWB;
  auto kern = gemm_mfma_kernel<BM, BN, A_KC, B_KC, EPI>;
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            lds_bytes) != hipSuccess)
      return fail(TM_ELAUNCH, "gemm_mfma: cannot reserve %d bytes of LDS", lds_bytes);
    attr_set = true;
  }
  const int64_t nblk = (int64_t)p.tiles_m * p.tiles_n;
  if (nblk > 0x7fffffff) return fail(TM_ESIZE, "gemm_mfma: too many tiles");
  static const std::string name = "gemm_mfma_kernel<" + std::to_string(BM) + "," + std::to_string(BN) + "," +
                                  (A_KC ? "true" : "false") + "," + (B_KC ? "true" : "false") + "," +
                                  std::to_string(EPI) + ">";
  g_last_kernel = name.c_str();
  kern<<<dim3((unsigned)nblk), 256, lds_bytes, s>>>(p);
  return check_launch("gemm_mfma");
}

// Picks the block tile: fewest passes over the chip's 256 compute units, larger tiles preferred
// (they read each operand element from LDS fewer times per flop).
static void pick_tile(int64_t M, int64_t N, int &bm, int &bn) {
  const int cand[4][2] = {{256, 256}, {256, 128}, {128, 256}, {128, 128}};
  const double speed[4] = {1.0, 0.9, 0.9, 0.75};
  double best = 1e300;
  for (int c = 0; c < 4; ++c) {
    const int64_t nb = ceil_div(M, cand[c][0]) * ceil_div(N, cand[c][1]);
    const double passes = (double)ceil_div(nb, 256);
    const double cost = passes * cand[c][0] * cand[c][1] / speed[c];
    if (cost < best) {
      best = cost;
      bm = cand[c][0];
      bn = cand[c][1];
    }
  }
}

template <bool A_KC, bool B_KC, int EPI> static int launch_layout(const GemmArgs &g, hipStream_t s) {
  int bm = 128, bn = 128;
  pick_tile(g.M, g.N, bm, bn);
  if (bm == 256 && bn == 256) return launch_tile<256, 256, A_KC, B_KC, EPI>(g, s);
  if (bm == 256 && bn == 128) return launch_tile<256, 128, A_KC, B_KC, EPI>(g, s);
  if (bm == 128 && bn == 256) return launch_tile<128, 256, A_KC, B_KC, EPI>(g, s);
  return launch_tile<128, 128, A_KC, B_KC, EPI>(g, s);
}

int gemm_mfma(const GemmArgs &g, hipStream_t s) {
  const bool akc = g.a_cs == 1, bkc = g.b_cs == 1;
  if (!g.accumulate_f32 && akc && bkc) return launch_layout<true, true, 0>(g, s);    // y = x W^T
  if (!g.accumulate_f32 && akc && !bkc) return launch_layout<true, false, 0>(g, s);  // dx = dy W
  if (g.accumulate_f32 && !akc && !bkc) return launch_layout<false, false, 1>(g, s); // dW += dy^T x
  return fail(TM_EINVAL, "gemm_mfma: operand layout not instantiated");
}

}  // namespace tmk

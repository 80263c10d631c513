// Flash-style causal attention on the CDNA4 matrix cores (bf16 in, fp32 accumulate).
//
// The s x s score matrix is never stored: a block walks key/value tiles of 64 rows, keeps running
// row maxima and sums in registers (online softmax) and accumulates the output in MFMA accumulators.
//
// Layout trick used throughout: the products are formed TRANSPOSED (S^T = K Q^T, O^T = V^T P^T, ...),
// so that in every 32x32 accumulator tile the lane index is the row that owns the softmax
// statistics (a query row in the forward and dQ kernels, a key row in the dK/dV kernel) and the 16
// accumulator registers run along the reduction axis of the NEXT product.  A lane's 8 consecutive
// accumulator registers are then exactly the 8 reduction-axis values the next MFMA expects from it,
// under a fixed permutation of that axis (slot (half h, e) <-> offset 8*(e/4) + 4*h + e%4) which the
// other operand follows by reading two 8-byte pieces from an LDS tile stored transposed.
// Row statistics therefore need one cross-half exchange per tile and no row-wise shuffles.
//
// Gradients are accumulated without atomics: dK/dV by a block that owns 128 key rows and loops over
// the query heads of its group and all later query tiles; dQ by a block that owns 128 query rows.
#include <math.h>

#include "attn.h"

namespace tmk {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int TILE = 64;        // rows of a staged tile (keys in fwd/dQ, queries in dK/dV)
constexpr int TRB = TILE * 2;   // bytes per row of a transposed tile [D][TILE]
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ int swz8(int r) { return (r ^ (r >> 3)) & 7; }

struct FlashParams {
  const bf16 *qkv;
  const bf16 *dctx;
  bf16 *ctx;
  bf16 *dqkv;
  float *lse;
  const float *lse_in;
  const float *dvec;
  int seq, batch, nq, nkv, row;  // row = (nq + 2 nkv) * D
  float scale;                   // 1 / sqrt(D)
};

// ---- staging of a [TILE][D] tile from global memory --------------------------------------------
// src points at (row 0, column 0) of the tile; consecutive rows are `stride` elements apart.
// Rows >= rows_valid are filled with zeros.  RM: row-major copy; TR: transposed copy [D][TILE].
template <int D, bool RM, bool TR>
__device__ __forceinline__ void stage_tile(const bf16 *src, int64_t stride, int rows_valid, char *rm, char *tr) {
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int RPP = 256 / CPR;           // rows per pass
  const int c = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
#pragma unroll
  for (int i = 0; i < TILE / RPP; ++i) {
    const int r = r0 + i * RPP;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < rows_valid) v = *reinterpret_cast<const u32x4 *>(src + (int64_t)r * stride + c * 8);
    if (RM) *reinterpret_cast<u32x4 *>(rm + r * (D * 2) + ((c ^ swz8(r)) << 4)) = v;
    if (TR) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int dcol = c * 8 + e;
        const uint16_t h = (uint16_t)((e & 1) ? (v[e >> 1] >> 16) : (v[e >> 1] & 0xffffu));
        *reinterpret_cast<uint16_t *>(tr + dcol * TRB + (((r >> 3) ^ swz8(dcol)) << 4) + ((r & 7) << 1)) = h;
      }
    }
  }
}

// A-operand fragment from a row-major tile: 8 consecutive reduction elements of row r
template <int D> __device__ __forceinline__ bf16x8 frag_rm(const char *rm, int r, int ks, int hh) {
  return *reinterpret_cast<const bf16x8 *>(rm + r * (D * 2) + ((((2 * ks + hh)) ^ swz8(r)) << 4));
}
// A-operand fragment from a transposed tile: row dcol, permuted reduction slots of step kk
__device__ __forceinline__ bf16x8 frag_tr(const char *tr, int dcol, int kk, int hh) {
  const char *base = tr + dcol * TRB + (hh << 3);
  const int sw = swz8(dcol);
  union { u32x2 u[2]; bf16x8 v; } x;
  x.u[0] = *reinterpret_cast<const u32x2 *>(base + (((2 * kk) ^ sw) << 4));
  x.u[1] = *reinterpret_cast<const u32x2 *>(base + (((2 * kk + 1) ^ sw) << 4));
  return x.v;
}
// B-operand fragments straight from global memory: 8 consecutive elements of row (l32) per step
template <int D>
__device__ __forceinline__ void load_row_frags(const bf16 *rowptr, bool valid, int hh, bf16x8 (&f)[D / 16]) {
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    union { u32x4 u; bf16x8 v; } x;
    x.u = u32x4{0u, 0u, 0u, 0u};
    if (valid) x.u = *reinterpret_cast<const u32x4 *>(rowptr + ks * 16 + hh * 8);
    f[ks] = x.v;
  }
}
// 8 accumulator registers (v0..v0+7) -> bf16 B-operand fragment
__device__ __forceinline__ bf16x8 pack8(const f32x16 &a, int v0) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)a[v0 + e];
  return r;
}
// offset along the accumulator-row axis of register v in a 32x32 tile
__device__ __forceinline__ int acc_row(int v, int hh) { return 8 * (v >> 2) + 4 * hh + (v & 3); }

// writes O^T-style accumulators (rows = head-dim slots, lane = token row) to out[token][col0 + d]
template <int D>
__device__ __forceinline__ void store_transposed(const f32x16 (&acc)[D / 32], float mul, bf16 *dst_row, int hh) {
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)(acc[dt][q4 * 4 + e] * mul);
      *reinterpret_cast<bf16x4 *>(dst_row + dt * 32 + 8 * q4 + 4 * hh) = o;
    }
}

// =================================================================================================
// forward: block = 128 query rows of one (batch entry, query head); wave = 32 query rows
// =================================================================================================
template <int D>
__global__ __launch_bounds__(256) void flash_fwd_kernel(const FlashParams p) {
  __shared__ __align__(16) char k_rm[TILE * D * 2];
  __shared__ __align__(16) char v_tr[D * TRB];
  const int qt = gridDim.x - 1 - blockIdx.x, g = blockIdx.y, n = blockIdx.z;
  const int kap = g / (p.nq / p.nkv);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, hh = lane >> 5;
  const int q0w = qt * 128 + wave * 32;
  const int q = q0w + l32;
  const bool qvalid = q < p.seq;
  const int64_t tstride = (int64_t)p.batch * p.row;  // elements between consecutive positions
  const bf16 *base = p.qkv + (int64_t)n * p.row;
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;

  bf16x8 qf[D / 16];
  load_row_frags<D>(base + (int64_t)q * tstride + g * D, qvalid, hh, qf);

  f32x16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float sc2 = p.scale * kLog2e;

  const int kv_end = (qt * 128 + 128 < p.seq) ? qt * 128 + 128 : p.seq;
  const int ntile = (kv_end + TILE - 1) / TILE;
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * TILE;
    __syncthreads();
    stage_tile<D, true, false>(base + (int64_t)j0 * tstride + koff, tstride, p.seq - j0, k_rm, nullptr);
    stage_tile<D, false, true>(base + (int64_t)j0 * tstride + voff, tstride, p.seq - j0, nullptr, v_tr);
    __syncthreads();
    if (j0 > q0w + 31) continue;  // every key of this tile lies after every query row of the wave

    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm<D>(k_rm, t * 32 + l32, ks, hh), qf[ks], s[t], 0, 0, 0);
    }
    const bool diag = j0 + TILE - 1 > q0w;  // some key index may exceed some query index
    float mx = m;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float x = s[t][v] * sc2;
        if (diag && j0 + t * 32 + acc_row(v, hh) > q) x = -INFINITY;
        s[t][v] = x;
        mx = fmaxf(mx, x);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float alpha = __builtin_amdgcn_exp2f(m - mx);
    m = mx;
    float ps = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float e = __builtin_amdgcn_exp2f(s[t][v] - mx);
        s[t][v] = e;
        ps += e;
      }
    l = l * alpha + ps;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
#pragma unroll
    for (int kk = 0; kk < TILE / 16; ++kk) {
      const bf16x8 pf = pack8(s[kk >> 1], 8 * (kk & 1));
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(v_tr, dt * 32 + l32, kk, hh), pf, o[dt], 0, 0, 0);
    }
  }
  l += __shfl_xor(l, 32, 64);
  if (qvalid) {
    const int64_t trow = (int64_t)q * p.batch + n;
    store_transposed<D>(o, 1.f / l, p.ctx + trow * (p.nq * D) + g * D, hh);
    if (hh == 0) p.lse[((int64_t)n * p.nq + g) * p.seq + q] = (m + log2f(l)) * 0.6931471805599453f;
  }
}

// =================================================================================================
// dQ: same walk as the forward pass; dQ^T += K^T dS^T
// =================================================================================================
template <int D>
__global__ __launch_bounds__(256) void flash_bwd_dq_kernel(const FlashParams p) {
  __shared__ __align__(16) char k_rm[TILE * D * 2];
  __shared__ __align__(16) char v_rm[TILE * D * 2];
  __shared__ __align__(16) char k_tr[D * TRB];
  const int qt = gridDim.x - 1 - blockIdx.x, g = blockIdx.y, n = blockIdx.z;
  const int kap = g / (p.nq / p.nkv);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, hh = lane >> 5;
  const int q0w = qt * 128 + wave * 32;
  const int q = q0w + l32;
  const bool qvalid = q < p.seq;
  const int64_t tstride = (int64_t)p.batch * p.row;
  const bf16 *base = p.qkv + (int64_t)n * p.row;
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;
  const int64_t cstride = (int64_t)p.batch * p.nq * D;

  bf16x8 qf[D / 16], dof[D / 16];
  load_row_frags<D>(base + (int64_t)q * tstride + g * D, qvalid, hh, qf);
  load_row_frags<D>(p.dctx + (int64_t)n * p.nq * D + (int64_t)q * cstride + g * D, qvalid, hh, dof);
  const int64_t si = ((int64_t)n * p.nq + g) * p.seq + q;
  const float lse2 = qvalid ? p.lse_in[si] * kLog2e : 0.f;
  const float dq_d = qvalid ? p.dvec[si] : 0.f;

  f32x16 acc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.f;
  const float sc2 = p.scale * kLog2e;

  const int kv_end = (qt * 128 + 128 < p.seq) ? qt * 128 + 128 : p.seq;
  const int ntile = (kv_end + TILE - 1) / TILE;
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * TILE;
    __syncthreads();
    stage_tile<D, true, true>(base + (int64_t)j0 * tstride + koff, tstride, p.seq - j0, k_rm, k_tr);
    stage_tile<D, true, false>(base + (int64_t)j0 * tstride + voff, tstride, p.seq - j0, v_rm, nullptr);
    __syncthreads();
    if (j0 > q0w + 31) continue;

    const bool diag = j0 + TILE - 1 > q0w;
    f32x16 ds[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = dp[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm<D>(k_rm, t * 32 + l32, ks, hh), qf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm<D>(v_rm, t * 32 + l32, ks, hh), dof[ks], dp, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float pr = __builtin_amdgcn_exp2f(s[v] * sc2 - lse2);
        if (diag && j0 + t * 32 + acc_row(v, hh) > q) pr = 0.f;
        ds[t][v] = pr * (dp[v] - dq_d);
      }
    }
#pragma unroll
    for (int kk = 0; kk < TILE / 16; ++kk) {
      const bf16x8 df = pack8(ds[kk >> 1], 8 * (kk & 1));
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(k_tr, dt * 32 + l32, kk, hh), df, acc[dt], 0, 0, 0);
    }
  }
  if (qvalid) store_transposed<D>(acc, p.scale, p.dqkv + ((int64_t)q * p.batch + n) * p.row + g * D, hh);
}

// =================================================================================================
// dK, dV: block = 128 key rows of one (batch entry, kv head); wave = 32 key rows; loops over the
// query heads of the group and over query tiles of 64 rows from the diagonal to the end
// =================================================================================================
template <int D>
__global__ __launch_bounds__(256) void flash_bwd_dkv_kernel(const FlashParams p) {
  extern __shared__ __align__(16) char smem[];  // 4 tiles + 2 * TILE floats (above the static 64 KB limit)
  char *q_rm = smem, *do_rm = smem + TILE * D * 2, *q_tr = smem + 2 * TILE * D * 2, *do_tr = q_tr + D * TRB;
  float *lse_s = reinterpret_cast<float *>(do_tr + D * TRB), *dv_s = lse_s + TILE;
  const int kt = blockIdx.x, kap = blockIdx.y, n = blockIdx.z;
  const int group = p.nq / p.nkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, hh = lane >> 5;
  const int j0w = kt * 128 + wave * 32;
  const int j = j0w + l32;
  const bool jvalid = j < p.seq;
  const int64_t tstride = (int64_t)p.batch * p.row;
  const bf16 *base = p.qkv + (int64_t)n * p.row;
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;
  const int64_t cstride = (int64_t)p.batch * p.nq * D;

  bf16x8 kf[D / 16], vf[D / 16];
  load_row_frags<D>(base + (int64_t)j * tstride + koff, jvalid, hh, kf);
  load_row_frags<D>(base + (int64_t)j * tstride + voff, jvalid, hh, vf);

  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dk[dt][v] = dv[dt][v] = 0.f;
  const float sc2 = p.scale * kLog2e;

  const int it_begin = (kt * 128) / TILE;
  const int it_end = (p.seq + TILE - 1) / TILE;
  for (int gi = 0; gi < group; ++gi) {
    const int g = kap * group + gi;
    const float *lse_g = p.lse_in + ((int64_t)n * p.nq + g) * p.seq;
    const float *dvec_g = p.dvec + ((int64_t)n * p.nq + g) * p.seq;
    for (int it = it_begin; it < it_end; ++it) {
      const int i0 = it * TILE;
      __syncthreads();
      stage_tile<D, true, true>(base + (int64_t)i0 * tstride + g * D, tstride, p.seq - i0, q_rm, q_tr);
      stage_tile<D, true, true>(p.dctx + (int64_t)n * p.nq * D + (int64_t)i0 * cstride + g * D, cstride, p.seq - i0,
                                do_rm, do_tr);
      if (threadIdx.x < TILE) {
        const int i = i0 + threadIdx.x;
        lse_s[threadIdx.x] = i < p.seq ? lse_g[i] * kLog2e : 0.f;
        dv_s[threadIdx.x] = i < p.seq ? dvec_g[i] : 0.f;
      }
      __syncthreads();
      if (i0 + TILE - 1 < j0w) continue;  // every query of this tile lies before every key row of the wave

      const bool diag = i0 < j0w + 31;  // some query index may be below some key index
      f32x16 pr[2], ds[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16 s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = dp[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm<D>(q_rm, t * 32 + l32, ks, hh), kf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rm<D>(do_rm, t * 32 + l32, ks, hh), vf[ks], dp, 0, 0, 0);
        }
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int ib = t * 32 + 8 * q4 + 4 * hh;  // four consecutive query rows of this lane
          const f32x4 l4 = *reinterpret_cast<const f32x4 *>(lse_s + ib);
          const f32x4 d4 = *reinterpret_cast<const f32x4 *>(dv_s + ib);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int v = q4 * 4 + e;
            float x = __builtin_amdgcn_exp2f(s[v] * sc2 - l4[e]);
            if (diag && i0 + ib + e < j) x = 0.f;
            pr[t][v] = x;
            ds[t][v] = x * (dp[v] - d4[e]);
          }
        }
      }
#pragma unroll
      for (int kk = 0; kk < TILE / 16; ++kk) {
        const bf16x8 pf = pack8(pr[kk >> 1], 8 * (kk & 1));
        const bf16x8 df = pack8(ds[kk >> 1], 8 * (kk & 1));
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(do_tr, dt * 32 + l32, kk, hh), pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(q_tr, dt * 32 + l32, kk, hh), df, dk[dt], 0, 0, 0);
        }
      }
    }
  }
  if (jvalid) {
    bf16 *out = p.dqkv + ((int64_t)j * p.batch + n) * p.row;
    store_transposed<D>(dk, p.scale, out + koff, hh);
    store_transposed<D>(dv, 1.f, out + voff, hh);
  }
}

bool attn_mfma_supported(int dtype, int64_t d) { return dtype == TM_DTYPE_BF16 && (d == 128 || d == 64); }

static FlashParams make_params(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d) {
  FlashParams p = {};
  p.seq = (int)seq;
  p.batch = (int)batch;
  p.nq = (int)nq;
  p.nkv = (int)nkv;
  p.row = (int)((nq + 2 * nkv) * d);
  p.scale = (float)(1.0 / sqrt((double)d));
  return p;
}

int attn_fwd_mfma_launch(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *qkv, void *ctx,
                         float *lse, hipStream_t s) {
  FlashParams p = make_params(seq, batch, nq, nkv, d);
  p.qkv = (const bf16 *)qkv;
  p.ctx = (bf16 *)ctx;
  p.lse = lse;
  dim3 grid((unsigned)ceil_div(seq, 128), (unsigned)nq, (unsigned)batch);
  g_last_kernel = "flash_fwd_kernel";
  if (d == 128)
    flash_fwd_kernel<128><<<grid, 256, 0, s>>>(p);
  else
    flash_fwd_kernel<64><<<grid, 256, 0, s>>>(p);
  return check_launch("flash_fwd");
}

int attn_bwd_mfma_launch(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *qkv,
                         const void *dctx, const float *lse, const float *dvec, void *dqkv, hipStream_t s) {
  FlashParams p = make_params(seq, batch, nq, nkv, d);
  p.qkv = (const bf16 *)qkv;
  p.dctx = (const bf16 *)dctx;
  p.lse_in = lse;
  p.dvec = dvec;
  p.dqkv = (bf16 *)dqkv;
  dim3 gq((unsigned)ceil_div(seq, 128), (unsigned)nq, (unsigned)batch);
  dim3 gk((unsigned)ceil_div(seq, 128), (unsigned)nkv, (unsigned)batch);
  const int lds = (int)(4 * TILE * d * 2 + 2 * TILE * sizeof(float));
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(flash_bwd_dkv_kernel<128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TILE * 128 * 2 + 2 * TILE * 4) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void *>(flash_bwd_dkv_kernel<64>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TILE * 64 * 2 + 2 * TILE * 4) != hipSuccess)
      return fail(TM_ELAUNCH, "flash_bwd: cannot reserve LDS");
    attr_set = true;
  }
  g_last_kernel = "flash_bwd_dq_kernel+flash_bwd_dkv_kernel";
  if (d == 128) {
    flash_bwd_dq_kernel<128><<<gq, 256, 0, s>>>(p);
    flash_bwd_dkv_kernel<128><<<gk, 256, lds, s>>>(p);
  } else {
    flash_bwd_dq_kernel<64><<<gq, 256, 0, s>>>(p);
    flash_bwd_dkv_kernel<64><<<gk, 256, lds, s>>>(p);
  }
  return check_launch("flash_bwd");
}

}  // namespace tmk

// LayerNorm / RMSNorm forward and backward, column reductions (bias and gain gradients).
// HBM-bound kernels: 16-byte accesses, fp32 arithmetic, wavefront shuffles for row sums.
#include "common.h"
#include "../../include/tm_ops.h"

namespace tmk {

constexpr int kNormThreads = 512;
constexpr int kNormMaxChunks = 4;  // 16-byte chunks per thread: hidden <= 512 * 4 * Vec::N

// ---------------------------------------------------------------------------------------
// forward: one block per token row; the row stays in registers between the passes.
// Every access goes through a per-row buffer descriptor (chunks past the row read as zero).
// ---------------------------------------------------------------------------------------
template <typename T, int KIND, int NCH>
__global__ __launch_bounds__(kNormThreads) void norm_fwd_kernel(
    const T *__restrict__ x, const T *__restrict__ gain, const T *__restrict__ offset, T *__restrict__ out,
    float *__restrict__ mean_out, float *__restrict__ rstd_out, int h, float eps) {
  constexpr int VN = Vec<T>::N;
  __shared__ float red[2 * kNormThreads / kWave];
  const int64_t row = blockIdx.x;
  const uint32_t row_bytes = (uint32_t)h * sizeof(T);
  const rsrc_t rx = make_rsrc(x + row * h, row_bytes), ro = make_rsrc(out + row * h, row_bytes);
  const rsrc_t rg = make_rsrc(gain, row_bytes), rf = make_rsrc(KIND == TM_NORM_LAYERNORM ? offset : gain, row_bytes);
  const int nchunk = h / VN;

  float vals[NCH][VN];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) buf_load_vec<T>(rx, (threadIdx.x + c * kNormThreads) * 16u, vals[c]);
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      s1 += vals[c][i];
      s2 += vals[c][i] * vals[c][i];
    }
  block_sum2<kNormThreads>(s1, s2, red);
  float mu = 0.f, rstd;
  if (KIND == TM_NORM_LAYERNORM) {
    mu = s1 / h;
    float q = 0.f, dummy = 0.f;  // second pass over registers: sum of squared deviations
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const bool live = threadIdx.x + c * kNormThreads < nchunk;
#pragma unroll
      for (int i = 0; i < VN; ++i) {
        const float dlt = vals[c][i] - mu;
        q += live ? dlt * dlt : 0.f;
      }
    }
    block_sum2<kNormThreads>(q, dummy, red);
    rstd = 1.0f / sqrtf(q / h + eps);
  } else {
    rstd = 1.0f / sqrtf(s2 / h + eps);
  }
  if (threadIdx.x == 0) {
    if (mean_out) mean_out[row] = mu;
    rstd_out[row] = rstd;
  }
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const uint32_t off = (threadIdx.x + c * kNormThreads) * 16u;
    float g[VN], o[VN], r[VN];
    buf_load_vec<T>(rg, off, g);
    if (KIND == TM_NORM_LAYERNORM) buf_load_vec<T>(rf, off, o);
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      const float xh = (vals[c][i] - mu) * rstd;
      r[i] = (KIND == TM_NORM_LAYERNORM) ? xh * g[i] + o[i] : xh * g[i];
    }
    buf_store_vec<T>(ro, off, r);
  }
}

// ---------------------------------------------------------------------------------------
// backward: block b handles rows b, b+G, ...; each thread keeps the gain/offset gradient of
// its own columns in registers and writes one partial row per block at the end.
// partial layout: [G][3][h] fp32 (gain partials, offset partials, and with XSUM the column sums of the
// stored dx: the gradient of the bias of the linear map that produced x's residual input, which would
// otherwise cost one more pass over dx)
// ---------------------------------------------------------------------------------------
template <typename T, int KIND, int NCH, bool XSUM>
__global__ __launch_bounds__(kNormThreads) void norm_bwd_kernel(
    const T *__restrict__ dout, const T *__restrict__ x, const float *__restrict__ mean,
    const float *__restrict__ rstd, const T *__restrict__ gain, const T *dres, T *dx,
    float *__restrict__ partial, int64_t rows, int h) {
  constexpr int VN = Vec<T>::N;
  __shared__ float red[2 * kNormThreads / kWave];
  const uint32_t row_bytes = (uint32_t)h * sizeof(T);
  const rsrc_t rg = make_rsrc(gain, row_bytes);
  float gacc[NCH][VN], oacc[NCH][VN], gn[NCH][VN], xacc[XSUM ? NCH : 1][VN];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    buf_load_vec<T>(rg, (threadIdx.x + c * kNormThreads) * 16u, gn[c]);
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      gacc[c][i] = oacc[c][i] = 0.f;
      if (XSUM) xacc[c][i] = 0.f;
    }
  }
  // The loads of a block's NEXT row are in flight while it reduces and stores the current one (the raw 16-byte
  // chunks wait in registers): without that a block spends most of a row's time waiting for its three loads.
  typedef uint32_t raw4 __attribute__((ext_vector_type(4)));
  raw4 nw[NCH], nx[NCH], nr[NCH];
  auto fetch = [&](int64_t row) {
    const rsrc_t rd = make_rsrc(dout + row * h, row_bytes), rx = make_rsrc(x + row * h, row_bytes);
    const rsrc_t rr = make_rsrc(dres ? dres + row * h : dout, dres ? row_bytes : 0u);  // no residual: reads zeros
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const uint32_t off = (threadIdx.x + c * kNormThreads) * 16u;
      nw[c] = __builtin_bit_cast(raw4, __builtin_amdgcn_raw_buffer_load_b128(rd, off, 0, 0));
      nx[c] = __builtin_bit_cast(raw4, __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0));
      nr[c] = __builtin_bit_cast(raw4, __builtin_amdgcn_raw_buffer_load_b128(rr, off, 0, 0));
    }
  };
  auto unpack = [](raw4 raw, float (&out)[VN]) {
    union { raw4 r; Vec<T> v; } u;
    u.r = raw;
#pragma unroll
    for (int i = 0; i < VN; ++i) out[i] = to_f32(u.v.v[i]);
  };
  if ((int64_t)blockIdx.x < rows) fetch(blockIdx.x);
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const rsrc_t ro = make_rsrc(dx + row * h, row_bytes);
    const float mu = (KIND == TM_NORM_LAYERNORM) ? mean[row] : 0.f;
    const float rs = rstd[row];
    float w[NCH][VN], xh[NCH][VN], res[NCH][VN];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      unpack(nw[c], w[c]);
      unpack(nx[c], xh[c]);
      unpack(nr[c], res[c]);
    }
    if (row + gridDim.x < rows) fetch(row + gridDim.x);
    const int nchunk = h / VN;
    float sw = 0.f, swx = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const bool live = threadIdx.x + c * kNormThreads < nchunk;  // x reads as 0 past the row: xhat would be -mu*rs
#pragma unroll
      for (int i = 0; i < VN; ++i) {
        const float d = w[c][i];
        const float xv = live ? (xh[c][i] - mu) * rs : 0.f;
        xh[c][i] = xv;
        w[c][i] = d * gn[c][i];
        gacc[c][i] += d * xv;
        oacc[c][i] += d;
        sw += w[c][i];
        swx += w[c][i] * xv;
      }
    }
    block_sum2<kNormThreads>(sw, swx, red);
    const float mw = (KIND == TM_NORM_LAYERNORM) ? sw / h : 0.f;
    const float mwx = swx / h;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
#pragma unroll
      for (int i = 0; i < VN; ++i) {
        res[c][i] += (w[c][i] - mw - xh[c][i] * mwx) * rs;
        if (XSUM) xacc[c][i] += to_f32(from_f32<T>(res[c][i]));  // the value as stored
      }
      buf_store_vec<T>(ro, (threadIdx.x + c * kNormThreads) * 16u, res[c]);
    }
  }
  const rsrc_t rp = make_rsrc(partial + (int64_t)blockIdx.x * 3 * h, (uint32_t)h * 4u);
  const rsrc_t rq = make_rsrc(partial + (int64_t)blockIdx.x * 3 * h + h, (uint32_t)h * 4u);
  const rsrc_t rz = make_rsrc(partial + (int64_t)blockIdx.x * 3 * h + 2 * h, (uint32_t)h * 4u);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const uint32_t col = (threadIdx.x + c * kNormThreads) * VN;
#pragma unroll
    for (int v4 = 0; v4 < VN / 4; ++v4) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = gacc[c][v4 * 4 + i];
        b[i] = oacc[c][v4 * 4 + i];
      }
      buf_store_vec<float>(rp, (col + v4 * 4) * 4u, a);
      buf_store_vec<float>(rq, (col + v4 * 4) * 4u, b);
      if (XSUM) {
        float z[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) z[i] = xacc[c][v4 * 4 + i];
        buf_store_vec<float>(rz, (col + v4 * 4) * 4u, z);
      }
    }
  }
}

// the three column reductions of the norm's backward pass in one launch: slice s of the partial rows goes to outs[s]
// (NULL: skipped); same summation order as reduce_partials_kernel
struct ReduceOuts {
  float *out[3];
};
__global__ __launch_bounds__(256) void reduce_partials3_kernel(const float *__restrict__ partial, int R, int h, ReduceOuts outs,
                                                               int accumulate) {
  __shared__ float sm[4][64];
  const int lane = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int per_slice = (h + 63) / 64;
  const int slice = blockIdx.x / per_slice, c = (blockIdx.x % per_slice) * 64 + lane;
  float *out = outs.out[slice];
  if (!out) return;  // uniform over the block
  const int64_t ld = 3 * (int64_t)h;
  const float *src = partial + (int64_t)slice * h;
  float s = 0.f;
  if (c < h) {
    int r = ry;
    for (; r + 12 < R; r += 16) {
      const float a0 = src[(int64_t)r * ld + c], a1 = src[(int64_t)(r + 4) * ld + c];
      const float a2 = src[(int64_t)(r + 8) * ld + c], a3 = src[(int64_t)(r + 12) * ld + c];
      s += a0;
      s += a1;
      s += a2;
      s += a3;
    }
    for (; r < R; r += 4) s += src[(int64_t)r * ld + c];
  }
  sm[ry][lane] = s;
  __syncthreads();
  if (ry == 0 && c < h) {
    const float t = ((sm[0][lane] + sm[1][lane]) + sm[2][lane]) + sm[3][lane];
    out[c] = accumulate ? out[c] + t : t;
  }
}

// out[c] (+)= sum_{r<R} partial[r*ld + c].  Block = 64 columns x 4 row lanes; lane y adds rows
// y, y+4, ... in ascending order, then the four lane sums are added in lane order: a fixed order.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partial, int R, int64_t ld,
                                                              int n, float *__restrict__ out, int accumulate) {
  __shared__ float sm[4][64];
  const int lane = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (c < n) {
    int r = ry;
    for (; r + 12 < R; r += 16) {  // four independent loads in flight per trip
      const float a0 = partial[(int64_t)r * ld + c], a1 = partial[(int64_t)(r + 4) * ld + c];
      const float a2 = partial[(int64_t)(r + 8) * ld + c], a3 = partial[(int64_t)(r + 12) * ld + c];
      s += a0;
      s += a1;
      s += a2;
      s += a3;
    }
    for (; r < R; r += 4) s += partial[(int64_t)r * ld + c];
  }
  sm[ry][lane] = s;
  __syncthreads();
  if (ry == 0 && c < n) {
    const float t = ((sm[0][lane] + sm[1][lane]) + sm[2][lane]) + sm[3][lane];
    out[c] = accumulate ? out[c] + t : t;
  }
}

// ---------------------------------------------------------------------------------------
// column sums of dy[T,N] (bias gradients): grid (column groups, row groups) -> partial[R][N]
// ---------------------------------------------------------------------------------------
constexpr int kColLanes = 64, kColRowsPerBlock = 4;

template <typename T>
__global__ __launch_bounds__(kColLanes *kColRowsPerBlock) void colsum_partial_kernel(
    const T *__restrict__ dy, float *__restrict__ partial, int64_t rows, int n, int rows_per_group) {
  constexpr int VN = Vec<T>::N;
  __shared__ float sm[kColRowsPerBlock][kColLanes * VN];
  const int lane = threadIdx.x % kColLanes, ry = threadIdx.x / kColLanes;
  const int col = (blockIdx.x * kColLanes + lane) * VN;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_group;
  const int64_t r1 = (r0 + rows_per_group < rows) ? r0 + rows_per_group : rows;
  float acc[VN];
#pragma unroll
  for (int i = 0; i < VN; ++i) acc[i] = 0.f;
  if (col < n) {
    for (int64_t r = r0 + ry; r < r1; r += kColRowsPerBlock) {
      float v[VN];
      load_vec<T>(dy + r * n + col, v);
#pragma unroll
      for (int i = 0; i < VN; ++i) acc[i] += v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < VN; ++i) sm[ry][lane * VN + i] = acc[i];
  __syncthreads();
  if (ry == 0 && col < n) {
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < kColRowsPerBlock; ++k) s += sm[k][lane * VN + i];
      partial[(int64_t)blockIdx.y * n + col + i] = s;
    }
  }
}

static int norm_bwd_blocks(int64_t T) { return (int)(T < 256 ? T : 256); }
static int colsum_groups(int64_t T) { return (int)(T < 32 * kColRowsPerBlock ? ceil_div(T, kColRowsPerBlock) : 32); }

// chunks per thread, rounded up to an instantiated count
static int pick_nch(int h, int vn) {
  const int need = (int)ceil_div(h / vn, kNormThreads);
  const int opts[] = {1, 2, 3, 4, 6, 8};
  for (int o : opts)
    if (need <= o) return o;
  return -1;
}
#define TM_NCH_SWITCH(nch, CALL)                    \
  switch (nch) {                                    \
    case 1: { constexpr int NCH = 1; CALL; } break; \
    case 2: { constexpr int NCH = 2; CALL; } break; \
    case 3: { constexpr int NCH = 3; CALL; } break; \
    case 4: { constexpr int NCH = 4; CALL; } break; \
    case 6: { constexpr int NCH = 6; CALL; } break; \
    default: { constexpr int NCH = 8; CALL; } break; \
  }

template <typename T>
static int norm_fwd_t(int kind, int64_t rows, int h, float eps, const void *x, const void *gain, const void *offset,
                      void *out, float *mean, float *rstd, hipStream_t s) {
  const int nch = pick_nch(h, Vec<T>::N);
  g_last_kernel = "norm_fwd_kernel";
  if (kind == TM_NORM_LAYERNORM) {
    TM_NCH_SWITCH(nch, (norm_fwd_kernel<T, TM_NORM_LAYERNORM, NCH><<<dim3((unsigned)rows), kNormThreads, 0, s>>>(
                           (const T *)x, (const T *)gain, (const T *)offset, (T *)out, mean, rstd, h, eps)))
  } else {
    TM_NCH_SWITCH(nch, (norm_fwd_kernel<T, TM_NORM_RMSNORM, NCH><<<dim3((unsigned)rows), kNormThreads, 0, s>>>(
                           (const T *)x, (const T *)gain, nullptr, (T *)out, mean, rstd, h, eps)))
  }
  return check_launch("norm_fwd");
}

template <typename T, bool XSUM>
static int norm_bwd_t(int kind, int64_t rows, int h, const void *dout, const void *x, const float *mean,
                      const float *rstd, const void *gain, const void *dres, void *dx, float *partial, hipStream_t s) {
  const int G = norm_bwd_blocks(rows);
  const int nch = pick_nch(h, Vec<T>::N);
  g_last_kernel = "norm_bwd_kernel";
  if (kind == TM_NORM_LAYERNORM) {
    TM_NCH_SWITCH(nch, (norm_bwd_kernel<T, TM_NORM_LAYERNORM, NCH, XSUM><<<G, kNormThreads, 0, s>>>(
                           (const T *)dout, (const T *)x, mean, rstd, (const T *)gain, (const T *)dres, (T *)dx,
                           partial, rows, h)))
  } else {
    TM_NCH_SWITCH(nch, (norm_bwd_kernel<T, TM_NORM_RMSNORM, NCH, XSUM><<<G, kNormThreads, 0, s>>>(
                           (const T *)dout, (const T *)x, mean, rstd, (const T *)gain, (const T *)dres, (T *)dx,
                           partial, rows, h)))
  }
  return check_launch("norm_bwd");
}

}  // namespace tmk

using namespace tmk;

static int check_width(const char *what, int dtype, int64_t T, int64_t h) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "%s: unknown dtype %d", what, dtype);
  if (T <= 0 || h <= 0) return fail(TM_EINVAL, "%s: empty shape [%lld, %lld]", what, (long long)T, (long long)h);
  if (h % 8) return fail(TM_ESIZE, "%s: row width %lld is not a multiple of 8", what, (long long)h);
  if (T > 0x7fffffffLL / 8) return fail(TM_ESIZE, "%s: %lld rows exceed the supported range", what, (long long)T);
  return TM_OK;
}

extern "C" int64_t tm_op_reduce_scratch_bytes(int64_t T, int64_t width) {
  if (T <= 0 || width <= 0) return TM_EINVAL;
  const int64_t g1 = norm_bwd_blocks(T), g2 = colsum_groups(T);
  return (g1 > g2 ? g1 : g2) * width * (int64_t)sizeof(float);  // callers of the norm pass width = 3h
}

extern "C" int tm_op_norm_fwd(int dtype, int kind, int64_t T, int64_t h, double eps, const void *x, const void *gain,
                              const void *offset, void *out, float *mean, float *rstd, void *stream) {
  if (int e = check_width("norm_fwd", dtype, T, h)) return e;
  if (kind != TM_NORM_LAYERNORM && kind != TM_NORM_RMSNORM) return fail(TM_EINVAL, "norm_fwd: unknown kind %d", kind);
  if (!x || !gain || !out || !rstd || (kind == TM_NORM_LAYERNORM && (!offset || !mean)))
    return fail(TM_EINVAL, "norm_fwd: NULL pointer");
  const int64_t hmax = (int64_t)kNormThreads * kNormMaxChunks * (dtype == TM_DTYPE_BF16 ? 8 : 4);
  if (h > hmax) return fail(TM_ESIZE, "norm_fwd: width %lld above the limit %lld", (long long)h, (long long)hmax);
  hipStream_t s = (hipStream_t)stream;
  return dtype == TM_DTYPE_BF16
             ? norm_fwd_t<bf16>(kind, T, (int)h, (float)eps, x, gain, offset, out, mean, rstd, s)
             : norm_fwd_t<float>(kind, T, (int)h, (float)eps, x, gain, offset, out, mean, rstd, s);
}

static int norm_bwd_any(int dtype, int kind, int64_t T, int64_t h, const void *dout, const void *x, const float *mean,
                        const float *rstd, const void *gain, const void *dres, void *dx, float *dgain, float *doffset,
                        float *dx_colsum, void *scratch, int accumulate, void *stream) {
  if (int e = check_width("norm_bwd", dtype, T, h)) return e;
  if (kind != TM_NORM_LAYERNORM && kind != TM_NORM_RMSNORM) return fail(TM_EINVAL, "norm_bwd: unknown kind %d", kind);
  if (!dout || !x || !rstd || !gain || !dx || !dgain || !scratch || (kind == TM_NORM_LAYERNORM && (!mean || !doffset)))
    return fail(TM_EINVAL, "norm_bwd: NULL pointer");
  const int64_t hmax = (int64_t)kNormThreads * kNormMaxChunks * (dtype == TM_DTYPE_BF16 ? 8 : 4);
  if (h > hmax) return fail(TM_ESIZE, "norm_bwd: width %lld above the limit %lld", (long long)h, (long long)hmax);
  hipStream_t s = (hipStream_t)stream;
  float *partial = (float *)scratch;
  int e;
  if (dx_colsum)
    e = dtype == TM_DTYPE_BF16 ? norm_bwd_t<bf16, true>(kind, T, (int)h, dout, x, mean, rstd, gain, dres, dx, partial, s)
                               : norm_bwd_t<float, true>(kind, T, (int)h, dout, x, mean, rstd, gain, dres, dx, partial, s);
  else
    e = dtype == TM_DTYPE_BF16 ? norm_bwd_t<bf16, false>(kind, T, (int)h, dout, x, mean, rstd, gain, dres, dx, partial, s)
                               : norm_bwd_t<float, false>(kind, T, (int)h, dout, x, mean, rstd, gain, dres, dx, partial, s);
  if (e) return e;
  const int G = norm_bwd_blocks(T);
  ReduceOuts outs{{dgain, kind == TM_NORM_LAYERNORM ? doffset : nullptr, dx_colsum}};
  reduce_partials3_kernel<<<3 * (int)ceil_div(h, 64), 256, 0, s>>>(partial, G, (int)h, outs, accumulate);
  return check_launch("norm_bwd reduce");
}

extern "C" int tm_op_norm_bwd(int dtype, int kind, int64_t T, int64_t h, const void *dout, const void *x,
                              const float *mean, const float *rstd, const void *gain, const void *dres, void *dx,
                              float *dgain, float *doffset, void *scratch, int accumulate, void *stream) {
  return norm_bwd_any(dtype, kind, T, h, dout, x, mean, rstd, gain, dres, dx, dgain, doffset, nullptr, scratch, accumulate, stream);
}

extern "C" int tm_op_norm_bwd_colsum(int dtype, int kind, int64_t T, int64_t h, const void *dout, const void *x,
                                     const float *mean, const float *rstd, const void *gain, const void *dres, void *dx,
                                     float *dgain, float *doffset, float *dx_colsum, void *scratch, int accumulate,
                                     void *stream) {
  if (!dx_colsum) return fail(TM_EINVAL, "norm_bwd_colsum: NULL pointer");
  return norm_bwd_any(dtype, kind, T, h, dout, x, mean, rstd, gain, dres, dx, dgain, doffset, dx_colsum, scratch, accumulate, stream);
}

extern "C" int tm_op_bias_grad(int dtype, int64_t T, int64_t N, const void *dy, float *db, void *scratch,
                               int accumulate, void *stream) {
  if (int e = check_width("bias_grad", dtype, T, N)) return e;
  if (!dy || !db || !scratch) return fail(TM_EINVAL, "bias_grad: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  const int R = colsum_groups(T);
  const int rows_per_group = (int)ceil_div(T, R);
  float *partial = (float *)scratch;
  const int vn = dtype == TM_DTYPE_BF16 ? 8 : 4;
  g_last_kernel = "colsum_partial_kernel";
  dim3 grid((unsigned)ceil_div(N, (int64_t)kColLanes * vn), (unsigned)R);
  if (dtype == TM_DTYPE_BF16)
    colsum_partial_kernel<bf16><<<grid, kColLanes * kColRowsPerBlock, 0, s>>>((const bf16 *)dy, partial, T, (int)N,
                                                                              rows_per_group);
  else
    colsum_partial_kernel<float><<<grid, kColLanes * kColRowsPerBlock, 0, s>>>((const float *)dy, partial, T, (int)N,
                                                                               rows_per_group);
  reduce_partials_kernel<<<(int)ceil_div(N, 64), 256, 0, s>>>(partial, R, N, (int)N, db, accumulate);
  return check_launch("bias_grad");
}

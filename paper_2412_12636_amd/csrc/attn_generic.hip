// Causal attention without matrix cores: the fp32 stage dtype, and bf16 head sizes the MFMA
// kernels do not take.  One wavefront per query row (forward, dQ) or per key row (dK, dV); scores of
// the row live in LDS.  Summation orders are fixed, so results are bit-reproducible.
#include <math.h>

#include "attn.h"

namespace tmk {

// qkv row layout: [ Q heads (nq*d) | K heads (nkv*d) | V heads (nkv*d) ], token row t = pos*batch + n
struct AttnShape {
  int seq, batch, nq, nkv, d, row;  // row = (nq + 2 nkv) * d
  float scale;
};

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_generic(const T *__restrict__ qkv, T *__restrict__ ctx,
                                                      float *__restrict__ lse, AttnShape a) {
  extern __shared__ float sc[];  // seq scores
  const int i = blockIdx.x, g = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int kap = g / (a.nq / a.nkv);
  const T *q = qkv + ((int64_t)i * a.batch + n) * a.row + g * a.d;
  const int koff = a.nq * a.d + kap * a.d, voff = (a.nq + a.nkv) * a.d + kap * a.d;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) {
    const T *k = qkv + ((int64_t)j * a.batch + n) * a.row + koff;
    float s = 0.f;
    for (int e = 0; e < a.d; ++e) s = fmaf(to_f32(q[e]), to_f32(k[e]), s);
    s *= a.scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= i; j += 64) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.f / sum;
  for (int e = lane; e < a.d; e += 64) {
    float o = 0.f;
    for (int j = 0; j <= i; ++j) o = fmaf(sc[j], to_f32(qkv[((int64_t)j * a.batch + n) * a.row + voff + e]), o);
    ctx[((int64_t)i * a.batch + n) * (a.nq * a.d) + g * a.d + e] = from_f32<T>(o * inv);
  }
  if (lane == 0) lse[((int64_t)n * a.nq + g) * a.seq + i] = mx + logf(sum);
}

// dvec[n,g,i] = sum_e dctx[i,g,e] * ctx[i,g,e]
template <typename T>
__global__ __launch_bounds__(64) void attn_dvec_kernel(const T *__restrict__ ctx, const T *__restrict__ dctx,
                                                      float *__restrict__ dvec, AttnShape a) {
  const int i = blockIdx.x, g = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int64_t off = ((int64_t)i * a.batch + n) * (a.nq * a.d) + g * a.d;
  float s = 0.f;
  for (int e = lane; e < a.d; e += 64) s = fmaf(to_f32(ctx[off + e]), to_f32(dctx[off + e]), s);
  s = wave_sum(s);
  if (lane == 0) dvec[((int64_t)n * a.nq + g) * a.seq + i] = s;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_generic(const T *__restrict__ qkv, const T *__restrict__ dctx,
                                                         const float *__restrict__ lse,
                                                         const float *__restrict__ dvec, T *__restrict__ dqkv,
                                                         AttnShape a) {
  extern __shared__ float ds[];  // seq values of dS for this row
  const int i = blockIdx.x, g = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int kap = g / (a.nq / a.nkv);
  const int64_t trow = (int64_t)i * a.batch + n;
  const T *q = qkv + trow * a.row + g * a.d;
  const T *dc = dctx + trow * (a.nq * a.d) + g * a.d;
  const int koff = a.nq * a.d + kap * a.d, voff = (a.nq + a.nkv) * a.d + kap * a.d;
  const float l = lse[((int64_t)n * a.nq + g) * a.seq + i], D = dvec[((int64_t)n * a.nq + g) * a.seq + i];
  for (int j = lane; j <= i; j += 64) {
    const T *k = qkv + ((int64_t)j * a.batch + n) * a.row + koff;
    const T *v = qkv + ((int64_t)j * a.batch + n) * a.row + voff;
    float s = 0.f, dp = 0.f;
    for (int e = 0; e < a.d; ++e) {
      s = fmaf(to_f32(q[e]), to_f32(k[e]), s);
      dp = fmaf(to_f32(dc[e]), to_f32(v[e]), dp);
    }
    const float p = expf(s * a.scale - l);
    ds[j] = p * (dp - D);
  }
  __syncthreads();
  for (int e = lane; e < a.d; e += 64) {
    float o = 0.f;
    for (int j = 0; j <= i; ++j) o = fmaf(ds[j], to_f32(qkv[((int64_t)j * a.batch + n) * a.row + koff + e]), o);
    dqkv[trow * a.row + g * a.d + e] = from_f32<T>(o * a.scale);
  }
}

// one wavefront per (key row j, kv head, batch entry); loops over the query heads of the group
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_generic(const T *__restrict__ qkv, const T *__restrict__ dctx,
                                                          const float *__restrict__ lse,
                                                          const float *__restrict__ dvec, T *__restrict__ dqkv,
                                                          AttnShape a) {
  extern __shared__ float sm[];  // p[seq], ds[seq]
  float *pbuf = sm, *dsbuf = sm + a.seq;
  const int j = blockIdx.x, kap = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int group = a.nq / a.nkv;
  const int64_t jrow = (int64_t)j * a.batch + n;
  const int koff = a.nq * a.d + kap * a.d, voff = (a.nq + a.nkv) * a.d + kap * a.d;
  const T *k = qkv + jrow * a.row + koff;
  const T *v = qkv + jrow * a.row + voff;
  // up to 4 output columns per lane (d <= 256)
  float dk[4] = {0.f, 0.f, 0.f, 0.f}, dv[4] = {0.f, 0.f, 0.f, 0.f};
  for (int gi = 0; gi < group; ++gi) {
    const int g = kap * group + gi;
    __syncthreads();
    for (int i = j + lane; i < a.seq; i += 64) {
      const int64_t irow = (int64_t)i * a.batch + n;
      const T *q = qkv + irow * a.row + g * a.d;
      const T *dc = dctx + irow * (a.nq * a.d) + g * a.d;
      float s = 0.f, dp = 0.f;
      for (int e = 0; e < a.d; ++e) {
        s = fmaf(to_f32(q[e]), to_f32(k[e]), s);
        dp = fmaf(to_f32(dc[e]), to_f32(v[e]), dp);
      }
      const int64_t si = ((int64_t)n * a.nq + g) * a.seq + i;
      const float p = expf(s * a.scale - lse[si]);
      pbuf[i] = p;
      dsbuf[i] = p * (dp - dvec[si]);
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int e = lane + 64 * c;
      if (e < a.d) {
        for (int i = j; i < a.seq; ++i) {
          const int64_t irow = (int64_t)i * a.batch + n;
          dv[c] = fmaf(pbuf[i], to_f32(dctx[irow * (a.nq * a.d) + g * a.d + e]), dv[c]);
          dk[c] = fmaf(dsbuf[i], to_f32(qkv[irow * a.row + g * a.d + e]), dk[c]);
        }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int e = lane + 64 * c;
    if (e < a.d) {
      dqkv[jrow * a.row + koff + e] = from_f32<T>(dk[c] * a.scale);
      dqkv[jrow * a.row + voff + e] = from_f32<T>(dv[c]);
    }
  }
}

static AttnShape make_shape(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d) {
  AttnShape a;
  a.seq = (int)seq;
  a.batch = (int)batch;
  a.nq = (int)nq;
  a.nkv = (int)nkv;
  a.d = (int)d;
  a.row = (int)((nq + 2 * nkv) * d);
  a.scale = (float)(1.0 / sqrt((double)d));
  return a;
}

template <typename T>
static int fwd_t(const AttnShape &a, const void *qkv, void *ctx, float *lse, hipStream_t s) {
  dim3 grid(a.seq, a.nq, a.batch);
  g_last_kernel = "attn_fwd_generic";
  attn_fwd_generic<T><<<grid, 64, a.seq * sizeof(float), s>>>((const T *)qkv, (T *)ctx, lse, a);
  return check_launch("attn_fwd_generic");
}

template <typename T>
static int bwd_t(const AttnShape &a, const void *qkv, const void *dctx, const float *lse, const float *dvec,
                 void *dqkv, hipStream_t s) {
  g_last_kernel = "attn_bwd_generic";
  attn_bwd_dq_generic<T><<<dim3(a.seq, a.nq, a.batch), 64, a.seq * sizeof(float), s>>>(
      (const T *)qkv, (const T *)dctx, lse, dvec, (T *)dqkv, a);
  attn_bwd_dkv_generic<T><<<dim3(a.seq, a.nkv, a.batch), 64, 2 * a.seq * sizeof(float), s>>>(
      (const T *)qkv, (const T *)dctx, lse, dvec, (T *)dqkv, a);
  return check_launch("attn_bwd_generic");
}

int attn_generic_max_seq() { return 8192; }  // 2 * seq floats of LDS in the dK/dV kernel

int attn_fwd_generic_launch(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                            const void *qkv, void *ctx, float *lse, hipStream_t s) {
  const AttnShape a = make_shape(seq, batch, nq, nkv, d);
  return dtype == TM_DTYPE_BF16 ? fwd_t<bf16>(a, qkv, ctx, lse, s) : fwd_t<float>(a, qkv, ctx, lse, s);
}

int attn_dvec_launch(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *ctx,
                     const void *dctx, float *dvec, hipStream_t s) {
  const AttnShape a = make_shape(seq, batch, nq, nkv, d);
  dim3 grid(a.seq, a.nq, a.batch);
  if (dtype == TM_DTYPE_BF16)
    attn_dvec_kernel<bf16><<<grid, 64, 0, s>>>((const bf16 *)ctx, (const bf16 *)dctx, dvec, a);
  else
    attn_dvec_kernel<float><<<grid, 64, 0, s>>>((const float *)ctx, (const float *)dctx, dvec, a);
  return check_launch("attn_dvec");
}

int attn_bwd_generic_launch(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                            const void *qkv, const void *dctx, const float *lse, const float *dvec, void *dqkv,
                            hipStream_t s) {
  const AttnShape a = make_shape(seq, batch, nq, nkv, d);
  return dtype == TM_DTYPE_BF16 ? bwd_t<bf16>(a, qkv, dctx, lse, dvec, dqkv, s)
                                : bwd_t<float>(a, qkv, dctx, lse, dvec, dqkv, s);
}

}  // namespace tmk

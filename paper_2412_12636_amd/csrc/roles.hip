// The layers only the first and the last pipeline stage have (section 6.1 of the paper: the
// word-embedding layer and the output layer, of one shape), in the tensor-parallel form a rank runs with
// every collective served locally: vocabulary-parallel embedding (+ learned positions) forward and
// backward, and the last stage's final norm -> output layer -> vocabulary-parallel cross-entropy, forward
// and backward in one call.  The products and the norm are the stage's own kernels; this file adds the
// gather, the deterministic scatter-add, and the row-wise cross-entropy.
#include <math.h>

#include "common.h"
#include "../../include/tm_ops.h"
#include "../../include/tm_roles.h"

namespace tmk {

constexpr int kRoleThreads = 256;

// ---- embedding forward: one block per token row ---------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kRoleThreads) void embed_fwd_kernel(const int32_t *__restrict__ tokens, const T *__restrict__ w,
                                                                const T *__restrict__ pos, T *__restrict__ out, int batch,
                                                                int h, int v_local, int v0) {
  constexpr int VN = Vec<T>::N;
  const int64_t t = blockIdx.x;
  const int r = tokens[t] - v0;
  const bool inside = r >= 0 && r < v_local;
  const int64_t p = t / batch;  // position of the token row
  for (int c = threadIdx.x * VN; c < h; c += kRoleThreads * VN) {
    float a[VN], b[VN];
#pragma unroll
    for (int i = 0; i < VN; ++i) a[i] = b[i] = 0.f;
    if (inside) load_vec<T>(w + (int64_t)r * h + c, a);
    if (pos) load_vec<T>(pos + p * h + c, b);
#pragma unroll
    for (int i = 0; i < VN; ++i) a[i] += b[i];
    store_vec<T>(out + t * h + c, a);
  }
}

// ---- embedding backward: one block per vocabulary row, its tokens' rows added in token order (reproducible) -----
template <typename T>
__global__ __launch_bounds__(kRoleThreads) void embed_bwd_kernel(const int32_t *__restrict__ tokens, const T *__restrict__ dx0,
                                                                float *__restrict__ dw, int64_t n_tokens, int h, int v0,
                                                                int accumulate) {
  constexpr int VN = Vec<T>::N;
  constexpr int MAXCH = 8;  // h <= 256 * 8 * VN
  // 256 tokens are compared at once (one per thread); the waves' ballots go to LDS and every thread then walks the set
  // bits in ascending token order, so the sum is taken in the same order as a serial scan
  __shared__ unsigned long long hits[kRoleThreads / 64];
  const int want = (int)blockIdx.x + v0;
  float acc[MAXCH][VN];
#pragma unroll
  for (int k = 0; k < MAXCH; ++k)
#pragma unroll
    for (int i = 0; i < VN; ++i) acc[k][i] = 0.f;
  for (int64_t t0 = 0; t0 < n_tokens; t0 += kRoleThreads) {
    const int64_t t = t0 + threadIdx.x;
    const unsigned long long b = __builtin_amdgcn_ballot_w64(t < n_tokens && tokens[t] == want);
    __syncthreads();  // the previous chunk's masks have been read by everyone
    if ((threadIdx.x & 63) == 0) hits[threadIdx.x >> 6] = b;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kRoleThreads / 64; ++w) {
      unsigned long long m = hits[w];  // uniform over the block
      while (m) {
        const int i = w * 64 + __builtin_ctzll(m);
        m &= m - 1;
#pragma unroll
        for (int k = 0; k < MAXCH; ++k) {
          const int c = (k * kRoleThreads + threadIdx.x) * VN;
          if (c < h) {
            float a[VN];
            load_vec<T>(dx0 + (t0 + i) * h + c, a);
#pragma unroll
            for (int e = 0; e < VN; ++e) acc[k][e] += a[e];
          }
        }
      }
    }
  }
  float *row = dw + (int64_t)blockIdx.x * h;
#pragma unroll
  for (int k = 0; k < MAXCH; ++k) {
    const int c = (k * kRoleThreads + threadIdx.x) * VN;
    if (c < h) {
#pragma unroll
      for (int e = 0; e < VN; ++e) row[c + e] = accumulate ? row[c + e] + acc[k][e] : acc[k][e];
    }
  }
}

// dpos[p] (+)= sum over batch entries of dx0[p, n]; rows p >= seq: left alone (accumulate) or cleared
template <typename T>
__global__ __launch_bounds__(kRoleThreads) void pos_grad_kernel(const T *__restrict__ dx0, float *__restrict__ dpos, int seq,
                                                               int batch, int h, int accumulate) {
  constexpr int VN = Vec<T>::N;
  const int p = blockIdx.x;
  for (int c = threadIdx.x * VN; c < h; c += kRoleThreads * VN) {
    float s[VN];
#pragma unroll
    for (int i = 0; i < VN; ++i) s[i] = 0.f;
    if (p < seq)
      for (int n = 0; n < batch; ++n) {
        float a[VN];
        load_vec<T>(dx0 + ((int64_t)p * batch + n) * h + c, a);
#pragma unroll
        for (int i = 0; i < VN; ++i) s[i] += a[i];
      }
    float *row = dpos + (int64_t)p * h + c;
#pragma unroll
    for (int i = 0; i < VN; ++i) row[i] = accumulate ? row[i] + s[i] : s[i];
  }
}

// ---- cross-entropy over the rank's vocabulary shard, one block per token row -----------------------
// Reads the row three times (maximum, sum of exponentials, write-back): it sits in cache.  Writes
// loss_t and replaces the logits by their gradient (probability - one-hot where the target is local) * scale.
template <typename T>
__global__ __launch_bounds__(kRoleThreads) void xent_kernel(T *__restrict__ logits, const int32_t *__restrict__ targets,
                                                           float *__restrict__ loss_t, int v_local, int v0, float scale) {
  constexpr int VN = Vec<T>::N;
  __shared__ float red[2 * kRoleThreads / kWave];
  T *row = logits + (int64_t)blockIdx.x * v_local;
  const int tgt = targets[blockIdx.x] - v0;
  float mx = -INFINITY;
  for (int c = threadIdx.x * VN; c < v_local; c += kRoleThreads * VN) {
    float a[VN];
    load_vec<T>(row + c, a);
#pragma unroll
    for (int i = 0; i < VN; ++i) mx = fmaxf(mx, a[i]);
  }
  mx = wave_max(mx);
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int i = 1; i < kRoleThreads / kWave; ++i) mx = fmaxf(mx, red[i]);
  float se = 0.f, picked = 0.f;
  for (int c = threadIdx.x * VN; c < v_local; c += kRoleThreads * VN) {
    float a[VN];
    load_vec<T>(row + c, a);
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      se += expf(a[i] - mx);
      if (c + i == tgt) picked = a[i];
    }
  }
  block_sum2<kRoleThreads>(se, picked, red);
  if (threadIdx.x == 0) loss_t[blockIdx.x] = mx + logf(se) - picked;
  const float inv = scale / se;
  for (int c = threadIdx.x * VN; c < v_local; c += kRoleThreads * VN) {
    float a[VN];
    load_vec<T>(row + c, a);
#pragma unroll
    for (int i = 0; i < VN; ++i) a[i] = expf(a[i] - mx) * inv - (c + i == tgt ? scale : 0.f);
    store_vec<T>(row + c, a);
  }
}

// loss[0] = mean of loss_t, added in index order by one block
__global__ __launch_bounds__(kRoleThreads) void mean_kernel(const float *__restrict__ v, int64_t n, float *__restrict__ out) {
  __shared__ float red[2 * kRoleThreads / kWave];
  float s = 0.f, unused = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += kRoleThreads) s += v[i];
  block_sum2<kRoleThreads>(s, unused, red);
  if (threadIdx.x == 0) out[0] = s / (float)n;
}

static int check_embed(const char *what, int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "%s: unknown dtype %d", what, dtype);
  if (seq <= 0 || batch <= 0 || h <= 0 || v_local <= 0) return fail(TM_EINVAL, "%s: empty shape", what);
  if (h % 8) return fail(TM_ESIZE, "%s: width %lld is not a multiple of 8", what, (long long)h);
  if (seq * batch > 0x7fffffffLL || v_local > 0x7fffffffLL || h > 0x7fffffffLL)
    return fail(TM_ESIZE, "%s: dimension above 2^31", what);
  return TM_OK;
}

}  // namespace tmk

using namespace tmk;

extern "C" int tm_op_embed_fwd(int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local, int64_t v0,
                               const int32_t *tokens, const void *w, const void *pos_emb, void *x0, void *stream) {
  if (int e = check_embed("embed_fwd", dtype, seq, batch, h, v_local)) return e;
  if (!tokens || !w || !x0) return fail(TM_EINVAL, "embed_fwd: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  const unsigned grid = (unsigned)(seq * batch);
  g_last_kernel = "embed_fwd_kernel";
  if (dtype == TM_DTYPE_BF16)
    embed_fwd_kernel<bf16><<<grid, kRoleThreads, 0, s>>>(tokens, (const bf16 *)w, (const bf16 *)pos_emb, (bf16 *)x0, (int)batch,
                                                         (int)h, (int)v_local, (int)v0);
  else
    embed_fwd_kernel<float><<<grid, kRoleThreads, 0, s>>>(tokens, (const float *)w, (const float *)pos_emb, (float *)x0,
                                                          (int)batch, (int)h, (int)v_local, (int)v0);
  return check_launch("embed_fwd");
}

extern "C" int tm_op_embed_bwd(int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local, int64_t v0,
                               const int32_t *tokens, const void *dx0, float *dw, float *dpos, int64_t n_pos,
                               int accumulate, void *stream) {
  if (int e = check_embed("embed_bwd", dtype, seq, batch, h, v_local)) return e;
  if (!tokens || !dx0 || !dw) return fail(TM_EINVAL, "embed_bwd: NULL pointer");
  if (dpos && n_pos < seq) return fail(TM_EINVAL, "embed_bwd: %lld positions for a sequence of %lld", (long long)n_pos, (long long)seq);
  const int64_t hmax = (int64_t)kRoleThreads * 8 * (dtype == TM_DTYPE_BF16 ? 8 : 4);
  if (h > hmax) return fail(TM_ESIZE, "embed_bwd: width %lld above the limit %lld", (long long)h, (long long)hmax);
  hipStream_t s = (hipStream_t)stream;
  g_last_kernel = "embed_bwd_kernel";
  if (dtype == TM_DTYPE_BF16)
    embed_bwd_kernel<bf16><<<(unsigned)v_local, kRoleThreads, 0, s>>>(tokens, (const bf16 *)dx0, dw, seq * batch, (int)h, (int)v0,
                                                                      accumulate);
  else
    embed_bwd_kernel<float><<<(unsigned)v_local, kRoleThreads, 0, s>>>(tokens, (const float *)dx0, dw, seq * batch, (int)h,
                                                                       (int)v0, accumulate);
  if (dpos) {
    if (dtype == TM_DTYPE_BF16)
      pos_grad_kernel<bf16><<<(unsigned)n_pos, kRoleThreads, 0, s>>>((const bf16 *)dx0, dpos, (int)seq, (int)batch, (int)h, accumulate);
    else
      pos_grad_kernel<float><<<(unsigned)n_pos, kRoleThreads, 0, s>>>((const float *)dx0, dpos, (int)seq, (int)batch, (int)h,
                                                                      accumulate);
  }
  return check_launch("embed_bwd");
}

extern "C" int tm_op_xent(int dtype, int64_t T, int64_t v_local, int64_t v0, void *logits, const int32_t *targets,
                          double dloss, float *loss_t, float *loss, void *stream) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "xent: unknown dtype %d", dtype);
  if (T <= 0 || v_local <= 0) return fail(TM_EINVAL, "xent: empty shape");
  if (v_local % 8) return fail(TM_ESIZE, "xent: shard of %lld entries is not a multiple of 8", (long long)v_local);
  if (T > 0x7fffffffLL || v_local > 0x7fffffffLL) return fail(TM_ESIZE, "xent: dimension above 2^31");
  if (!logits || !targets || !loss_t || !loss) return fail(TM_EINVAL, "xent: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  const float scale = (float)(dloss / (double)T);
  g_last_kernel = "xent_kernel";
  if (dtype == TM_DTYPE_BF16)
    xent_kernel<bf16><<<(unsigned)T, kRoleThreads, 0, s>>>((bf16 *)logits, targets, loss_t, (int)v_local, (int)v0, scale);
  else
    xent_kernel<float><<<(unsigned)T, kRoleThreads, 0, s>>>((float *)logits, targets, loss_t, (int)v_local, (int)v0, scale);
  mean_kernel<<<1, kRoleThreads, 0, s>>>(loss_t, T, loss);
  return check_launch("xent");
}

// workspace layout of the last-stage call
namespace {
struct HeadPlan {
  int64_t hn, mean, rstd, logits, dhn, loss_t, reduce, total;
};
HeadPlan head_plan(int dtype, int64_t T, int64_t h, int64_t v_local) {
  const int64_t es = dtype == TM_DTYPE_BF16 ? 2 : 4;
  HeadPlan p;
  int64_t at = 0;
  auto take = [&](int64_t bytes) {
    const int64_t r = at;
    at += (bytes + 255) / 256 * 256;
    return r;
  };
  p.hn = take(T * h * es);
  p.mean = take(T * 4);
  p.rstd = take(T * 4);
  p.logits = take(T * v_local * es);
  p.dhn = take(T * h * es);
  p.loss_t = take(T * 4);
  p.reduce = take(tm_op_reduce_scratch_bytes(T, 3 * h));
  p.total = at;
  return p;
}
}  // namespace

extern "C" int64_t tm_head_workspace_bytes(int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local) {
  if (int e = check_embed("head_workspace_bytes", dtype, seq, batch, h, v_local)) return e;
  return head_plan(dtype, seq * batch, h, v_local).total;
}

extern "C" int tm_head_fwd_bwd(int dtype, int norm, double eps, int64_t seq, int64_t batch, int64_t h, int64_t v_local,
                               int64_t v0, const void *y, const int32_t *targets, const void *gain, const void *offset,
                               const void *w, double dloss, void *workspace, int64_t workspace_bytes, float *loss, void *dy,
                               float *dgain, float *doffset, float *dw, int accumulate, void *stream) {
  if (int e = check_embed("head_fwd_bwd", dtype, seq, batch, h, v_local)) return e;
  if (v_local % 8) return fail(TM_ESIZE, "head_fwd_bwd: shard of %lld entries is not a multiple of 8", (long long)v_local);
  if (!y || !targets || !gain || !w || !workspace || !loss || !dy || !dgain || !dw)
    return fail(TM_EINVAL, "head_fwd_bwd: NULL pointer");
  if (norm == TM_NORM_LAYERNORM && (!offset || !doffset)) return fail(TM_EINVAL, "head_fwd_bwd: LayerNorm needs its offset");
  if (((uintptr_t)workspace) & 255) return fail(TM_EALIGN, "head_fwd_bwd: workspace must be 256-byte aligned");
  const int64_t T = seq * batch;
  const HeadPlan p = head_plan(dtype, T, h, v_local);
  if (workspace_bytes < p.total)
    return fail(TM_ESIZE, "head_fwd_bwd: workspace of %lld bytes, %lld needed", (long long)workspace_bytes, (long long)p.total);
  char *ws = (char *)workspace;
  // hn = Norm(y); logits = hn W^T
  if (int e = tm_op_norm_fwd(dtype, norm, T, h, eps, y, gain, offset, ws + p.hn, (float *)(ws + p.mean), (float *)(ws + p.rstd), stream)) return e;
  if (int e = tm_op_linear_fwd(dtype, T, v_local, h, ws + p.hn, w, nullptr, nullptr, ws + p.logits, stream)) return e;
  // loss and, in place of the logits, their gradient
  if (int e = tm_op_xent(dtype, T, v_local, v0, ws + p.logits, targets, dloss, (float *)(ws + p.loss_t), loss, stream)) return e;
  // dhn = dlogits W; dW (+)= dlogits^T hn; dy = norm backward
  if (int e = tm_op_linear_dgrad(dtype, T, v_local, h, ws + p.logits, w, ws + p.dhn, stream)) return e;
  if (int e = tm_op_linear_wgrad(dtype, T, v_local, h, ws + p.logits, ws + p.hn, dw, accumulate, stream)) return e;
  return tm_op_norm_bwd(dtype, norm, T, h, ws + p.dhn, y, (const float *)(ws + p.mean), (const float *)(ws + p.rstd), gain, nullptr,
                        dy, dgain, doffset, ws + p.reduce, accumulate, stream);
}

// One rank's mixture-of-experts MLP shard (the paper's Table 3 workloads; fixed-size expert buffers as in its
// section 4.2): router with top-k gates, capacity dispatch into per-expert buffers, identity all-to-all over the
// expert-parallel groups, the experts' MLPs (this library's own linear / activation steps, one pass per local
// expert), combine; and the backward pass of all of it.  Every sum has a fixed order: no atomics.
#include <math.h>
#include <string.h>

#include <deque>
#include <string>
#include <vector>

#include "common.h"
#include "../../include/tm_moe.h"
#include "../../include/tm_ops.h"

namespace tmk {

constexpr int kMoeMaxExperts = 64, kMoeMaxTopK = 8, kMoeThreads = 256;
static_assert(kMoeMaxExperts <= kWave, "one lane per expert count");
constexpr int kWgradSegTokens = 128;  // tokens per block of the router weight gradient
__device__ __forceinline__ int ceil_div_dev(int a, int b) { return (a + b - 1) / b; }

struct MoeDims {
  int64_t T, h, f, E, ep, k, C, El, rows, es;
};

static int moe_validate(const tm_moe_config_t *c) {
  if (!c) return fail(TM_EINVAL, "moe config is NULL");
  if (c->tokens <= 0 || c->hidden <= 0 || c->ffn <= 0 || c->capacity <= 0 || c->ep <= 0)
    return fail(TM_EINVAL, "moe config: every size must be positive");
  if (c->dtype != TM_DTYPE_FP32 && c->dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "moe config: unknown dtype %d", c->dtype);
  if (c->act != TM_ACT_GELU_TANH && c->act != TM_ACT_GELU_ERF) return fail(TM_EINVAL, "moe config: the experts use a GeLU form");
  if (c->hidden % 8 || c->ffn % 8) return fail(TM_ESIZE, "moe config: hidden and ffn must be multiples of 8");
  if (c->n_experts < 1 || c->n_experts > kMoeMaxExperts) return fail(TM_ESIZE, "moe config: 1 to %d experts", kMoeMaxExperts);
  if (c->n_experts % c->ep) return fail(TM_ESIZE, "moe config: n_experts must be a multiple of ep");
  if (c->top_k < 1 || c->top_k > kMoeMaxTopK || c->top_k > c->n_experts)
    return fail(TM_ESIZE, "moe config: top_k between 1 and min(n_experts, %d)", kMoeMaxTopK);
  const int64_t rows = (int64_t)c->n_experts * c->capacity, widest = c->hidden > c->ffn ? c->hidden : c->ffn;
  if (rows * widest >= (1LL << 31) || (int64_t)c->tokens * widest >= (1LL << 31) || (int64_t)c->tokens * c->top_k >= (1LL << 30))
    return fail(TM_ESIZE, "moe config: a tensor has 2^31 elements or more");
  return TM_OK;
}

static MoeDims moe_dims(const tm_moe_config_t *c) {
  MoeDims d;
  d.T = c->tokens, d.h = c->hidden, d.f = c->ffn, d.E = c->n_experts, d.ep = c->ep, d.k = c->top_k, d.C = c->capacity;
  d.El = d.E / d.ep;
  d.rows = d.E * d.C;
  d.es = c->dtype == TM_DTYPE_BF16 ? 2 : 4;
  return d;
}

struct MoeTensor {
  std::string name;
  int64_t offset, rows, cols;
};
static std::vector<MoeTensor> moe_tensors(const tm_moe_config_t *c, int64_t *total) {
  const MoeDims d = moe_dims(c);
  std::vector<MoeTensor> v;
  int64_t at = 0;
  auto add = [&](const std::string &n, int64_t r, int64_t cc) {
    v.push_back({n, at, r, cc});
    at += r * cc;
  };
  add("w_router", d.E, d.h);
  for (int64_t j = 0; j < d.El; ++j) {
    const std::string sfx = "." + std::to_string(j);
    add("w_fc1" + sfx, d.f, d.h);
    if (c->has_bias) add("b_fc1" + sfx, d.f, 1);
    add("w_fc2" + sfx, d.h, d.f);
    if (c->has_bias) add("b_fc2" + sfx, d.h, 1);
  }
  if (total) *total = at;
  return v;
}

struct MoePlan {
  int64_t logits, top_idx, gates, slot_row, row_src, buf, u, g, o, d_o, dg, dbuf, dgate, dlog, reduce, total;
  int64_t reduce_bytes, wr_part, wr_segs;
};
static MoePlan moe_plan(const tm_moe_config_t *c) {
  const MoeDims d = moe_dims(c);
  MoePlan p;
  int64_t at = 0;
  auto take = [&](int64_t bytes) {
    const int64_t r = at;
    at += (bytes + 255) / 256 * 256;
    return r;
  };
  p.logits = take(d.T * d.E * 4);
  p.top_idx = take(d.T * d.k * 4);
  p.gates = take(d.T * d.k * 4);
  p.slot_row = take(d.T * d.k * 4);
  p.row_src = take(d.rows * 4);
  p.buf = take(d.rows * d.h * d.es);
  p.u = take(d.rows * d.f * d.es);
  p.g = take(d.rows * d.f * d.es);
  p.o = take(d.rows * d.h * d.es);
  p.d_o = take(d.rows * d.h * d.es);
  p.dg = take(d.rows * d.f * d.es);
  p.dbuf = take(d.rows * d.h * d.es);
  p.dgate = take(d.T * d.k * 4);
  p.dlog = take(d.T * d.k * 4);
  p.wr_segs = ceil_div(d.T, kWgradSegTokens);
  p.wr_part = take(p.wr_segs * d.E * d.h * 4);
  p.reduce_bytes = tm_op_reduce_scratch_bytes(d.ep * d.C, d.h > d.f ? d.h : d.f);
  p.reduce = take(p.reduce_bytes);
  p.total = at;
  return p;
}

// ---- router: one block per 8 tokens; a thread keeps 8 x 16 partial logits over its share of the hidden axis, so a
// chunk of a router row is fetched once for 8 tokens (one block per token fetched the whole router matrix per token:
// 1.3 GB through L2 at 2048 tokens and 16 experts).  More than 16 experts: in groups of 16.
constexpr int kRouterTokens = 8, kRouterGroup = 16;
template <typename T>
__global__ __launch_bounds__(kMoeThreads) void moe_router_kernel(const T *__restrict__ c, const T *__restrict__ wr,
                                                                 float *__restrict__ logits, int *__restrict__ top_idx,
                                                                 float *__restrict__ gates, int n_tokens, int h, int E, int k) {
  constexpr int VN = Vec<T>::N;
  constexpr int NWAVE = kMoeThreads / kWave;
  __shared__ float part[NWAVE][kRouterTokens][kRouterGroup];
  __shared__ float lg[kRouterTokens][kMoeMaxExperts];
  const int t0 = blockIdx.x * kRouterTokens, tid = threadIdx.x, nch = h / VN;
  const int wave = tid / kWave, lane = tid % kWave;
  for (int e0 = 0; e0 < E; e0 += kRouterGroup) {
    float acc[kRouterTokens][kRouterGroup];
#pragma unroll
    for (int j = 0; j < kRouterTokens; ++j)
#pragma unroll
      for (int e = 0; e < kRouterGroup; ++e) acc[j][e] = 0.f;
    for (int ch = tid; ch < nch; ch += kMoeThreads) {
      // All 24 loads of a chunk are issued before the first use, raw, with no branches around them (tokens past the
      // end repeat the last token, experts past the end the last expert; those results are never stored).
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      u32x4 ra[kRouterTokens], rw[kRouterGroup];
#pragma unroll
      for (int j = 0; j < kRouterTokens; ++j) {
        const int tj = t0 + j < n_tokens ? t0 + j : n_tokens - 1;
        ra[j] = *reinterpret_cast<const u32x4 *>(c + (int64_t)tj * h + ch * VN);
      }
#pragma unroll
      for (int e = 0; e < kRouterGroup; ++e) {
        const int ee = e0 + e < E ? e0 + e : E - 1;
        rw[e] = *reinterpret_cast<const u32x4 *>(wr + (int64_t)ee * h + ch * VN);
      }
      float a[kRouterTokens][VN];
#pragma unroll
      for (int j = 0; j < kRouterTokens; ++j) {
        union { u32x4 raw; Vec<T> v; } u;
        u.raw = ra[j];
#pragma unroll
        for (int i = 0; i < VN; ++i) a[j][i] = to_f32(u.v.v[i]);
      }
#pragma unroll
      for (int e = 0; e < kRouterGroup; ++e) {
        union { u32x4 raw; Vec<T> v; } u;
        u.raw = rw[e];
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          const float w = to_f32(u.v.v[i]);
#pragma unroll
          for (int j = 0; j < kRouterTokens; ++j) acc[j][e] = fmaf(a[j][i], w, acc[j][e]);
        }
      }
    }
    // lanes, then waves in wave order
#pragma unroll
    for (int j = 0; j < kRouterTokens; ++j)
#pragma unroll
      for (int e = 0; e < kRouterGroup; ++e) {
        const float v = wave_sum(acc[j][e]);
        if (lane == 0) part[wave][j][e] = v;
      }
    __syncthreads();
    if (tid < kRouterTokens * kRouterGroup) {
      const int j = tid / kRouterGroup, e = tid % kRouterGroup;
      float v = part[0][j][e];
#pragma unroll
      for (int w = 1; w < NWAVE; ++w) v += part[w][j][e];
      if (e0 + e < E) lg[j][e0 + e] = v;
    }
    __syncthreads();
  }
  for (int i = tid; i < kRouterTokens * E; i += kMoeThreads) {
    const int j = i / E, e = i % E;
    if (t0 + j < n_tokens) logits[(int64_t)(t0 + j) * E + e] = lg[j][e];
  }
  if (tid < kRouterTokens && t0 + tid < n_tokens) {
    // the k largest, ties to the lower index; gates = softmax over the chosen logits
    const int t = t0 + tid;
    const float *row = lg[tid];
    uint64_t used = 0;
    float val[kMoeMaxTopK];
    int idx[kMoeMaxTopK];
    for (int i = 0; i < k; ++i) {
      int best = -1;
      for (int e = 0; e < E; ++e)
        if (!((used >> e) & 1) && (best < 0 || row[e] > row[best])) best = e;
      used |= 1ull << best;
      idx[i] = best;
      val[i] = row[best];
    }
    const float top = val[0];  // the maximum
    float sum = 0.f;
    for (int i = 0; i < k; ++i) {
      val[i] = expf(val[i] - top);
      sum += val[i];
    }
    for (int i = 0; i < k; ++i) {
      top_idx[(int64_t)t * k + i] = idx[i];
      gates[(int64_t)t * k + i] = val[i] / sum;
    }
  }
}

// ---- dispatch plan: position of every assignment inside its expert's buffer, in assignment order ---------
// One block of 16 waves; wave w owns a contiguous segment of the assignments.  Pass 1 counts the segment's
// assignments per expert (a ballot per expert over 64 assignments at a time; lane e keeps expert e's count),
// the counts of the earlier segments give each wave its starting fill levels, and pass 2 hands out the rows:
// an assignment's position is its expert's fill level plus the number of earlier lanes in the same ballot.
constexpr int kPlanWaves = 16;
__global__ __launch_bounds__(kPlanWaves * kWave) void moe_plan_kernel(const int *__restrict__ top_idx, int *__restrict__ slot_row,
                                                                      int *__restrict__ row_src, int n_assign, int E, int El,
                                                                      int ep, int C) {
  __shared__ int counts[kPlanWaves][kMoeMaxExperts];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int seg = (int)ceil_div_dev(ceil_div_dev(n_assign, kPlanWaves), kWave) * kWave;
  const int a_begin = wave * seg;
  const int a_end = a_begin + seg < n_assign ? a_begin + seg : n_assign;
  int cnt = 0;
  for (int a0 = a_begin; a0 < a_end; a0 += kWave) {
    const int mine = a0 + lane < a_end ? top_idx[a0 + lane] : -1;
    for (int e = 0; e < E; ++e) {
      const uint64_t mask = __ballot(mine == e);
      if (lane == e) cnt += __popcll(mask);
    }
  }
  counts[wave][lane] = cnt;
  __syncthreads();
  int used = 0;  // lane e: rows of expert e's buffer taken by earlier segments (may pass C: the surplus was dropped)
  for (int w = 0; w < wave; ++w) used += counts[w][lane];
  const uint64_t below = (1ull << lane) - 1ull;
  for (int a0 = a_begin; a0 < a_end; a0 += kWave) {
    const int a = a0 + lane;
    const int mine = a < a_end ? top_idx[a] : -1;
    int row = -1;
    for (int e = 0; e < E; ++e) {
      const uint64_t mask = __ballot(mine == e);
      if (mask == 0) continue;  // uniform over the wave
      const int before = __shfl(used, e, kWave);
      if (mine == e) {
        const int pos = before + __popcll(mask & below);
        if (pos < C) row = ((e % El) * ep + e / El) * C + pos;
      }
      if (lane == e) used += __popcll(mask);
    }
    if (a < a_end) {
      slot_row[a] = row;
      if (row >= 0) row_src[row] = a;
    }
  }
  // rows no assignment took
  for (int e = wave; e < E; e += kPlanWaves) {
    int total = 0;
    for (int w = 0; w < kPlanWaves; ++w) total += counts[w][e];
    const int base = ((e % El) * ep + e / El) * C;
    for (int r = (total < C ? total : C) + lane; r < C; r += kWave) row_src[base + r] = -1;
  }
}

// ---- buffers: row = the token's input row, or zero ---------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kMoeThreads) void moe_gather_kernel(const T *__restrict__ c, const int *__restrict__ row_src,
                                                                 T *__restrict__ buf, int h, int k) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  constexpr int VN = Vec<T>::N;
  const int64_t row = blockIdx.x;
  const int src = row_src[row];
  u32x4 *dst = reinterpret_cast<u32x4 *>(buf + row * h);
  const u32x4 *from = reinterpret_cast<const u32x4 *>(c + (int64_t)(src < 0 ? 0 : src / k) * h);
  for (int ch = threadIdx.x; ch < h / VN; ch += kMoeThreads) dst[ch] = src < 0 ? u32x4{0u, 0u, 0u, 0u} : from[ch];
}

// ---- combine: out[t] = sum over kept assignments of gate * o[row] ----------------------------------
template <typename T>
__global__ __launch_bounds__(kMoeThreads) void moe_combine_kernel(const T *__restrict__ o, const int *__restrict__ slot_row,
                                                                  const float *__restrict__ gates, T *__restrict__ out, int h,
                                                                  int k) {
  constexpr int VN = Vec<T>::N;
  const int64_t t = blockIdx.x;
  int rows[kMoeMaxTopK];
  float gt[kMoeMaxTopK];
#pragma unroll
  for (int i = 0; i < kMoeMaxTopK; ++i) {
    rows[i] = i < k ? slot_row[t * k + i] : -1;
    gt[i] = i < k ? gates[t * k + i] : 0.f;
  }
  for (int ch = threadIdx.x; ch < h / VN; ch += kMoeThreads) {
    float acc[VN];
#pragma unroll
    for (int j = 0; j < VN; ++j) acc[j] = 0.f;
#pragma unroll
    for (int i = 0; i < kMoeMaxTopK; ++i) {
      if (rows[i] < 0) continue;
      float a[VN];
      load_vec<T>(o + (int64_t)rows[i] * h + ch * VN, a);
#pragma unroll
      for (int j = 0; j < VN; ++j) acc[j] = fmaf(gt[i], a[j], acc[j]);
    }
    store_vec<T>(out + t * h + ch * VN, acc);
  }
}

// ---- combine, backward: d_o[row] = gate * dout[token]; dgate = <dout[token], o[row]> ------------------
template <typename T>
__global__ __launch_bounds__(kMoeThreads) void moe_combine_bwd_kernel(const T *__restrict__ dout, const T *__restrict__ o,
                                                                      const int *__restrict__ row_src,
                                                                      const float *__restrict__ gates, T *__restrict__ d_o,
                                                                      float *__restrict__ dgate, int h, int k) {
  constexpr int VN = Vec<T>::N;
  __shared__ float red[2 * kMoeThreads / kWave];
  const int64_t row = blockIdx.x;
  const int src = row_src[row];
  if (src < 0) {
    float z[VN];
#pragma unroll
    for (int j = 0; j < VN; ++j) z[j] = 0.f;
    for (int ch = threadIdx.x; ch < h / VN; ch += kMoeThreads) store_vec<T>(d_o + row * h + ch * VN, z);
    return;
  }
  const int64_t t = src / k;
  const float gate = gates[src];
  float dot = 0.f, unused = 0.f;
  for (int ch = threadIdx.x; ch < h / VN; ch += kMoeThreads) {
    float d[VN], a[VN];
    load_vec<T>(dout + t * h + ch * VN, d);
    load_vec<T>(o + row * h + ch * VN, a);
#pragma unroll
    for (int j = 0; j < VN; ++j) {
      dot = fmaf(d[j], a[j], dot);
      d[j] *= gate;
    }
    store_vec<T>(d_o + row * h + ch * VN, d);
  }
  block_sum2<kMoeThreads>(dot, unused, red);
  if (threadIdx.x == 0) dgate[src] = dot;
}

// ---- dispatch and router, backward: dc[t] = sum of the kept rows of dbuf + sum_i dlogit_i Wr[idx_i] --
template <typename T>
__global__ __launch_bounds__(kMoeThreads) void moe_dispatch_bwd_kernel(const T *__restrict__ dbuf, const T *__restrict__ wr,
                                                                       const int *__restrict__ slot_row,
                                                                       const int *__restrict__ top_idx,
                                                                       const float *__restrict__ gates,
                                                                       const float *__restrict__ dgate, float *__restrict__ dlog,
                                                                       T *__restrict__ dc, int h, int k) {
  constexpr int VN = Vec<T>::N;
  const int64_t t = blockIdx.x;
  int rows[kMoeMaxTopK], idx[kMoeMaxTopK];
  float dch[kMoeMaxTopK];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kMoeMaxTopK; ++i) {
    rows[i] = i < k ? slot_row[t * k + i] : -1;
    idx[i] = i < k ? top_idx[t * k + i] : 0;
    const float gt = i < k ? gates[t * k + i] : 0.f;
    const float dg = (i < k && rows[i] >= 0) ? dgate[t * k + i] : 0.f;  // a dropped assignment has no gate gradient of its own
    dch[i] = dg;
    s = fmaf(gt, dg, s);
  }
#pragma unroll
  for (int i = 0; i < kMoeMaxTopK; ++i) {
    const float gt = i < k ? gates[t * k + i] : 0.f;
    dch[i] = gt * (dch[i] - s);  // softmax over the chosen logits
    if (threadIdx.x == 0 && i < k) dlog[t * k + i] = dch[i];
  }
  for (int ch = threadIdx.x; ch < h / VN; ch += kMoeThreads) {
    float acc[VN];
#pragma unroll
    for (int j = 0; j < VN; ++j) acc[j] = 0.f;
#pragma unroll
    for (int i = 0; i < kMoeMaxTopK; ++i) {
      if (rows[i] < 0) continue;
      float a[VN];
      load_vec<T>(dbuf + (int64_t)rows[i] * h + ch * VN, a);
#pragma unroll
      for (int j = 0; j < VN; ++j) acc[j] += a[j];
    }
#pragma unroll
    for (int i = 0; i < kMoeMaxTopK; ++i) {
      if (i >= k) continue;
      float w[VN];
      load_vec<T>(wr + (int64_t)idx[i] * h + ch * VN, w);
#pragma unroll
      for (int j = 0; j < VN; ++j) acc[j] = fmaf(dch[i], w[j], acc[j]);
    }
    store_vec<T>(dc + t * h + ch * VN, acc);
  }
}

// ---- router weights: dWr[e, col] (+)= sum over tokens, in token order, of dlogit[t, e] c[t, col] ------
// A block owns 256 columns and one segment of the tokens and keeps one fp32 accumulator per (expert, column)
// in LDS; a token touches the accumulators of its k chosen experts only.  The segments' partial sums are
// added in segment order by a second kernel.
template <typename T>
__global__ __launch_bounds__(kMoeThreads) void moe_router_wgrad_kernel(const T *__restrict__ c, const int *__restrict__ top_idx,
                                                                       const float *__restrict__ dlog, float *__restrict__ part,
                                                                       int n_tok, int h, int E, int k) {
  extern __shared__ __align__(16) char smem[];
  float *acc = reinterpret_cast<float *>(smem);                         // [E][256]
  int *s_idx = reinterpret_cast<int *>(acc + (size_t)E * kMoeThreads);  // [segment tokens][k]
  float *s_dl = reinterpret_cast<float *>(s_idx + kWgradSegTokens * kMoeMaxTopK);
  const int tid = threadIdx.x, col = blockIdx.x * kMoeThreads + tid, seg = blockIdx.y;
  const bool valid = col < h;
  const int t0 = seg * kWgradSegTokens;
  const int n = n_tok - t0 < kWgradSegTokens ? n_tok - t0 : kWgradSegTokens;
  for (int e = 0; e < E; ++e) acc[e * kMoeThreads + tid] = 0.f;
  for (int i = tid; i < n * k; i += kMoeThreads) {
    s_idx[i] = top_idx[(int64_t)t0 * k + i];
    s_dl[i] = dlog[(int64_t)t0 * k + i];
  }
  __syncthreads();
#pragma unroll 8
  for (int tt = 0; tt < n; ++tt) {
    const float cv = valid ? to_f32(c[(int64_t)(t0 + tt) * h + col]) : 0.f;
    for (int i = 0; i < k; ++i) {
      float *a = acc + s_idx[tt * k + i] * kMoeThreads + tid;
      *a = fmaf(s_dl[tt * k + i], cv, *a);
    }
  }
  if (valid)
    for (int e = 0; e < E; ++e) part[((int64_t)seg * E + e) * h + col] = acc[e * kMoeThreads + tid];
}

__global__ __launch_bounds__(kMoeThreads) void moe_router_wgrad_reduce_kernel(const float *__restrict__ part, float *__restrict__ dwr,
                                                                              int64_t n, int segs, int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * kMoeThreads + threadIdx.x;
  if (i >= n) return;
  float sum = accumulate ? dwr[i] : 0.f;
  for (int sg = 0; sg < segs; ++sg) sum += part[(int64_t)sg * n + i];
  dwr[i] = sum;
}

template <typename K> static int set_lds(K kernel, int bytes, const char *what) {
  if (bytes > 160 * 1024) return fail(TM_ESIZE, "%s: needs %d bytes of LDS", what, bytes);
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return fail(TM_ELAUNCH, "%s: cannot reserve %d bytes of LDS", what, bytes);
  }
  return TM_OK;
}

}  // namespace tmk

using namespace tmk;

extern "C" int64_t tm_moe_param_count(const tm_moe_config_t *cfg) {
  if (int e = moe_validate(cfg)) return e;
  int64_t total = 0;
  moe_tensors(cfg, &total);
  return total;
}

extern "C" int tm_moe_param_layout(const tm_moe_config_t *cfg, int index, const char **name, int64_t *offset_elems,
                                   int64_t shape[2]) {
  if (int e = moe_validate(cfg)) return e;
  const std::vector<MoeTensor> v = moe_tensors(cfg, nullptr);
  if (index == -1) return (int)v.size();
  if (index < 0 || index >= (int)v.size()) return fail(TM_EINVAL, "moe_param_layout: index %d out of range", index);
  if (name) {
    static thread_local std::deque<std::string> pool;  // growing a deque never moves the strings
    const std::string *found = nullptr;
    for (const std::string &s : pool)
      if (s == v[index].name) found = &s;
    if (!found) {
      pool.push_back(v[index].name);
      found = &pool.back();
    }
    *name = found->c_str();
  }
  if (offset_elems) *offset_elems = v[index].offset;
  if (shape) shape[0] = v[index].rows, shape[1] = v[index].cols;
  return TM_OK;
}

extern "C" int64_t tm_moe_workspace_bytes(const tm_moe_config_t *cfg) {
  if (int e = moe_validate(cfg)) return e;
  return moe_plan(cfg).total;
}

extern "C" int64_t tm_moe_workspace_offset(const tm_moe_config_t *cfg, int region, int64_t *bytes) {
  if (int e = moe_validate(cfg)) return e;
  const MoePlan p = moe_plan(cfg);
  const MoeDims d = moe_dims(cfg);
  int64_t off, n;
  switch (region) {
    case TM_MOE_WS_LOGITS: off = p.logits, n = d.T * d.E * 4; break;
    case TM_MOE_WS_TOP_IDX: off = p.top_idx, n = d.T * d.k * 4; break;
    case TM_MOE_WS_GATES: off = p.gates, n = d.T * d.k * 4; break;
    case TM_MOE_WS_SLOT_ROW: off = p.slot_row, n = d.T * d.k * 4; break;
    default: return fail(TM_EINVAL, "moe_workspace_offset: unknown region %d", region);
  }
  if (bytes) *bytes = n;
  return off;
}

static int moe_check_call(const char *what, const tm_moe_config_t *cfg, const void *const *ptrs, int n, int64_t ws_bytes) {
  if (int e = moe_validate(cfg)) return e;
  for (int i = 0; i < n; ++i) {
    if (!ptrs[i]) return fail(TM_EINVAL, "%s: NULL pointer", what);
    if (((uintptr_t)ptrs[i]) & 255) return fail(TM_EALIGN, "%s: pointers must be 256-byte aligned", what);
  }
  const int64_t need = moe_plan(cfg).total;
  if (ws_bytes < need) return fail(TM_ESIZE, "%s: workspace of %lld bytes, %lld needed", what, (long long)ws_bytes, (long long)need);
  return TM_OK;
}

#define TM_TRY(expr)       \
  do {                     \
    const int _e = (expr); \
    if (_e) return _e;     \
  } while (0)

extern "C" int tm_moe_fwd(const tm_moe_config_t *cfg, const void *params, const void *c, void *out, void *workspace,
                          int64_t workspace_bytes, void *stream) {
  const void *ptrs[] = {params, c, out, workspace};
  if (int e = moe_check_call("moe_fwd", cfg, ptrs, 4, workspace_bytes)) return e;
  const MoeDims d = moe_dims(cfg);
  const MoePlan p = moe_plan(cfg);
  int64_t total = 0;
  const std::vector<MoeTensor> tn = moe_tensors(cfg, &total);
  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const char *par = (const char *)params;
  const int dt = cfg->dtype;
  float *logits = (float *)(ws + p.logits), *gates = (float *)(ws + p.gates);
  int *top_idx = (int *)(ws + p.top_idx), *slot_row = (int *)(ws + p.slot_row), *row_src = (int *)(ws + p.row_src);
  g_last_kernel = "moe_router_kernel";
  const unsigned router_blocks = (unsigned)ceil_div(d.T, (int64_t)kRouterTokens);
  if (dt == TM_DTYPE_BF16)
    moe_router_kernel<bf16><<<router_blocks, kMoeThreads, 0, s>>>((const bf16 *)c, (const bf16 *)par, logits, top_idx, gates, (int)d.T,
                                                                  (int)d.h, (int)d.E, (int)d.k);
  else
    moe_router_kernel<float><<<router_blocks, kMoeThreads, 0, s>>>((const float *)c, (const float *)par, logits, top_idx, gates,
                                                                   (int)d.T, (int)d.h, (int)d.E, (int)d.k);
  moe_plan_kernel<<<1, kPlanWaves * kWave, 0, s>>>(top_idx, slot_row, row_src, (int)(d.T * d.k), (int)d.E, (int)d.El, (int)d.ep, (int)d.C);
  if (dt == TM_DTYPE_BF16)
    moe_gather_kernel<bf16><<<(unsigned)d.rows, kMoeThreads, 0, s>>>((const bf16 *)c, row_src, (bf16 *)(ws + p.buf), (int)d.h, (int)d.k);
  else
    moe_gather_kernel<float><<<(unsigned)d.rows, kMoeThreads, 0, s>>>((const float *)c, row_src, (float *)(ws + p.buf), (int)d.h, (int)d.k);
  TM_TRY(check_launch("moe_fwd routing"));
  // the experts: local expert j works on the ep buffers that the identity exchange leaves with it
  const int64_t grows = d.ep * d.C;
  const int per = cfg->has_bias ? 4 : 2;
  for (int64_t j = 0; j < d.El; ++j) {
    const MoeTensor &w1 = tn[1 + j * per], &w2 = tn[1 + j * per + (cfg->has_bias ? 2 : 1)];
    const void *b1 = cfg->has_bias ? par + tn[1 + j * per + 1].offset * d.es : nullptr;
    const void *b2 = cfg->has_bias ? par + tn[1 + j * per + 3].offset * d.es : nullptr;
    char *buf = ws + p.buf + j * grows * d.h * d.es, *u = ws + p.u + j * grows * d.f * d.es;
    char *g = ws + p.g + j * grows * d.f * d.es, *o = ws + p.o + j * grows * d.h * d.es;
    TM_TRY(tm_op_linear_fwd(dt, grows, d.f, d.h, buf, par + w1.offset * d.es, b1, nullptr, u, stream));
    TM_TRY(tm_op_act_fwd(dt, cfg->act, grows, d.f, u, g, stream));
    TM_TRY(tm_op_linear_fwd(dt, grows, d.h, d.f, g, par + w2.offset * d.es, b2, nullptr, o, stream));
  }
  g_last_kernel = "moe_combine_kernel";
  if (dt == TM_DTYPE_BF16)
    moe_combine_kernel<bf16><<<(unsigned)d.T, kMoeThreads, 0, s>>>((const bf16 *)(ws + p.o), slot_row, gates, (bf16 *)out, (int)d.h, (int)d.k);
  else
    moe_combine_kernel<float><<<(unsigned)d.T, kMoeThreads, 0, s>>>((const float *)(ws + p.o), slot_row, gates, (float *)out, (int)d.h, (int)d.k);
  return check_launch("moe_fwd combine");
}

extern "C" int tm_moe_bwd(const tm_moe_config_t *cfg, const void *params, const void *c, const void *dout, void *dc,
                          float *grads, int accumulate, void *workspace, int64_t workspace_bytes, void *stream) {
  const void *ptrs[] = {params, c, dout, dc, grads, workspace};
  if (int e = moe_check_call("moe_bwd", cfg, ptrs, 6, workspace_bytes)) return e;
  const MoeDims d = moe_dims(cfg);
  const MoePlan p = moe_plan(cfg);
  int64_t total = 0;
  const std::vector<MoeTensor> tn = moe_tensors(cfg, &total);
  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const char *par = (const char *)params;
  const int dt = cfg->dtype, acc = accumulate ? 1 : 0;
  float *gates = (float *)(ws + p.gates), *dgate = (float *)(ws + p.dgate), *dlog = (float *)(ws + p.dlog);
  int *top_idx = (int *)(ws + p.top_idx), *slot_row = (int *)(ws + p.slot_row), *row_src = (int *)(ws + p.row_src);
  g_last_kernel = "moe_combine_bwd_kernel";
  if (dt == TM_DTYPE_BF16)
    moe_combine_bwd_kernel<bf16><<<(unsigned)d.rows, kMoeThreads, 0, s>>>((const bf16 *)dout, (const bf16 *)(ws + p.o), row_src, gates,
                                                                          (bf16 *)(ws + p.d_o), dgate, (int)d.h, (int)d.k);
  else
    moe_combine_bwd_kernel<float><<<(unsigned)d.rows, kMoeThreads, 0, s>>>((const float *)dout, (const float *)(ws + p.o), row_src, gates,
                                                                           (float *)(ws + p.d_o), dgate, (int)d.h, (int)d.k);
  TM_TRY(check_launch("moe_bwd combine"));
  const int64_t grows = d.ep * d.C;
  const int per = cfg->has_bias ? 4 : 2;
  void *red = ws + p.reduce;
  for (int64_t j = 0; j < d.El; ++j) {
    const MoeTensor &w1 = tn[1 + j * per], &w2 = tn[1 + j * per + (cfg->has_bias ? 2 : 1)];
    char *buf = ws + p.buf + j * grows * d.h * d.es, *u = ws + p.u + j * grows * d.f * d.es;
    char *g = ws + p.g + j * grows * d.f * d.es, *dg = ws + p.dg + j * grows * d.f * d.es;
    char *d_o = ws + p.d_o + j * grows * d.h * d.es, *dbuf = ws + p.dbuf + j * grows * d.h * d.es;
    // o = g W2^T + b2
    TM_TRY(tm_op_linear_dgrad(dt, grows, d.h, d.f, d_o, par + w2.offset * d.es, dg, stream));
    TM_TRY(tm_op_linear_wgrad(dt, grows, d.h, d.f, d_o, g, grads + w2.offset, acc, stream));
    if (cfg->has_bias) TM_TRY(tm_op_bias_grad(dt, grows, d.h, d_o, grads + tn[1 + j * per + 3].offset, red, acc, stream));
    // g = gelu(u): du takes dg's place
    TM_TRY(tm_op_act_bwd(dt, cfg->act, grows, d.f, dg, u, dg, stream));
    // u = buf W1^T + b1
    TM_TRY(tm_op_linear_dgrad(dt, grows, d.f, d.h, dg, par + w1.offset * d.es, dbuf, stream));
    TM_TRY(tm_op_linear_wgrad(dt, grows, d.f, d.h, dg, buf, grads + w1.offset, acc, stream));
    if (cfg->has_bias) TM_TRY(tm_op_bias_grad(dt, grows, d.f, dg, grads + tn[1 + j * per + 1].offset, red, acc, stream));
  }
  const int wg_lds = (int)(d.E * kMoeThreads * 4) + kWgradSegTokens * kMoeMaxTopK * 8;
  const dim3 wg_grid((unsigned)ceil_div(d.h, kMoeThreads), (unsigned)p.wr_segs);
  float *wr_part = (float *)(ws + p.wr_part);
  g_last_kernel = "moe_dispatch_bwd_kernel";
  if (dt == TM_DTYPE_BF16) {
    moe_dispatch_bwd_kernel<bf16><<<(unsigned)d.T, kMoeThreads, 0, s>>>((const bf16 *)(ws + p.dbuf), (const bf16 *)par, slot_row, top_idx,
                                                                        gates, dgate, dlog, (bf16 *)dc, (int)d.h, (int)d.k);
    TM_TRY(set_lds(moe_router_wgrad_kernel<bf16>, wg_lds, "moe_bwd"));
    moe_router_wgrad_kernel<bf16><<<wg_grid, kMoeThreads, wg_lds, s>>>((const bf16 *)c, top_idx, dlog, wr_part, (int)d.T, (int)d.h,
                                                                       (int)d.E, (int)d.k);
  } else {
    moe_dispatch_bwd_kernel<float><<<(unsigned)d.T, kMoeThreads, 0, s>>>((const float *)(ws + p.dbuf), (const float *)par, slot_row,
                                                                         top_idx, gates, dgate, dlog, (float *)dc, (int)d.h, (int)d.k);
    TM_TRY(set_lds(moe_router_wgrad_kernel<float>, wg_lds, "moe_bwd"));
    moe_router_wgrad_kernel<float><<<wg_grid, kMoeThreads, wg_lds, s>>>((const float *)c, top_idx, dlog, wr_part, (int)d.T, (int)d.h,
                                                                        (int)d.E, (int)d.k);
  }
  moe_router_wgrad_reduce_kernel<<<(unsigned)ceil_div(d.E * d.h, kMoeThreads), kMoeThreads, 0, s>>>(wr_part, grads, d.E * d.h,
                                                                                                    (int)p.wr_segs, acc);
  return check_launch("moe_bwd router");
}

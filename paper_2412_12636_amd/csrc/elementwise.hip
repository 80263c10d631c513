// Activation (GeLU / SwiGLU) forward and backward, rotary positions, fused Adam.
// All HBM-bound: 16-byte accesses, fp32 arithmetic.
#include <math.h>

#include <mutex>

#include "adam.h"
#include "common.h"
#include "../../include/tm_ops.h"

namespace tmk {

constexpr int kEwThreads = 256;

__device__ __forceinline__ float gelu_tanh_f(float u) {
  const float k = 0.7978845608028654f;  // sqrt(2/pi)
  return 0.5f * u * (1.f + tanhf(k * (u + 0.044715f * u * u * u)));
}
__device__ __forceinline__ float gelu_tanh_grad_f(float u) {
  const float k = 0.7978845608028654f;
  const float th = tanhf(k * (u + 0.044715f * u * u * u));
  return 0.5f * (1.f + th) + 0.5f * u * (1.f - th * th) * k * (1.f + 0.134145f * u * u);
}
__device__ __forceinline__ float gelu_erf_f(float u) { return 0.5f * u * (1.f + erff(u * 0.7071067811865476f)); }
__device__ __forceinline__ float gelu_erf_grad_f(float u) {
  const float pdf = 0.3989422804014327f * expf(-0.5f * u * u);
  return 0.5f * (1.f + erff(u * 0.7071067811865476f)) + u * pdf;
}
__device__ __forceinline__ float sigmoid_f(float z) { return 1.f / (1.f + expf(-z)); }

// g = gelu(u), chunked over the flat array
template <typename T, int ACT>
__global__ __launch_bounds__(kEwThreads) void gelu_fwd_kernel(const T *__restrict__ u, T *__restrict__ g,
                                                             int64_t nchunk) {
  constexpr int VN = Vec<T>::N;
  for (int64_t ch = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; ch < nchunk;
       ch += (int64_t)gridDim.x * kEwThreads) {
    float a[VN];
    load_vec<T>(u + ch * VN, a);
#pragma unroll
    for (int i = 0; i < VN; ++i) a[i] = (ACT == TM_ACT_GELU_TANH) ? gelu_tanh_f(a[i]) : gelu_erf_f(a[i]);
    store_vec<T>(g + ch * VN, a);
  }
}

// du = dg * gelu'(u); du may alias dg
template <typename T, int ACT>
__global__ __launch_bounds__(kEwThreads) void gelu_bwd_kernel(const T *dg, const T *__restrict__ u, T *du,
                                                             int64_t nchunk) {
  constexpr int VN = Vec<T>::N;
  for (int64_t ch = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; ch < nchunk;
       ch += (int64_t)gridDim.x * kEwThreads) {
    float a[VN], d[VN];
    load_vec<T>(u + ch * VN, a);
    load_vec<T>(dg + ch * VN, d);
#pragma unroll
    for (int i = 0; i < VN; ++i)
      d[i] *= (ACT == TM_ACT_GELU_TANH) ? gelu_tanh_grad_f(a[i]) : gelu_erf_grad_f(a[i]);
    store_vec<T>(du + ch * VN, d);
  }
}

// u[T,2f] = [gate | up]  ->  g[T,f] = silu(gate) * up ; chunks_per_row = f / VN
template <typename T>
__global__ __launch_bounds__(kEwThreads) void swiglu_fwd_kernel(const T *__restrict__ u, T *__restrict__ g,
                                                               int64_t nchunk, int chunks_per_row, int f) {
  constexpr int VN = Vec<T>::N;
  for (int64_t ch = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; ch < nchunk;
       ch += (int64_t)gridDim.x * kEwThreads) {
    const int64_t row = ch / chunks_per_row;
    const int col = (int)(ch % chunks_per_row) * VN;
    float a[VN], b[VN];
    load_vec<T>(u + row * 2 * f + col, a);
    load_vec<T>(u + row * 2 * f + f + col, b);
#pragma unroll
    for (int i = 0; i < VN; ++i) a[i] = a[i] * sigmoid_f(a[i]) * b[i];
    store_vec<T>(g + row * f + col, a);
  }
}

template <typename T>
__global__ __launch_bounds__(kEwThreads) void swiglu_bwd_kernel(const T *__restrict__ dg, const T *__restrict__ u,
                                                               T *__restrict__ du, int64_t nchunk,
                                                               int chunks_per_row, int f) {
  constexpr int VN = Vec<T>::N;
  for (int64_t ch = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; ch < nchunk;
       ch += (int64_t)gridDim.x * kEwThreads) {
    const int64_t row = ch / chunks_per_row;
    const int col = (int)(ch % chunks_per_row) * VN;
    float a[VN], b[VN], d[VN], dgate[VN], dup[VN];
    load_vec<T>(u + row * 2 * f + col, a);
    load_vec<T>(u + row * 2 * f + f + col, b);
    load_vec<T>(dg + row * f + col, d);
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      const float sg = sigmoid_f(a[i]);
      dup[i] = d[i] * a[i] * sg;
      dgate[i] = d[i] * b[i] * sg * (1.f + a[i] * (1.f - sg));
    }
    store_vec<T>(du + row * 2 * f + col, dgate);
    store_vec<T>(du + row * 2 * f + f + col, dup);
  }
}

// One thread per (token row, pair index j): the angle is evaluated once in double precision
// (positions reach 16384, where an fp32 product loses the low bits of the angle) and reused
// for every head of the row.
template <typename T>
__global__ __launch_bounds__(kEwThreads) void rotary_kernel(T *buf, int64_t rows, int batch, int n_heads, int d,
                                                           int row_width, double theta, double sign) {
  const int half = d / 2;
  const int64_t idx = (int64_t)blockIdx.x * kEwThreads + threadIdx.x;
  if (idx >= rows * half) return;
  const int64_t t = idx / half;
  const int j = (int)(idx % half);
  const double pos = (double)(t / batch);
  const double ang = pos * pow(theta, -2.0 * j / d);
  double sd, cd;
  sincos(ang, &sd, &cd);
  const float c = (float)cd, s = (float)(sign * sd);
  T *row = buf + t * row_width;
  for (int hd = 0; hd < n_heads; ++hd) {
    const float lo = to_f32(row[hd * d + j]), hi = to_f32(row[hd * d + j + half]);
    row[hd * d + j] = from_f32<T>(lo * c - hi * s);
    row[hd * d + j + half] = from_f32<T>(hi * c + lo * s);
  }
}

// One wave per block measured 3 % faster than four on this sweep (finer units for the dispatcher).
constexpr int kAdamThreads = 64;

// One 16-byte chunk of each array per thread, blocks in address order (no grid-stride loop: with a
// long stride the HBM channels see scattered pages and the rate drops by a fifth), streaming
// (non-temporal) accesses since nothing is re-read.  Reads g,p,m,v; writes p,m,v (+ bf16 p, + zeroed g).
template <bool LOWP, bool ZERO>
__device__ __forceinline__ void adam_chunk(float *__restrict__ p, float *__restrict__ g, float *__restrict__ m,
                                           float *__restrict__ v, bf16 *__restrict__ p_lowp, int64_t n, int64_t i,
                                           const AdamScalars &a) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
  const int64_t nvec = n / 4;
  if (i < nvec) {
    f32x4 pv = __builtin_nontemporal_load(reinterpret_cast<f32x4 *>(p) + i);
    f32x4 gv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(g) + i);
    f32x4 mv = __builtin_nontemporal_load(reinterpret_cast<f32x4 *>(m) + i);
    f32x4 vv = __builtin_nontemporal_load(reinterpret_cast<f32x4 *>(v) + i);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float pk = pv[k], mk = mv[k], vk = vv[k];
      adam_one(pk, gv[k], mk, vk, a);
      pv[k] = pk;
      mv[k] = mk;
      vv[k] = vk;
    }
    __builtin_nontemporal_store(pv, reinterpret_cast<f32x4 *>(p) + i);
    __builtin_nontemporal_store(mv, reinterpret_cast<f32x4 *>(m) + i);
    __builtin_nontemporal_store(vv, reinterpret_cast<f32x4 *>(v) + i);
    if (LOWP) {
      bf16x4 lo;
#pragma unroll
      for (int k = 0; k < 4; ++k) lo[k] = (bf16)pv[k];
      __builtin_nontemporal_store(lo, reinterpret_cast<bf16x4 *>(p_lowp) + i);
    }
    if (ZERO) __builtin_nontemporal_store(f32x4{0.f, 0.f, 0.f, 0.f}, reinterpret_cast<f32x4 *>(g) + i);
  }
  // tail (n not a multiple of 4): the first threads of the grid
  const int64_t tail = nvec * 4 + i;
  if (tail < n) {
    float pk = p[tail], mk = m[tail], vk = v[tail];
    adam_one(pk, g[tail], mk, vk, a);
    p[tail] = pk;
    m[tail] = mk;
    v[tail] = vk;
    if (LOWP) p_lowp[tail] = (bf16)pk;
    if (ZERO) g[tail] = 0.f;
  }
}
template <bool LOWP, bool ZERO>
__global__ __launch_bounds__(kAdamThreads) void adam_kernel(float *__restrict__ p, float *__restrict__ g,
                                                         float *__restrict__ m, float *__restrict__ v,
                                                         bf16 *__restrict__ p_lowp, int64_t n, AdamScalars a) {
  adam_chunk<LOWP, ZERO>(p, g, m, v, p_lowp, n, (int64_t)blockIdx.x * kAdamThreads + threadIdx.x, a);
}
// The same update over several stretches of one state in one launch (the short vectors between the matrices of a
// layer): block b serves the stretch whose block range holds it.
template <bool LOWP, bool ZERO>
__global__ __launch_bounds__(kAdamThreads) void adam_segments_kernel(float *__restrict__ p, float *__restrict__ g,
                                                                  float *__restrict__ m, float *__restrict__ v,
                                                                  bf16 *__restrict__ p_lowp, AdamSegments segs, AdamScalars a) {
  int sidx = 0;
#pragma unroll
  for (int q = 1; q < kAdamMaxSegments; ++q)
    if (q < segs.n && (int)blockIdx.x >= segs.block0[q]) sidx = q;
  const int64_t first = segs.first[sidx], n = segs.count[sidx];
  const int64_t i = (int64_t)((int)blockIdx.x - segs.block0[sidx]) * kAdamThreads + threadIdx.x;
  adam_chunk<LOWP, ZERO>(p + first, g + first, m + first, v + first, LOWP ? p_lowp + first : nullptr, n, i, a);
}

// one chunk per thread, blocks in address order (see adam_kernel); the kernels' loops run once
static unsigned ew_grid(int64_t nchunk) {
  const int64_t blocks = ceil_div(nchunk, kEwThreads);
  return (unsigned)(blocks > 0 ? blocks : 1);
}

}  // namespace tmk

using namespace tmk;

static int check_ew(const char *what, int dtype, int64_t T, int64_t f) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "%s: unknown dtype %d", what, dtype);
  if (T <= 0 || f <= 0) return fail(TM_EINVAL, "%s: empty shape [%lld, %lld]", what, (long long)T, (long long)f);
  if (f % 8) return fail(TM_ESIZE, "%s: row width %lld is not a multiple of 8", what, (long long)f);
  return TM_OK;
}

extern "C" int tm_op_act_fwd(int dtype, int act, int64_t T, int64_t f, const void *u, void *g, void *stream) {
  if (int e = check_ew("act_fwd", dtype, T, f)) return e;
  if (!u || !g) return fail(TM_EINVAL, "act_fwd: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  const int vn = dtype == TM_DTYPE_BF16 ? 8 : 4;
  const int64_t nchunk = T * f / vn;
  const unsigned grid = ew_grid(nchunk);
  g_last_kernel = act == TM_ACT_SWIGLU ? "swiglu_fwd_kernel" : "gelu_fwd_kernel";
#define TM_LAUNCH(TT)                                                                                              \
  if (act == TM_ACT_GELU_TANH)                                                                                     \
    gelu_fwd_kernel<TT, TM_ACT_GELU_TANH><<<grid, kEwThreads, 0, s>>>((const TT *)u, (TT *)g, nchunk);             \
  else if (act == TM_ACT_GELU_ERF)                                                                                 \
    gelu_fwd_kernel<TT, TM_ACT_GELU_ERF><<<grid, kEwThreads, 0, s>>>((const TT *)u, (TT *)g, nchunk);              \
  else if (act == TM_ACT_SWIGLU)                                                                                   \
    swiglu_fwd_kernel<TT><<<grid, kEwThreads, 0, s>>>((const TT *)u, (TT *)g, nchunk, (int)(f / vn), (int)f);      \
  else                                                                                                             \
    return fail(TM_EINVAL, "act_fwd: unknown activation %d", act);
  if (dtype == TM_DTYPE_BF16) {
    TM_LAUNCH(bf16)
  } else {
    TM_LAUNCH(float)
  }
#undef TM_LAUNCH
  return check_launch("act_fwd");
}

extern "C" int tm_op_act_bwd(int dtype, int act, int64_t T, int64_t f, const void *dg, const void *u, void *du,
                             void *stream) {
  if (int e = check_ew("act_bwd", dtype, T, f)) return e;
  if (!u || !dg || !du) return fail(TM_EINVAL, "act_bwd: NULL pointer");
  if (act == TM_ACT_SWIGLU && dg == du) return fail(TM_EINVAL, "act_bwd: du may not alias dg under SwiGLU");
  hipStream_t s = (hipStream_t)stream;
  const int vn = dtype == TM_DTYPE_BF16 ? 8 : 4;
  const int64_t nchunk = T * f / vn;
  const unsigned grid = ew_grid(nchunk);
  g_last_kernel = act == TM_ACT_SWIGLU ? "swiglu_bwd_kernel" : "gelu_bwd_kernel";
#define TM_LAUNCH(TT)                                                                                              \
  if (act == TM_ACT_GELU_TANH)                                                                                     \
    gelu_bwd_kernel<TT, TM_ACT_GELU_TANH><<<grid, kEwThreads, 0, s>>>((const TT *)dg, (const TT *)u, (TT *)du,     \
                                                                      nchunk);                                    \
  else if (act == TM_ACT_GELU_ERF)                                                                                 \
    gelu_bwd_kernel<TT, TM_ACT_GELU_ERF><<<grid, kEwThreads, 0, s>>>((const TT *)dg, (const TT *)u, (TT *)du,      \
                                                                     nchunk);                                     \
  else if (act == TM_ACT_SWIGLU)                                                                                   \
    swiglu_bwd_kernel<TT><<<grid, kEwThreads, 0, s>>>((const TT *)dg, (const TT *)u, (TT *)du, nchunk,             \
                                                      (int)(f / vn), (int)f);                                     \
  else                                                                                                             \
    return fail(TM_EINVAL, "act_bwd: unknown activation %d", act);
  if (dtype == TM_DTYPE_BF16) {
    TM_LAUNCH(bf16)
  } else {
    TM_LAUNCH(float)
  }
#undef TM_LAUNCH
  return check_launch("act_bwd");
}

extern "C" int tm_op_rotary(int dtype, int64_t seq, int64_t batch, int64_t n_heads, int64_t d, int64_t row_width,
                            double theta, int inverse, void *buf, void *stream) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "rotary: unknown dtype %d", dtype);
  if (seq <= 0 || batch <= 0 || n_heads <= 0 || d <= 0 || !buf) return fail(TM_EINVAL, "rotary: bad argument");
  if (d % 2 || n_heads * d > row_width) return fail(TM_ESIZE, "rotary: heads do not fit the row");
  if (!(theta > 0.0)) return fail(TM_EINVAL, "rotary: theta must be positive");
  hipStream_t s = (hipStream_t)stream;
  const int64_t rows = seq * batch;
  const int64_t n = rows * (d / 2);
  const unsigned grid = (unsigned)ceil_div(n, kEwThreads);
  const double sign = inverse ? -1.0 : 1.0;
  g_last_kernel = "rotary_kernel";
  if (dtype == TM_DTYPE_BF16)
    rotary_kernel<bf16><<<grid, kEwThreads, 0, s>>>((bf16 *)buf, rows, (int)batch, (int)n_heads, (int)d,
                                                    (int)row_width, theta, sign);
  else
    rotary_kernel<float><<<grid, kEwThreads, 0, s>>>((float *)buf, rows, (int)batch, (int)n_heads, (int)d,
                                                     (int)row_width, theta, sign);
  return check_launch("rotary");
}

// ---- squared norm of a gradient vector ------------------------------------------------------------
// Two passes in a fixed order (reproducible): a block squares and adds 4096 consecutive elements (fp32 per
// thread over its 16, fp64 from there on) and writes one partial; one block adds the partials.
namespace tmk {
constexpr int kSqBlockElems = 4096;

__device__ __forceinline__ double block_sum_f64(double x, double *red) {  // 256 or 1024 threads; result in thread 0
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  const int w = threadIdx.x / kWave, l = threadIdx.x % kWave, nw = blockDim.x / kWave;
  if (l == 0) red[w] = x;
  __syncthreads();
  double s = 0.0;
  if (threadIdx.x == 0)
    for (int i = 0; i < nw; ++i) s += red[i];
  return s;
}

__global__ __launch_bounds__(256) void sq_sum_partial_kernel(const float *__restrict__ g, int64_t n, double *__restrict__ part) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  __shared__ double red[4];
  const int64_t base = (int64_t)blockIdx.x * kSqBlockElems;
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = base + (u * 256 + threadIdx.x) * 4;
    if (i + 4 <= n) {
      const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(g + i));
      acc += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    } else {
      for (int64_t j = i; j < n; ++j) acc += g[j] * g[j];
    }
  }
  const double s = block_sum_f64((double)acc, red);
  if (threadIdx.x == 0) part[blockIdx.x] = s;
}

__global__ __launch_bounds__(1024) void sq_sum_final_kernel(const double *__restrict__ part, int64_t nparts, double *__restrict__ out) {
  __shared__ double red[16];
  double acc = 0.0;
  for (int64_t i = threadIdx.x; i < nparts; i += 1024) acc += part[i];
  const double s = block_sum_f64(acc, red);
  if (threadIdx.x == 0) out[0] = s;
}
}  // namespace tmk

extern "C" int64_t tm_sq_sum_scratch_bytes(int64_t n) {
  if (n < 0) return TM_EINVAL;
  return ceil_div(n > 0 ? n : 1, (int64_t)kSqBlockElems) * (int64_t)sizeof(double);
}

extern "C" int tm_sq_sum(int64_t n, const float *g, void *scratch, double *out, void *stream) {
  if (n < 0) return fail(TM_EINVAL, "sq_sum: negative length");
  if (!g || !scratch || !out) return fail(TM_EINVAL, "sq_sum: NULL pointer");
  if ((((uintptr_t)g) & 15) || (((uintptr_t)scratch) & 7) || (((uintptr_t)out) & 7))
    return fail(TM_EALIGN, "sq_sum: g must be 16-byte, scratch and out 8-byte aligned");
  const int64_t blocks = ceil_div(n > 0 ? n : 1, (int64_t)kSqBlockElems);
  if (blocks > 0x7fffffffLL) return fail(TM_ESIZE, "sq_sum: vector too long");
  hipStream_t s = (hipStream_t)stream;
  g_last_kernel = "sq_sum_partial_kernel";
  sq_sum_partial_kernel<<<(unsigned)blocks, 256, 0, s>>>(g, n, (double *)scratch);
  sq_sum_final_kernel<<<1, 1024, 0, s>>>((const double *)scratch, blocks, out);
  return check_launch("sq_sum");
}

// ---- the same reduction for callers that cannot allocate ----------------------------------------------
// The block partials live in a file-scope device array instead of caller memory.  Each GPU holds its own copy of the
// array at its own address; the address is asked for once per device, with that device current, and host code
// uses that pointer, never the array's name (which on the host is only a stand-in for the symbol).
namespace tmk {
constexpr int64_t kSqStaticParts = 1 << 20;  // 8 MiB of partials: 2^20 blocks of 4096 elements
constexpr int kSqMaxDevices = 64;
}  // namespace tmk
static __device__ __align__(256) double scratch[tmk::kSqStaticParts];
static double *g_sq_scratch_ptr[tmk::kSqMaxDevices];  // per device, filled on first use
static std::mutex g_sq_scratch_mutex;

extern "C" int64_t tm_sq_sum_static_max_elems(void) { return kSqStaticParts * (int64_t)kSqBlockElems; }

extern "C" int tm_sq_sum_static(int64_t n, const float *g, double *out, void *stream) {
  if (n < 0) return fail(TM_EINVAL, "sq_sum_static: negative length");
  if (!g || !out) return fail(TM_EINVAL, "sq_sum_static: NULL pointer");
  if ((((uintptr_t)g) & 15) || (((uintptr_t)out) & 7)) return fail(TM_EALIGN, "sq_sum_static: g must be 16-byte, out 8-byte aligned");
  const int64_t blocks = ceil_div(n > 0 ? n : 1, (int64_t)kSqBlockElems);
  if (blocks > kSqStaticParts)
    return fail(TM_ESIZE, "sq_sum_static: %lld elements, the built-in scratch holds the partials of at most %lld",
                (long long)n, (long long)(kSqStaticParts * (int64_t)kSqBlockElems));
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kSqMaxDevices) {
    (void)hipGetLastError();
    return fail(TM_EARCH, "sq_sum_static: no current device below %d", kSqMaxDevices);
  }
  double *part = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_sq_scratch_mutex);
    if (!g_sq_scratch_ptr[dev]) {
      void *sym = nullptr;
      const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !sym) {
        (void)hipGetLastError();
        return fail(TM_ELAUNCH, "sq_sum_static: address of the built-in scratch on device %d: %s", dev, hipGetErrorString(e));
      }
      g_sq_scratch_ptr[dev] = (double *)sym;
    }
    part = g_sq_scratch_ptr[dev];
  }
  // nothing has to start at zero: the first kernel writes partials [0, blocks) and the second reads exactly those
  hipStream_t s = (hipStream_t)stream;
  g_last_kernel = "sq_sum_partial_kernel";
  sq_sum_partial_kernel<<<(unsigned)blocks, 256, 0, s>>>(g, n, part);
  sq_sum_final_kernel<<<1, 1024, 0, s>>>(part, blocks, out);
  return check_launch("sq_sum_static");
}

namespace tmk {
int adam_launch(int64_t n, float *p, float *g, float *m, float *v, void *p_bf16, const tm_adam_hparams_t *hp, int64_t step,
                hipStream_t s) {
  if (!hp || !p || !g || !m || !v) return fail(TM_EINVAL, "adam: NULL pointer");
  if (n < 0) return fail(TM_EINVAL, "adam: negative length");
  if (step < 1) return fail(TM_EINVAL, "adam: step must be >= 1 (got %lld)", (long long)step);
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0 && hp->beta2 >= 0.0 && hp->beta2 < 1.0))
    return fail(TM_EINVAL, "adam: betas must lie in [0, 1)");
  if (((uintptr_t)p | (uintptr_t)g | (uintptr_t)m | (uintptr_t)v) & 15 || ((uintptr_t)p_bf16 & 7))
    return fail(TM_EALIGN, "adam: arrays must be 16-byte aligned");
  if (n == 0) return TM_OK;
  const AdamScalars a = make_adam_scalars(hp, step);
  const bool lowp = p_bf16 != nullptr, zero = hp->zero_grads != 0;
  g_last_kernel = "adam_kernel";
  const int64_t nchunk = n / 4 > 0 ? n / 4 : 1;
  if (ceil_div(nchunk, (int64_t)kAdamThreads) > 0x7fffffffLL) return fail(TM_ESIZE, "adam: array too long for one launch");
  const unsigned grid = (unsigned)ceil_div(nchunk, (int64_t)kAdamThreads);
  if (lowp && zero)
    adam_kernel<true, true><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, (bf16 *)p_bf16, n, a);
  else if (lowp)
    adam_kernel<true, false><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, (bf16 *)p_bf16, n, a);
  else if (zero)
    adam_kernel<false, true><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, nullptr, n, a);
  else
    adam_kernel<false, false><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, nullptr, n, a);
  return check_launch("adam");
}
// n_seg stretches [first[i], first[i] + count[i]) of one state, in one launch where they are few and aligned
int adam_launch_segments(int n_seg, const int64_t *first, const int64_t *count, float *p, float *g, float *m, float *v,
                         void *p_bf16, const tm_adam_hparams_t *hp, int64_t step, hipStream_t s) {
  bool one = n_seg >= 1 && n_seg <= kAdamMaxSegments;
  int64_t blocks = 0;
  for (int i = 0; one && i < n_seg; ++i) {
    if (first[i] % 4 || count[i] <= 0) one = false;
    else blocks += ceil_div(count[i] / 4 > 0 ? count[i] / 4 : 1, (int64_t)kAdamThreads);
  }
  if (!one || blocks > 0x7fffffffLL) {  // one launch each
    for (int i = 0; i < n_seg; ++i) {
      if (count[i] <= 0) continue;
      if (int e = adam_launch(count[i], p + first[i], g + first[i], m + first[i], v + first[i],
                              p_bf16 ? (char *)p_bf16 + first[i] * 2 : nullptr, hp, step, s))
        return e;
    }
    return TM_OK;
  }
  if (!hp || !p || !g || !m || !v) return fail(TM_EINVAL, "adam: NULL pointer");
  if (step < 1) return fail(TM_EINVAL, "adam: step must be >= 1 (got %lld)", (long long)step);
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0 && hp->beta2 >= 0.0 && hp->beta2 < 1.0))
    return fail(TM_EINVAL, "adam: betas must lie in [0, 1)");
  if (((uintptr_t)p | (uintptr_t)g | (uintptr_t)m | (uintptr_t)v) & 15 || ((uintptr_t)p_bf16 & 7))
    return fail(TM_EALIGN, "adam: arrays must be 16-byte aligned");
  AdamSegments segs = {};
  segs.n = n_seg;
  int b0 = 0;
  for (int i = 0; i < n_seg; ++i) {
    segs.first[i] = first[i];
    segs.count[i] = count[i];
    segs.block0[i] = b0;
    b0 += (int)ceil_div(count[i] / 4 > 0 ? count[i] / 4 : 1, (int64_t)kAdamThreads);
  }
  const AdamScalars a = make_adam_scalars(hp, step);
  const bool lowp = p_bf16 != nullptr, zero = hp->zero_grads != 0;
  g_last_kernel = "adam_segments_kernel";
  if (lowp && zero)
    adam_segments_kernel<true, true><<<(unsigned)b0, kAdamThreads, 0, s>>>(p, g, m, v, (bf16 *)p_bf16, segs, a);
  else if (lowp)
    adam_segments_kernel<true, false><<<(unsigned)b0, kAdamThreads, 0, s>>>(p, g, m, v, (bf16 *)p_bf16, segs, a);
  else if (zero)
    adam_segments_kernel<false, true><<<(unsigned)b0, kAdamThreads, 0, s>>>(p, g, m, v, nullptr, segs, a);
  else
    adam_segments_kernel<false, false><<<(unsigned)b0, kAdamThreads, 0, s>>>(p, g, m, v, nullptr, segs, a);
  return check_launch("adam_segments");
}
}  // namespace tmk

extern "C" int tm_adam_step_flat(int64_t n, float *p, float *g, float *m, float *v, void *p_bf16,
                                 const tm_adam_hparams_t *hp, int64_t step, void *stream) {
  return adam_launch(n, p, g, m, v, p_bf16, hp, step, (hipStream_t)stream);
}

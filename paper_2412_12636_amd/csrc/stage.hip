// Host side of the library: configuration checks, flat parameter layout, workspace plan, and the
// sequencing of one pipeline stage's forward pass, backward pass and Adam step.  No kernels here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <deque>
#include <string>
#include <vector>

#include "attn.h"
#include "common.h"
#include "gemm.h"
#include "sandbox.h"
#include "../../include/tm_ops.h"
#include "../../include/tm_sandbox.h"

namespace tmk {

static thread_local char g_err[512] = "";
thread_local const char *g_last_kernel = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_launch(const char *what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TM_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
  return TM_OK;
}

// ---- parameter layout ------------------------------------------------------------------------------
struct TensorInfo {
  std::string name;
  int64_t offset, rows, cols;
};

struct LayerOffsets {  // element offsets inside one layer's block; -1 = absent
  int64_t norm1_gain, norm1_offset, w_qkv, b_qkv, w_out, b_out, norm2_gain, norm2_offset, w_fc1, b_fc1, w_fc2, b_fc2;
  int64_t total;
};

static int validate(const tm_stage_config_t *c) {
  if (!c) return fail(TM_EINVAL, "config is NULL");
  if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
      c->ffn <= 0 || c->seq <= 0 || c->micro_batch <= 0)
    return fail(TM_EINVAL, "config: every size must be positive");
  if (c->dtype != TM_DTYPE_FP32 && c->dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "config: unknown dtype %d", c->dtype);
  if (c->norm != TM_NORM_LAYERNORM && c->norm != TM_NORM_RMSNORM) return fail(TM_EINVAL, "config: unknown norm %d", c->norm);
  if (c->act < TM_ACT_GELU_TANH || c->act > TM_ACT_SWIGLU) return fail(TM_EINVAL, "config: unknown activation %d", c->act);
  if (c->pos != TM_POS_NONE && c->pos != TM_POS_ROTARY) return fail(TM_EINVAL, "config: unknown position code %d", c->pos);
  if (!(c->norm_eps >= 0.0)) return fail(TM_EINVAL, "config: norm_eps must be >= 0");
  if (c->pos == TM_POS_ROTARY && !(c->rope_theta > 0.0)) return fail(TM_EINVAL, "config: rope_theta must be positive");
  if (c->hidden % 8 || c->head_dim % 8 || c->ffn % 8)
    return fail(TM_ESIZE, "config: hidden, head_dim and ffn must be multiples of 8");
  const int hmax = c->dtype == TM_DTYPE_BF16 ? 16384 : 8192;
  if (c->hidden > hmax) return fail(TM_ESIZE, "config: hidden %d above the limit %d", c->hidden, hmax);
  if (c->head_dim > 256) return fail(TM_ESIZE, "config: head_dim %d above 256", c->head_dim);
  if (c->n_q_heads % c->n_kv_heads) return fail(TM_ESIZE, "config: n_q_heads must be a multiple of n_kv_heads");
  const int64_t T = (int64_t)c->seq * c->micro_batch;
  const int64_t widest = std::max<int64_t>(std::max<int64_t>(c->hidden, 2LL * c->ffn),
                                           (int64_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim);
  if (T * widest >= (1LL << 31) * 8) return fail(TM_ESIZE, "config: seq * micro_batch * width too large");
  if (T > 0x7fffffffLL / 8) return fail(TM_ESIZE, "config: too many tokens");
  // the same condition as the attention entry points: what the matrix-core kernels do not take goes to the
  // plain-ALU kernels, which hold a row of scores in LDS
  if (!attn_mfma_supported(c->dtype, c->head_dim) && c->seq > attn_generic_max_seq())
    return fail(TM_ESIZE, "config: seq above %d needs bf16 with head_dim 128", attn_generic_max_seq());
  return TM_OK;
}

static LayerOffsets layer_offsets(const tm_stage_config_t *c) {
  const int64_t h = c->hidden, A = (int64_t)c->n_q_heads * c->head_dim;
  const int64_t nqkv = (int64_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
  const int64_t f = c->ffn, f1 = c->act == TM_ACT_SWIGLU ? 2 * f : f;
  const bool ln = c->norm == TM_NORM_LAYERNORM, bias = c->has_bias != 0;
  LayerOffsets o;
  int64_t at = 0;
  auto take = [&](bool present, int64_t n) {
    if (!present) return (int64_t)-1;
    const int64_t r = at;
    at += n;
    return r;
  };
  o.norm1_gain = take(true, h);
  o.norm1_offset = take(ln, h);
  o.w_qkv = take(true, nqkv * h);
  o.b_qkv = take(bias, nqkv);
  o.w_out = take(true, h * A);
  o.b_out = take(bias, h);
  o.norm2_gain = take(true, h);
  o.norm2_offset = take(ln, h);
  o.w_fc1 = take(true, f1 * h);
  o.b_fc1 = take(bias, f1);
  o.w_fc2 = take(true, h * f);
  o.b_fc2 = take(bias, h);
  o.total = at;
  return o;
}

static std::vector<TensorInfo> tensor_list(const tm_stage_config_t *c) {
  const LayerOffsets o = layer_offsets(c);
  const int64_t h = c->hidden, A = (int64_t)c->n_q_heads * c->head_dim;
  const int64_t nqkv = (int64_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
  const int64_t f = c->ffn, f1 = c->act == TM_ACT_SWIGLU ? 2 * f : f;
  std::vector<TensorInfo> out;
  for (int l = 0; l < c->n_layers; ++l) {
    const int64_t b = (int64_t)l * o.total;
    auto add = [&](const char *nm, int64_t off, int64_t r, int64_t cc) {
      if (off < 0) return;
      out.push_back({"layer" + std::to_string(l) + "." + nm, b + off, r, cc});
    };
    add("norm1_gain", o.norm1_gain, h, 1);
    add("norm1_offset", o.norm1_offset, h, 1);
    add("w_qkv", o.w_qkv, nqkv, h);
    add("b_qkv", o.b_qkv, nqkv, 1);
    add("w_out", o.w_out, h, A);
    add("b_out", o.b_out, h, 1);
    add("norm2_gain", o.norm2_gain, h, 1);
    add("norm2_offset", o.norm2_offset, h, 1);
    add("w_fc1", o.w_fc1, f1, h);
    add("b_fc1", o.b_fc1, f1, 1);
    add("w_fc2", o.w_fc2, h, f);
    add("b_fc2", o.b_fc2, h, 1);
  }
  return out;
}

// ---- workspace plan --------------------------------------------------------------------------------
struct LayerStash {  // byte offsets into the workspace
  int64_t x, mean1, rstd1, a, qkv, lse, ctx, x1, mean2, rstd2, c, u, g;
};
struct Plan {
  std::vector<LayerStash> layer;
  int64_t dstream[2];  // ping-pong buffers for the gradient of the residual stream, [T,h]
  int64_t dwide;       // [T, max(f1, h)] : dg -> du, later da
  int64_t dmid;        // [T, f]  : dg under SwiGLU (du needs its own buffer)
  int64_t dx1;         // [T, h]
  int64_t dnorm;       // [T, h]  : gradient w.r.t. a norm's output (dc, da)
  int64_t dctx;        // [T, A]
  int64_t dqkv;        // [T, Nqkv]
  int64_t dvec;        // scratch of the attention backward pass
  int64_t reduce;      // scratch of the column reductions
  int64_t splitk;      // fp32 partial results of an input-gradient product whose reduction is split
  int64_t splitk_bytes;
  int64_t total;
};

static Plan make_plan(const tm_stage_config_t *c) {
  const int64_t es = c->dtype == TM_DTYPE_BF16 ? 2 : 4;
  const int64_t T = (int64_t)c->seq * c->micro_batch, h = c->hidden, A = (int64_t)c->n_q_heads * c->head_dim;
  const int64_t nqkv = (int64_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
  const int64_t f = c->ffn, f1 = c->act == TM_ACT_SWIGLU ? 2 * f : f;
  Plan p;
  int64_t at = 0;
  auto take = [&](int64_t bytes) {
    const int64_t r = at;
    at += (bytes + 255) / 256 * 256;
    return r;
  };
  const int64_t stat = (int64_t)c->micro_batch * c->n_q_heads * c->seq * 4;
  p.layer.resize(c->n_layers);
  for (auto &s : p.layer) {
    s.x = take(T * h * es);
    s.mean1 = take(T * 4);
    s.rstd1 = take(T * 4);
    s.a = take(T * h * es);
    s.qkv = take(T * nqkv * es);
    s.lse = take(stat);
    s.ctx = take(T * A * es);
    s.x1 = take(T * h * es);
    s.mean2 = take(T * 4);
    s.rstd2 = take(T * 4);
    s.c = take(T * h * es);
    s.u = take(T * f1 * es);
    s.g = take(T * f * es);
  }
  p.dstream[0] = take(T * h * es);
  p.dstream[1] = take(T * h * es);
  p.dwide = take(T * std::max(f1, h) * es);
  p.dmid = take(T * f * es);
  p.dx1 = take(T * h * es);
  p.dnorm = take(T * h * es);
  p.dctx = take(T * A * es);
  p.dqkv = take(T * nqkv * es);
  p.dvec = take(tm_op_attn_bwd_scratch_bytes(c->dtype, c->seq, c->micro_batch, c->n_q_heads, c->n_kv_heads, c->head_dim));
  const int64_t widest = std::max(std::max(3 * h, f1), std::max(nqkv, h));
  const int64_t n_params = layer_offsets(c).total * c->n_layers;
  p.reduce = take(std::max(tm_op_reduce_scratch_bytes(T, widest), tm_sq_sum_scratch_bytes(n_params)));
  p.splitk_bytes = 0;
  const int64_t lin[4][2] = {{nqkv, h}, {h, A}, {f1, h}, {h, f}};  // (N, K) of the four linear maps
  for (const auto &nk : lin)
    p.splitk_bytes = std::max(p.splitk_bytes, std::max<int64_t>(0, tm_op_linear_dgrad_scratch_bytes(c->dtype, T, nk[0], nk[1])));
  p.splitk = take(p.splitk_bytes);
  p.total = at;
  return p;
}

}  // namespace tmk

using namespace tmk;

// Event-based timing of every step a stage call enqueues (off by default).
struct ProfRecord {
  const char *kernel;
  double flops, bytes;
  hipEvent_t e0, e1;
};
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> pool;  // created on demand, reused after every collect
  size_t used = 0;
  std::vector<ProfRecord> recs;
  hipEvent_t take() {
    if (used == pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[used++];
  }
  void release() {
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
    pool.clear();
    recs.clear();
    used = 0;
  }
};

struct tm_stage {
  Profiler prof;
  tm_stage_config_t cfg;
  tm_stage_buffers_t buf;
  LayerOffsets lo;
  Plan plan;
  int64_t n_params;
  bool have_fwd;
  int grad_mode = TM_GRAD_ADD;
  std::vector<TensorInfo> tensors;
  // backward pass: the weight-gradient products run on a second stream beside the chain of input gradients
  hipStream_t side = nullptr;
  hipEvent_t ev_fork[4] = {nullptr, nullptr, nullptr, nullptr}, ev_join = nullptr;
  // ... and, in tm_stage_bwd_adam, each layer's optimizer update on a third
  hipStream_t opt = nullptr;
  hipEvent_t ev_opt[3] = {nullptr, nullptr, nullptr};
  // record / replay hook called at every collective call site (not owned)
  tm_comm_t *comm = nullptr;
};

static std::deque<std::string> &name_pool() {  // deque: growing it never moves the strings
  static thread_local std::deque<std::string> pool;
  return pool;
}

extern "C" const char *tm_last_error(void) { return g_err; }

extern "C" int64_t tm_stage_param_count(const tm_stage_config_t *cfg) {
  if (int e = validate(cfg)) return e;
  return layer_offsets(cfg).total * cfg->n_layers;
}

extern "C" int64_t tm_stage_workspace_bytes(const tm_stage_config_t *cfg) {
  if (int e = validate(cfg)) return e;
  return make_plan(cfg).total;
}

extern "C" int tm_stage_param_layout(const tm_stage_config_t *cfg, int index, const char **name, int64_t *offset_elems,
                                     int64_t shape[2]) {
  if (int e = validate(cfg)) return e;
  const std::vector<TensorInfo> t = tensor_list(cfg);
  if (index == -1) return (int)t.size();
  if (index < 0 || index >= (int)t.size()) return fail(TM_EINVAL, "param_layout: index %d out of range", index);
  if (name) {
    // names stay valid for the life of the calling thread
    auto &pool = name_pool();
    for (auto &s : pool)
      if (s == t[index].name) {
        *name = s.c_str();
        goto named;
      }
    pool.push_back(t[index].name);
    *name = pool.back().c_str();
  }
named:
  if (offset_elems) *offset_elems = t[index].offset;
  if (shape) {
    shape[0] = t[index].rows;
    shape[1] = t[index].cols;
  }
  return TM_OK;
}

extern "C" int tm_stage_init(const tm_stage_config_t *cfg, const tm_stage_buffers_t *b, tm_stage_t **out) {
  if (!out) return fail(TM_EINVAL, "stage_init: out is NULL");
  *out = nullptr;
  if (int e = validate(cfg)) return e;
  if (!b) return fail(TM_EINVAL, "stage_init: buffers is NULL");
  if (!b->params || !b->grads || !b->exp_avg || !b->exp_avg_sq || !b->workspace)
    return fail(TM_EINVAL, "stage_init: a required buffer is NULL");
  if (cfg->dtype == TM_DTYPE_BF16 && !b->master) return fail(TM_EINVAL, "stage_init: bf16 stages need master weights");
  const void *ptrs[] = {b->params, b->master, b->grads, b->exp_avg, b->exp_avg_sq, b->workspace};
  for (const void *q : ptrs)
    if (((uintptr_t)q) & 255) return fail(TM_EALIGN, "stage_init: buffers must be 256-byte aligned");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return fail(TM_EARCH, "stage_init: no usable HIP device");
  }
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(TM_EARCH, "stage_init: device is %s, this library is built for gfx950", prop.gcnArchName);
  const Plan plan = make_plan(cfg);
  if (b->workspace_bytes < plan.total)
    return fail(TM_ESIZE, "stage_init: workspace of %lld bytes, %lld needed", (long long)b->workspace_bytes,
                (long long)plan.total);
  tm_stage *st = new tm_stage();
  st->cfg = *cfg;
  st->buf = *b;
  st->lo = layer_offsets(cfg);
  st->plan = plan;
  st->n_params = st->lo.total * cfg->n_layers;
  st->have_fwd = false;
  *out = st;
  return TM_OK;
}

extern "C" void tm_stage_destroy(tm_stage_t *st) {
  if (!st) return;
  st->prof.release();
  for (hipEvent_t e : st->ev_fork)
    if (e) (void)hipEventDestroy(e);
  if (st->ev_join) (void)hipEventDestroy(st->ev_join);
  if (st->side) (void)hipStreamDestroy(st->side);
  for (hipEvent_t e : st->ev_opt)
    if (e) (void)hipEventDestroy(e);
  if (st->opt) (void)hipStreamDestroy(st->opt);
  delete st;
}

extern "C" int tm_stage_grad_mode(tm_stage_t *st, int mode) {
  if (!st) return fail(TM_EINVAL, "grad_mode: NULL handle");
  if (mode < TM_GRAD_ADD || mode > TM_GRAD_TRANSIENT) return fail(TM_EINVAL, "grad_mode: unknown mode %d", mode);
  st->grad_mode = mode;
  return TM_OK;
}

extern "C" int tm_stage_profile_enable(tm_stage_t *st, int enable) {
  if (!st) return fail(TM_EINVAL, "profile_enable: NULL handle");
  st->prof.on = enable != 0;
  if (!enable) st->prof.release();
  return TM_OK;
}

extern "C" int tm_stage_profile_collect(tm_stage_t *st, tm_profile_entry_t *entries, int max_entries) {
  if (!st || (!entries && max_entries > 0)) return fail(TM_EINVAL, "profile_collect: NULL argument");
  Profiler &pr = st->prof;
  int n = 0;
  for (const ProfRecord &r : pr.recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) {
      (void)hipGetLastError();
      return fail(TM_ELAUNCH, "profile_collect: event query failed");
    }
    int k = 0;
    for (; k < n; ++k)
      if (!strcmp(entries[k].kernel, r.kernel)) break;
    if (k == n) {
      if (n == max_entries) continue;  // table full: the remaining kernels are dropped
      entries[n].kernel = r.kernel;
      entries[n].ms = 0.0;
      entries[n].flops = entries[n].bytes = 0.0;
      entries[n].launches = 0;
      ++n;
    }
    entries[k].ms += ms;
    entries[k].flops += r.flops;
    entries[k].bytes += r.bytes;
    entries[k].launches += 1;
  }
  pr.recs.clear();
  pr.used = 0;
  return n;
}

namespace {
struct Dims {
  int64_t T, h, A, nqkv, f, f1, es;
};
Dims dims_of(const tm_stage_config_t &c) {
  Dims d;
  d.T = (int64_t)c.seq * c.micro_batch;
  d.h = c.hidden;
  d.A = (int64_t)c.n_q_heads * c.head_dim;
  d.nqkv = (int64_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  d.f = c.ffn;
  d.f1 = c.act == TM_ACT_SWIGLU ? 2 * d.f : d.f;
  d.es = c.dtype == TM_DTYPE_BF16 ? 2 : 4;
  return d;
}
}  // namespace

#define TM_TRY(expr)          \
  do {                        \
    const int _e = (expr);    \
    if (_e) return _e;        \
  } while (0)

// Runs one step; with profiling on, brackets it with events on the stream and notes its
// algorithmic work (flops for the matrix-core steps, HBM bytes for the streaming ones).
#define TM_STEP(FLOPS, BYTES, expr)                                             \
  do {                                                                          \
    hipEvent_t _e0 = nullptr, _e1 = nullptr;                                    \
    if (st->prof.on) {                                                          \
      _e0 = st->prof.take();                                                    \
      _e1 = st->prof.take();                                                    \
      if (!_e0 || !_e1) return fail(TM_ELAUNCH, "profiler: cannot create events"); \
      (void)hipEventRecord(_e0, s);                                             \
    }                                                                           \
    const int _e = (expr);                                                      \
    if (_e) return _e;                                                          \
    if (st->prof.on) {                                                          \
      (void)hipEventRecord(_e1, s);                                             \
      st->prof.recs.push_back({g_last_kernel, (double)(FLOPS), (double)(BYTES), _e0, _e1}); \
    }                                                                           \
  } while (0)

extern "C" int tm_stage_tune(tm_stage_t *st, void *stream) {
  if (!st) return fail(TM_EINVAL, "stage_tune: NULL handle");
  const tm_stage_config_t &c = st->cfg;
  if (c.dtype != TM_DTYPE_BF16) return TM_OK;  // the fp32 path has one kernel per product
  const Dims d = dims_of(c);
  hipStream_t s = (hipStream_t)stream;
  char *ws = (char *)st->buf.workspace;
  const char *par = (const char *)st->buf.params;
  const LayerOffsets &o = st->lo;
  st->have_fwd = false;  // the stash is about to be overwritten
  const int64_t wide = std::max(std::max(d.h, d.f1), d.nqkv);
  const int64_t in_a = 0, in_b = (d.T * wide * 2 + 255) / 256 * 256, out = 2 * in_b;
  struct Lin {
    int64_t N, K, w;
  } lins[4] = {{d.nqkv, d.h, o.w_qkv}, {d.h, d.A, o.w_out}, {d.f1, d.h, o.w_fc1}, {d.h, d.f, o.w_fc2}};
  // Weights: every layer's own (cold in the real sequence, so cold here).  Activations and results: the
  // same workspace region every time (just written by the previous step in the real sequence).
  std::vector<GemmArgs> v((size_t)c.n_layers);
  for (const Lin &l : lins) {
    auto weights = [&](int layer) -> const void * { return par + ((int64_t)layer * o.total + l.w) * 2; };
    if (out + d.T * std::max(l.N, l.K) * 2 <= st->plan.total) {
      // y = x W^T
      for (int i = 0; i < c.n_layers; ++i)
        v[i] = GemmArgs{d.T, l.N, l.K, ws + in_a, l.K, 1, weights(i), l.K, 1, ws + out, l.N, nullptr, nullptr, 0};
      TM_TRY(gemm_mfma_tune(v.data(), c.n_layers, s));
      // dx = dy W
      for (int i = 0; i < c.n_layers; ++i)
        v[i] = GemmArgs{d.T, l.K, l.N, ws + in_a, l.N, 1, weights(i), 1, l.K, ws + out, l.K, nullptr, nullptr, 0};
      TM_TRY(gemm_mfma_tune(v.data(), c.n_layers, s));
    }
    // dW = dy^T x; the results rotate through as many separate regions as the workspace holds
    const int64_t dw_bytes = (l.N * l.K * 4 + 255) / 256 * 256;
    const int n_out = (int)std::min<int64_t>((st->plan.total - out) / dw_bytes, c.n_layers);
    if (n_out > 0) {
      for (int i = 0; i < n_out; ++i)
        v[i] = GemmArgs{l.N, l.K, d.T, ws + in_a, 1, l.N, ws + in_b, 1, l.K, ws + out + i * dw_bytes, l.K, nullptr, nullptr, 2};
      TM_TRY(gemm_mfma_tune(v.data(), n_out, s));
    }
  }
  return TM_OK;
}

extern "C" int tm_stage_fwd(tm_stage_t *st, const void *x_in, void *y_out, void *stream) {
  if (!st || !x_in || !y_out) return fail(TM_EINVAL, "stage_fwd: NULL argument");
  if ((((uintptr_t)x_in) | ((uintptr_t)y_out)) & 255) return fail(TM_EALIGN, "stage_fwd: tensors must be 256-byte aligned");
  const tm_stage_config_t &c = st->cfg;
  const Dims d = dims_of(c);
  const int dt = c.dtype;
  char *ws = (char *)st->buf.workspace;
  const char *par = (const char *)st->buf.params;
  hipStream_t s = (hipStream_t)stream;
  st->have_fwd = false;
  const double es = (double)d.es, Th = (double)d.T * d.h;
  const double attn_flops = 2.0 * c.micro_batch * c.n_q_heads * (double)c.seq * c.seq * c.head_dim;  // causal half
  tm_comm_t *cm = st->comm;
  // with the tensor-parallel scope stored or served from the tape, a row-parallel map's partial product must
  // exist on its own: the product runs without its fused epilogue and bias / residual are added after the hook
  const bool tp_cut = comm_intercepts(cm, TM_SCOPE_TP);
  const int64_t act_bytes = d.T * d.h * d.es;
  void *part = ws + st->plan.dx1;  // scratch of the backward pass, free during the forward pass

  for (int l = 0; l < c.n_layers; ++l) {
    const LayerStash &k = st->plan.layer[l];
    const LayerOffsets &o = st->lo;
    const int64_t pb = (int64_t)l * o.total;
    auto P = [&](int64_t off) -> const void * { return off < 0 ? nullptr : par + (pb + off) * d.es; };
    void *x = ws + k.x;
    if (l == 0) {
      g_last_kernel = "copy_stage_input";
      TM_STEP(0, 2 * es * Th,
              hipMemcpyAsync(x, x_in, d.T * d.h * d.es, hipMemcpyDeviceToDevice, s) == hipSuccess
                  ? TM_OK
                  : fail(TM_ELAUNCH, "stage_fwd: copy of the stage input failed"));
      if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_RECV, TM_SCOPE_PP, TM_SITE_X, dt, x, act_bytes, s));
    }
    void *y = (l + 1 < c.n_layers) ? (void *)(ws + st->plan.layer[l + 1].x) : y_out;
    // a = Norm(x)
    TM_STEP(0, 2 * es * Th,
            tm_op_norm_fwd(dt, c.norm, d.T, d.h, c.norm_eps, x, P(o.norm1_gain), P(o.norm1_offset), ws + k.a,
                           (float *)(ws + k.mean1), (float *)(ws + k.rstd1), s));
    // qkv = a Wqkv^T + b
    TM_STEP(2.0 * d.T * d.nqkv * d.h, 0,
            tm_op_linear_fwd(dt, d.T, d.nqkv, d.h, ws + k.a, P(o.w_qkv), P(o.b_qkv), nullptr, ws + k.qkv, s));
    if (c.pos == TM_POS_ROTARY)
      TM_STEP(0, 2 * es * d.T * (c.n_q_heads + c.n_kv_heads) * c.head_dim,
              tm_op_rotary(dt, c.seq, c.micro_batch, c.n_q_heads + c.n_kv_heads, c.head_dim, d.nqkv, c.rope_theta, 0,
                           ws + k.qkv, s));
    TM_STEP(attn_flops, 0,
            tm_op_attn_fwd(dt, c.seq, c.micro_batch, c.n_q_heads, c.n_kv_heads, c.head_dim, ws + k.qkv, ws + k.ctx,
                           (float *)(ws + k.lse), s));
    // x1 = x + ctx Wout^T + b   (row-parallel projection; its all-reduce is the identity here)
    if (!tp_cut) {
      TM_STEP(2.0 * d.T * d.h * d.A, 0,
              tm_op_linear_fwd(dt, d.T, d.h, d.A, ws + k.ctx, P(o.w_out), P(o.b_out), x, ws + k.x1, s));
      if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_ALL_REDUCE, TM_SCOPE_TP, TM_SITE_ATTN_OUT, dt, ws + k.x1, act_bytes, s));
    } else {
      TM_STEP(2.0 * d.T * d.h * d.A, 0, tm_op_linear_fwd(dt, d.T, d.h, d.A, ws + k.ctx, P(o.w_out), nullptr, nullptr, part, s));
      TM_TRY(tm_comm_call(cm, TM_COLL_ALL_REDUCE, TM_SCOPE_TP, TM_SITE_ATTN_OUT, dt, part, act_bytes, s));
      TM_STEP(0, 3 * es * Th, tm_op_bias_residual_add(dt, d.T, d.h, part, P(o.b_out), x, ws + k.x1, s));
    }
    // c = Norm(x1)
    TM_STEP(0, 2 * es * Th,
            tm_op_norm_fwd(dt, c.norm, d.T, d.h, c.norm_eps, ws + k.x1, P(o.norm2_gain), P(o.norm2_offset), ws + k.c,
                           (float *)(ws + k.mean2), (float *)(ws + k.rstd2), s));
    // u = c W1^T + b ; g = act(u)
    TM_STEP(2.0 * d.T * d.f1 * d.h, 0,
            tm_op_linear_fwd(dt, d.T, d.f1, d.h, ws + k.c, P(o.w_fc1), P(o.b_fc1), nullptr, ws + k.u, s));
    TM_STEP(0, es * d.T * (d.f1 + d.f), tm_op_act_fwd(dt, c.act, d.T, d.f, ws + k.u, ws + k.g, s));
    // y = x1 + g W2^T + b
    if (!tp_cut) {
      TM_STEP(2.0 * d.T * d.h * d.f, 0,
              tm_op_linear_fwd(dt, d.T, d.h, d.f, ws + k.g, P(o.w_fc2), P(o.b_fc2), ws + k.x1, y, s));
      if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_ALL_REDUCE, TM_SCOPE_TP, TM_SITE_MLP_OUT, dt, y, act_bytes, s));
    } else {
      TM_STEP(2.0 * d.T * d.h * d.f, 0, tm_op_linear_fwd(dt, d.T, d.h, d.f, ws + k.g, P(o.w_fc2), nullptr, nullptr, part, s));
      TM_TRY(tm_comm_call(cm, TM_COLL_ALL_REDUCE, TM_SCOPE_TP, TM_SITE_MLP_OUT, dt, part, act_bytes, s));
      TM_STEP(0, 3 * es * Th, tm_op_bias_residual_add(dt, d.T, d.h, part, P(o.b_fc2), ws + k.x1, y, s));
    }
  }
  if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_SEND, TM_SCOPE_PP, TM_SITE_Y, dt, y_out, act_bytes, s));
  st->have_fwd = true;
  return TM_OK;
}

static int adam_slice(tm_stage *st, int64_t first, int64_t count, const tm_adam_hparams_t *hp, int64_t step,
                      hipStream_t s) {
  const bool lowp = st->cfg.dtype == TM_DTYPE_BF16;
  float *p = lowp ? st->buf.master : (float *)st->buf.params;
  return adam_launch(count, p + first, st->buf.grads + first, st->buf.exp_avg + first, st->buf.exp_avg_sq + first,
                     lowp ? (char *)st->buf.params + first * 2 : nullptr, hp, step, s);
}

// hp != NULL: every layer's parameters are updated as soon as its gradients are complete
static int stage_bwd(tm_stage_t *st, const void *dy_in, void *dx_out, void *stream, const tm_adam_hparams_t *hp,
                     int64_t step) {
  if (!st || !dy_in || !dx_out) return fail(TM_EINVAL, "stage_bwd: NULL argument");
  if ((((uintptr_t)dy_in) | ((uintptr_t)dx_out)) & 255) return fail(TM_EALIGN, "stage_bwd: tensors must be 256-byte aligned");
  if (!st->have_fwd) return fail(TM_ESTATE, "stage_bwd: no forward pass to differentiate");
  if (hp) {  // before the first launch: a product's fused update would already have written with bad scalars
    if (step < 1) return fail(TM_EINVAL, "stage_bwd_adam: step must be >= 1 (got %lld)", (long long)step);
    if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0 && hp->beta2 >= 0.0 && hp->beta2 < 1.0))
      return fail(TM_EINVAL, "stage_bwd_adam: betas must lie in [0, 1)");
  }
  if (hp && comm_intercepts(st->comm, TM_SCOPE_DP))
    return fail(TM_ESTATE, "stage_bwd_adam: the attached hook intercepts the data-parallel scope; the update must follow tm_stage_grad_sync");
  const tm_stage_config_t &c = st->cfg;
  const Dims d = dims_of(c);
  const int dt = c.dtype;
  char *ws = (char *)st->buf.workspace;
  const char *par = (const char *)st->buf.params;
  float *grads = st->buf.grads;
  hipStream_t s = (hipStream_t)stream;
  const Plan &pl = st->plan;
  void *red = ws + pl.reduce;
  const bool bias = c.has_bias != 0;
  const int acc = st->grad_mode == TM_GRAD_ADD ? 1 : 0;
  const double es = (double)d.es, Th = (double)d.T * d.h;
  const double attn_flops = 2.0 * c.micro_batch * c.n_q_heads * (double)c.seq * c.seq * c.head_dim;
  auto mm = [&](int64_t n, int64_t kk) { return 2.0 * d.T * n * kk; };

  // One stream by default: every product fills the chip, and measured on the 175B shard the forked form below is
  // no faster (the overlapped products contend for the same operand path).  TM_BWD_STREAMS=2 (not while profiling,
  // which times the steps one by one) forks each weight-gradient product, which depends only on tensors the main
  // chain has already produced, onto a side stream; the main stream waits for the side stream before it reuses
  // the scratch buffers (start of the next layer) and before the call returns in stream order.
  const char *streams_env = getenv("TM_BWD_STREAMS");
  bool two = !st->prof.on && streams_env && atoi(streams_env) >= 2;
  if (two && !st->side) {
    bool ok = hipStreamCreateWithFlags(&st->side, hipStreamNonBlocking) == hipSuccess;
    for (hipEvent_t &e : st->ev_fork) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&st->ev_join, hipEventDisableTiming) == hipSuccess;
    if (!ok) return fail(TM_ELAUNCH, "stage_bwd: cannot create the side stream");
  }
  if (two && hp && !st->opt) {
    bool ok = hipStreamCreateWithFlags(&st->opt, hipStreamNonBlocking) == hipSuccess;
    for (hipEvent_t &e : st->ev_opt) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
    if (!ok) return fail(TM_ELAUNCH, "stage_bwd: cannot create the optimizer stream");
  }
  hipStream_t sw = two ? st->side : s;  // the stream of the weight-gradient products
  int n_fork = 0;
  auto fork = [&]() -> int {            // what the main stream has enqueued so far precedes later side work
    if (!two) return TM_OK;
    hipEvent_t e = st->ev_fork[n_fork++ & 3];
    if (hipEventRecord(e, s) != hipSuccess || hipStreamWaitEvent(st->side, e, 0) != hipSuccess)
      return fail(TM_ELAUNCH, "stage_bwd: fork failed");
    return TM_OK;
  };
  auto join = [&]() -> int {            // what the side stream has enqueued so far precedes later main work
    if (!two) return TM_OK;
    if (hipEventRecord(st->ev_join, st->side) != hipSuccess || hipStreamWaitEvent(s, st->ev_join, 0) != hipSuccess)
      return fail(TM_ELAUNCH, "stage_bwd: join failed");
    return TM_OK;
  };

  tm_comm_t *cm = st->comm;
  const int64_t act_bytes = d.T * d.h * d.es;
  // tm_stage_bwd_adam with the gradients in overwrite mode: the update of a weight matrix rides in the epilogue of
  // its weight-gradient product (the gradient is still stored, but never read back, and the state streams while
  // other blocks of the product still multiply); what is left for the flat sweep are the vectors between the
  // matrices.  TM_ADAM_UNFUSED=1 keeps the whole update in the flat sweep.
  const bool fuse = hp && acc == 0 && dt == TM_DTYPE_BF16 && !hp->zero_grads && getenv("TM_ADAM_UNFUSED") == nullptr;
  const AdamScalars ascal = hp ? make_adam_scalars(hp, step) : AdamScalars{};
  struct Range { int64_t first, count; };
  std::vector<Range> fused;  // this layer's matrices already updated, element ranges relative to the layer's block
  // bytes per parameter a weight-gradient product moves besides its operands when the update rides in its epilogue:
  // three fp32 states read and written, the bf16 copy, and the gradient where it is stored
  // (plus the product's two operands, read once)
  const double fused_bytes_per_param = fuse ? 26.0 + (st->grad_mode != TM_GRAD_TRANSIENT ? 4.0 : 0.0) : 0.0;
  auto wgrad_bytes = [&](int64_t N, int64_t K, const void *dyp, const void *xp, int64_t pb, int64_t w_off) -> double {
    return fuse && linear_wgrad_adam_supported(d.T, N, K, dyp, xp, grads + pb + w_off)
               ? fused_bytes_per_param * (double)N * (double)K + es * (double)d.T * (double)(N + K)
               : 0.0;
  };
  auto wgrad = [&](int64_t pb, int64_t w_off, int64_t N, int64_t K, const void *dyp, const void *xp) -> int {
    float *dw = grads + pb + w_off;
    if (fuse && linear_wgrad_adam_supported(d.T, N, K, dyp, xp, dw)) {
      AdamTarget t;
      t.master = st->buf.master + pb + w_off;
      t.exp_avg = st->buf.exp_avg + pb + w_off;
      t.exp_avg_sq = st->buf.exp_avg_sq + pb + w_off;
      t.lowp = (bf16 *)st->buf.params + pb + w_off;
      t.a = ascal;
      t.store_grad = st->grad_mode != TM_GRAD_TRANSIENT;
      fused.push_back({w_off, N * K});
      return linear_wgrad_adam(d.T, N, K, dyp, xp, dw, t, sw);
    }
    return tm_op_linear_wgrad(dt, d.T, N, K, dyp, xp, dw, acc, sw);
  };
  auto run = [&]() -> int {
  const void *dy = dy_in;
  if (cm) {
    void *at = const_cast<void *>(dy_in);
    if (comm_intercepts(cm, TM_SCOPE_PP)) {
      // the received gradient may be replaced: it needs a buffer of the library's own (the one the pattern of
      // alternating gradient streams leaves free for the top layer's input)
      at = ws + pl.dstream[c.n_layers & 1];
      if (hipMemcpyAsync(at, dy_in, (size_t)act_bytes, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return fail(TM_ELAUNCH, "stage_bwd: copy of the incoming gradient failed");
      dy = at;
    }
    TM_TRY(tm_comm_call(cm, TM_COLL_RECV, TM_SCOPE_PP, TM_SITE_DY, dt, at, act_bytes, s));
  }
  for (int l = c.n_layers - 1; l >= 0; --l) {
    TM_TRY(join());  // the layer above is done with the scratch buffers
    const LayerStash &k = pl.layer[l];
    const LayerOffsets &o = st->lo;
    const int64_t pb = (int64_t)l * o.total;
    auto P = [&](int64_t off) -> const void * { return off < 0 ? nullptr : par + (pb + off) * d.es; };
    auto G = [&](int64_t off) -> float * { return off < 0 ? nullptr : grads + pb + off; };
    void *dx = (l == 0) ? dx_out : (void *)(ws + pl.dstream[l & 1]);

    // y = x1 + g W2^T + b2
    void *dg = (c.act == TM_ACT_SWIGLU) ? (void *)(ws + pl.dmid) : (void *)(ws + pl.dwide);
    TM_STEP(mm(d.h, d.f), 0, tm_op_linear_dgrad_ws(dt, d.T, d.h, d.f, dy, P(o.w_fc2), dg, ws + pl.splitk, pl.splitk_bytes, s));
    TM_TRY(fork());
    fused.clear();
    TM_STEP(mm(d.h, d.f), wgrad_bytes(d.h, d.f, dy, ws + k.g, pb, o.w_fc2), wgrad(pb, o.w_fc2, d.h, d.f, dy, ws + k.g));
    // (below the top layer this bias gradient has come out of the first norm's backward pass of the layer above)
    if (bias && l == c.n_layers - 1) TM_STEP(0, es * Th, tm_op_bias_grad(dt, d.T, d.h, dy, G(o.b_fc2), red, acc, s));
    // activation
    void *du = ws + pl.dwide;
    TM_STEP(0, es * d.T * (d.f + 2 * d.f1), tm_op_act_bwd(dt, c.act, d.T, d.f, dg, ws + k.u, du, s));
    // u = c W1^T + b1
    void *dc = ws + pl.dnorm;
    TM_STEP(mm(d.f1, d.h), 0, tm_op_linear_dgrad_ws(dt, d.T, d.f1, d.h, du, P(o.w_fc1), dc, ws + pl.splitk, pl.splitk_bytes, s));
    if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_ALL_REDUCE, TM_SCOPE_TP, TM_SITE_D_MLP_IN, dt, dc, act_bytes, s));
    TM_TRY(fork());
    TM_STEP(mm(d.f1, d.h), wgrad_bytes(d.f1, d.h, du, ws + k.c, pb, o.w_fc1), wgrad(pb, o.w_fc1, d.f1, d.h, du, ws + k.c));
    if (bias) TM_STEP(0, es * d.T * d.f1, tm_op_bias_grad(dt, d.T, d.f1, du, G(o.b_fc1), red, acc, s));
    // c = Norm(x1): dx1 = dy + norm gradient
    void *dx1 = ws + pl.dx1;
    // with biases the column sums of dx1, the out-projection's bias gradient, come out of the same pass
    if (bias)
      TM_STEP(0, 4 * es * Th,
              tm_op_norm_bwd_colsum(dt, c.norm, d.T, d.h, dc, ws + k.x1, (const float *)(ws + k.mean2),
                                    (const float *)(ws + k.rstd2), P(o.norm2_gain), dy, dx1, G(o.norm2_gain),
                                    G(o.norm2_offset), G(o.b_out), red, acc, s));
    else
      TM_STEP(0, 4 * es * Th,
              tm_op_norm_bwd(dt, c.norm, d.T, d.h, dc, ws + k.x1, (const float *)(ws + k.mean2),
                             (const float *)(ws + k.rstd2), P(o.norm2_gain), dy, dx1, G(o.norm2_gain),
                             G(o.norm2_offset), red, acc, s));
    // x1 = x + ctx Wout^T + bout
    TM_STEP(mm(d.h, d.A), 0, tm_op_linear_dgrad_ws(dt, d.T, d.h, d.A, dx1, P(o.w_out), ws + pl.dctx, ws + pl.splitk, pl.splitk_bytes, s));
    TM_TRY(fork());
    TM_STEP(mm(d.h, d.A), wgrad_bytes(d.h, d.A, dx1, ws + k.ctx, pb, o.w_out), wgrad(pb, o.w_out, d.h, d.A, dx1, ws + k.ctx));
    // attention, rotary
    TM_STEP(2 * attn_flops, 0,
            tm_op_attn_bwd(dt, c.seq, c.micro_batch, c.n_q_heads, c.n_kv_heads, c.head_dim, ws + k.qkv, ws + k.ctx,
                           ws + pl.dctx, (const float *)(ws + k.lse), ws + pl.dvec, ws + pl.dqkv, s));
    if (c.pos == TM_POS_ROTARY)
      TM_STEP(0, 2 * es * d.T * (c.n_q_heads + c.n_kv_heads) * c.head_dim,
              tm_op_rotary(dt, c.seq, c.micro_batch, c.n_q_heads + c.n_kv_heads, c.head_dim, d.nqkv, c.rope_theta, 1,
                           ws + pl.dqkv, s));
    // qkv = a Wqkv^T + b
    void *da = ws + pl.dnorm;
    TM_STEP(mm(d.nqkv, d.h), 0, tm_op_linear_dgrad_ws(dt, d.T, d.nqkv, d.h, ws + pl.dqkv, P(o.w_qkv), da, ws + pl.splitk, pl.splitk_bytes, s));
    if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_ALL_REDUCE, TM_SCOPE_TP, TM_SITE_D_ATTN_IN, dt, da, act_bytes, s));
    TM_TRY(fork());
    TM_STEP(mm(d.nqkv, d.h), wgrad_bytes(d.nqkv, d.h, ws + pl.dqkv, ws + k.a, pb, o.w_qkv), wgrad(pb, o.w_qkv, d.nqkv, d.h, ws + pl.dqkv, ws + k.a));
    if (bias) TM_STEP(0, es * d.T * d.nqkv, tm_op_bias_grad(dt, d.T, d.nqkv, ws + pl.dqkv, G(o.b_qkv), red, acc, s));
    // a = Norm(x): dx = dx1 + norm gradient
    // dx is the output gradient of the layer below: its column sums are that layer's FC2 bias gradient
    if (bias && l > 0)
      TM_STEP(0, 4 * es * Th,
              tm_op_norm_bwd_colsum(dt, c.norm, d.T, d.h, da, ws + k.x, (const float *)(ws + k.mean1),
                                    (const float *)(ws + k.rstd1), P(o.norm1_gain), dx1, dx, G(o.norm1_gain),
                                    G(o.norm1_offset), grads + pb - o.total + o.b_fc2, red, acc, s));
    else
      TM_STEP(0, 4 * es * Th,
              tm_op_norm_bwd(dt, c.norm, d.T, d.h, da, ws + k.x, (const float *)(ws + k.mean1),
                             (const float *)(ws + k.rstd1), P(o.norm1_gain), dx1, dx, G(o.norm1_gain),
                             G(o.norm1_offset), red, acc, s));
    dy = dx;
    if (hp) {
      // this layer's gradients: the products on the side stream and the norm / bias gradients on the main one
      hipStream_t so = two ? st->opt : s;
      if (two) {
        if (hipEventRecord(st->ev_opt[0], s) != hipSuccess || hipStreamWaitEvent(st->opt, st->ev_opt[0], 0) != hipSuccess ||
            hipEventRecord(st->ev_opt[1], st->side) != hipSuccess ||
            hipStreamWaitEvent(st->opt, st->ev_opt[1], 0) != hipSuccess)
          return fail(TM_ELAUNCH, "stage_bwd: optimizer fork failed");
      }
      const double per_param = 28.0 + (d.es == 2 ? 2.0 : 0.0) + (hp->zero_grads ? 4.0 : 0.0);
      hipStream_t s_keep = s;
      s = so;  // TM_STEP brackets the stream named s
      // the flat sweep over what the products have not updated: the stretches between the fused matrices
      std::sort(fused.begin(), fused.end(), [](const Range &a, const Range &b) { return a.first < b.first; });
      // (one launch for all of them: the vectors of a layer are a few thousand elements each)
      std::vector<int64_t> seg_first, seg_count;
      int64_t at = 0, left = 0;
      for (size_t i = 0; i <= fused.size(); ++i) {
        const int64_t end = i < fused.size() ? fused[i].first : o.total;
        if (end > at) {
          seg_first.push_back(pb + at);
          seg_count.push_back(end - at);
          left += end - at;
        }
        if (i < fused.size()) at = fused[i].first + fused[i].count;
      }
      if (left > 0) {
        const bool lowp = c.dtype == TM_DTYPE_BF16;
        float *master = lowp ? st->buf.master : (float *)st->buf.params;
        TM_STEP(0, per_param * (double)left,
                adam_launch_segments((int)seg_first.size(), seg_first.data(), seg_count.data(), master, st->buf.grads,
                                     st->buf.exp_avg, st->buf.exp_avg_sq, lowp ? st->buf.params : nullptr, hp, step, so));
      }
      s = s_keep;
    }
  }
  if (hp && two) {
    if (hipEventRecord(st->ev_opt[2], st->opt) != hipSuccess || hipStreamWaitEvent(s, st->ev_opt[2], 0) != hipSuccess)
      return fail(TM_ELAUNCH, "stage_bwd: optimizer join failed");
  }
  TM_TRY(join());
  if (cm) TM_TRY(tm_comm_call(cm, TM_COLL_SEND, TM_SCOPE_PP, TM_SITE_DX, dt, dx_out, act_bytes, s));
  return TM_OK;
  };
  const int rc = run();
  if (rc != TM_OK && two) {
    // a step failed after work was forked: whatever the internal streams still hold must precede later work on the
    // caller's stream (the message of the failure is kept)
    hipStream_t main_stream = (hipStream_t)stream;
    if (hipEventRecord(st->ev_join, st->side) == hipSuccess) (void)hipStreamWaitEvent(main_stream, st->ev_join, 0);
    if (st->opt && hipEventRecord(st->ev_opt[2], st->opt) == hipSuccess) (void)hipStreamWaitEvent(main_stream, st->ev_opt[2], 0);
    (void)hipGetLastError();
  }
  return rc;
}

extern "C" int tm_stage_attach_comm(tm_stage_t *st, tm_comm_t *c) {
  if (!st) return fail(TM_EINVAL, "attach_comm: NULL handle");
  st->comm = c;
  return TM_OK;
}

extern "C" int tm_stage_grad_sync(tm_stage_t *st, void *stream) {
  if (!st) return fail(TM_EINVAL, "grad_sync: NULL handle");
  if (!st->comm) return TM_OK;  // no peers: the local gradient is the reduced one
  TM_TRY(tm_comm_call(st->comm, TM_COLL_ALL_REDUCE, TM_SCOPE_DP, TM_SITE_GRADS, TM_DTYPE_FP32, st->buf.grads, st->n_params * 4, stream));
  return tm_comm_call(st->comm, TM_COLL_BARRIER, TM_SCOPE_DP, TM_SITE_STEP_END, TM_DTYPE_FP32, nullptr, 0, stream);
}

extern "C" int tm_stage_bwd(tm_stage_t *st, const void *dy_in, void *dx_out, void *stream) {
  return stage_bwd(st, dy_in, dx_out, stream, nullptr, 0);
}

extern "C" int tm_stage_bwd_adam(tm_stage_t *st, const void *dy_in, void *dx_out, const tm_adam_hparams_t *hp,
                                 int64_t step, void *stream) {
  if (!hp) return fail(TM_EINVAL, "stage_bwd_adam: NULL hyper-parameters");
  return stage_bwd(st, dy_in, dx_out, stream, hp, step);
}

extern "C" int tm_stage_grad_sq_sum(tm_stage_t *st, double *out, void *stream) {
  if (!st || !out) return fail(TM_EINVAL, "grad_sq_sum: NULL argument");
  hipStream_t s = (hipStream_t)stream;
  TM_STEP(0, 4.0 * (double)st->n_params,
          tm_sq_sum(st->n_params, st->buf.grads, (char *)st->buf.workspace + st->plan.reduce, out, stream));
  return TM_OK;
}

extern "C" int tm_adam_step_range(tm_stage_t *st, int64_t first, int64_t count, const tm_adam_hparams_t *hp,
                                  int64_t step, void *stream) {
  if (!st || !hp) return fail(TM_EINVAL, "adam_step_range: NULL argument");
  if (first < 0 || count < 0 || first + count > st->n_params)
    return fail(TM_EINVAL, "adam_step_range: [%lld, %lld) is outside the %lld parameters", (long long)first,
                (long long)(first + count), (long long)st->n_params);
  if (first % 8) return fail(TM_EALIGN, "adam_step_range: the first element must be a multiple of 8");
  hipStream_t s = (hipStream_t)stream;
  const double per_param = 28.0 + (st->cfg.dtype == TM_DTYPE_BF16 ? 2.0 : 0.0) + (hp->zero_grads ? 4.0 : 0.0);
  TM_STEP(0, per_param * (double)count, adam_slice(st, first, count, hp, step, s));
  return TM_OK;
}

extern "C" int tm_adam_step(tm_stage_t *st, const tm_adam_hparams_t *hp, int64_t step, void *stream) {
  if (!st || !hp) return fail(TM_EINVAL, "adam_step: NULL argument");
  const bool lowp = st->cfg.dtype == TM_DTYPE_BF16;
  float *p = lowp ? st->buf.master : (float *)st->buf.params;
  hipStream_t s = (hipStream_t)stream;
  const double per_param = 28.0 + (lowp ? 2.0 : 0.0) + (hp->zero_grads ? 4.0 : 0.0);
  TM_STEP(0, per_param * (double)st->n_params,
          tm_adam_step_flat(st->n_params, p, st->buf.grads, st->buf.exp_avg, st->buf.exp_avg_sq,
                            lowp ? st->buf.params : nullptr, hp, step, stream));
  return TM_OK;
}

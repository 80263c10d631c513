// Record / replay layer of the communication-free sandbox (section 4.2 of the paper; boundary-only
// scope as in section 4.3): a hook object that every collective call site of the stage goes through.
// Pre-record: the completed call's tensor is copied to the host and appended to a tape file.  Replay:
// the tensor is overwritten from the tape (held in pinned host memory), `send` and `barrier` are
// skipped.  Host code plus one small kernel (bias and residual added after an intercepted all-reduce).
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "common.h"
#include "sandbox.h"
#include "../../include/tm_sandbox.h"

namespace tmk {

constexpr char kMagic[8] = {'T', 'M', 'T', 'A', 'P', 'E', '0', '1'};
constexpr int64_t kStageBytes = 64ll << 20;  // pinned staging buffer of the recorder

struct TapeRecord {  // 64 bytes on disk
  uint32_t kind, scope, site, dtype;
  uint64_t bytes, checksum;
  uint8_t zero[32];
};
static_assert(sizeof(TapeRecord) == 64, "tape record");

// multiply-xor over 64-bit words (tail zero-padded); `c` carries across pieces whose sizes are multiples of 8
static uint64_t checksum_words(uint64_t c, const void *data, int64_t bytes) {
  const uint8_t *p = (const uint8_t *)data;
  int64_t i = 0;
  for (; i + 8 <= bytes; i += 8) {
    uint64_t w;
    memcpy(&w, p + i, 8);
    c = (c ^ w) * 0x100000001b3ull;
  }
  if (i < bytes) {
    uint64_t w = 0;
    memcpy(&w, p + i, (size_t)(bytes - i));
    c = (c ^ w) * 0x100000001b3ull;
  }
  return c;
}
constexpr uint64_t kChecksumSeed = 0xcbf29ce484222325ull;

static int64_t pad64(int64_t n) { return (n + 63) / 64 * 64; }

struct Entry {
  TapeRecord rec;
  int64_t arena_off;
};

}  // namespace tmk

using namespace tmk;

struct tm_comm {
  int mode = TM_COMM_PASS, scopes = 0;
  std::string path;
  FILE *f = nullptr;
  tm_comm_stats_t stats{};
  // record
  void *staging = nullptr;
  // replay
  std::vector<Entry> entries;
  char *arena = nullptr;
  size_t at = 0;
};

namespace tmk {
bool comm_intercepts(const tm_comm *c, int scope) { return c && c->mode != TM_COMM_PASS && (c->scopes & scope) != 0; }
}  // namespace tmk

static void comm_free(tm_comm *c) {
  if (c->f) fclose(c->f);
  if (c->staging) (void)hipHostFree(c->staging);
  if (c->arena) (void)hipHostFree(c->arena);
  delete c;
}

static int load_tape(tm_comm *c) {
  FILE *f = fopen(c->path.c_str(), "rb");
  if (!f) return fail(TM_EINVAL, "comm_open: cannot read tape %s", c->path.c_str());
  c->f = f;
  char magic[8];
  uint64_t count = 0;
  if (fread(magic, 1, 8, f) != 8 || fread(&count, 8, 1, f) != 1 || memcmp(magic, kMagic, 8) != 0)
    return fail(TM_EINVAL, "comm_open: %s is not a tape file", c->path.c_str());
  // pass 1: the records; payloads of scopes off the boundary are skipped, never read
  int64_t total = 0;
  std::vector<long> payload_at;
  for (uint64_t i = 0; i < count; ++i) {
    TapeRecord r;
    if (fread(&r, sizeof(r), 1, f) != 1) return fail(TM_EINVAL, "comm_open: tape ends inside record %llu", (unsigned long long)i);
    if (r.kind > TM_COLL_BARRIER || (int64_t)r.bytes < 0) return fail(TM_EINVAL, "comm_open: record %llu is malformed", (unsigned long long)i);
    const long here = ftell(f);
    if (r.scope & (uint32_t)c->scopes) {
      c->entries.push_back({r, total});
      payload_at.push_back(here);
      total += pad64((int64_t)r.bytes);
    }
    if (fseek(f, here + (long)pad64((int64_t)r.bytes), SEEK_SET) != 0) return fail(TM_EINVAL, "comm_open: seek failed");
  }
  // the file must hold the last payload completely
  fseek(f, 0, SEEK_END);
  const long end = ftell(f);
  for (size_t i = 0; i < c->entries.size(); ++i)
    if (payload_at[i] + (long)c->entries[i].rec.bytes > end) return fail(TM_EINVAL, "comm_open: tape ends inside a payload");
  // pass 2: the boundary's payloads into pinned host memory
  if (total > 0) {
    if (hipHostMalloc((void **)&c->arena, (size_t)total, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      c->arena = nullptr;
      return fail(TM_ELAUNCH, "comm_open: cannot pin %lld bytes of host memory", (long long)total);
    }
  }
  for (size_t i = 0; i < c->entries.size(); ++i) {
    const Entry &e = c->entries[i];
    if (e.rec.bytes == 0) continue;
    char *dst = c->arena + e.arena_off;
    if (fseek(f, payload_at[i], SEEK_SET) != 0 || fread(dst, 1, (size_t)e.rec.bytes, f) != (size_t)e.rec.bytes)
      return fail(TM_EINVAL, "comm_open: cannot read the payload of entry %zu", i);
    if (checksum_words(kChecksumSeed, dst, (int64_t)e.rec.bytes) != e.rec.checksum)
      return fail(TM_ESTATE, "comm_open: checksum of entry %zu does not match its payload", i);
    c->stats.tape_bytes += (int64_t)e.rec.bytes;
  }
  c->stats.tape_entries = (int64_t)c->entries.size();
  fclose(f);
  c->f = nullptr;
  return TM_OK;
}

extern "C" int tm_comm_open(const char *path, int mode, int scopes, tm_comm_t **out) {
  if (!out) return fail(TM_EINVAL, "comm_open: out is NULL");
  *out = nullptr;
  if (mode < TM_COMM_PASS || mode > TM_COMM_REPLAY) return fail(TM_EINVAL, "comm_open: unknown mode %d", mode);
  if (scopes & ~(TM_SCOPE_TP | TM_SCOPE_PP | TM_SCOPE_DP)) return fail(TM_EINVAL, "comm_open: unknown scope bits %d", scopes);
  if (mode != TM_COMM_PASS && !path) return fail(TM_EINVAL, "comm_open: a tape path is required");
  tm_comm *c = new tm_comm();
  c->mode = mode;
  c->scopes = scopes;
  c->path = path ? path : "";
  if (mode == TM_COMM_RECORD) {
    c->f = fopen(path, "wb");
    const uint64_t zero = 0;
    if (!c->f || fwrite(kMagic, 1, 8, c->f) != 8 || fwrite(&zero, 8, 1, c->f) != 1) {
      comm_free(c);
      return fail(TM_EINVAL, "comm_open: cannot create tape %s", path);
    }
  } else if (mode == TM_COMM_REPLAY) {
    if (int e = load_tape(c)) {
      comm_free(c);
      return e;
    }
  }
  *out = c;
  return TM_OK;
}

static int record_call(tm_comm *c, int kind, int scope, int site, int dtype, const void *buf, int64_t bytes, hipStream_t s) {
  if (!c->staging && bytes > 0) {
    if (hipHostMalloc(&c->staging, (size_t)kStageBytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      c->staging = nullptr;
      return fail(TM_ELAUNCH, "comm_call: cannot pin the staging buffer");
    }
  }
  TapeRecord r;
  memset(&r, 0, sizeof(r));
  r.kind = (uint32_t)kind;
  r.scope = (uint32_t)scope;
  r.site = (uint32_t)site;
  r.dtype = (uint32_t)dtype;
  r.bytes = (uint64_t)bytes;
  const long rec_at = ftell(c->f);
  if (fwrite(&r, sizeof(r), 1, c->f) != 1) return fail(TM_ELAUNCH, "comm_call: tape write failed");
  uint64_t sum = kChecksumSeed;
  for (int64_t off = 0; off < bytes; off += kStageBytes) {
    const int64_t n = bytes - off < kStageBytes ? bytes - off : kStageBytes;
    // the call has completed in stream order once this copy has; then the piece goes to the file
    if (hipMemcpyAsync(c->staging, (const char *)buf + off, (size_t)n, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
      (void)hipGetLastError();
      return fail(TM_ELAUNCH, "comm_call: copy to the host failed");
    }
    sum = checksum_words(sum, c->staging, n);
    if (fwrite(c->staging, 1, (size_t)n, c->f) != (size_t)n) return fail(TM_ELAUNCH, "comm_call: tape write failed");
  }
  static const char zeros[64] = {0};
  const int64_t padn = pad64(bytes) - bytes;
  if (padn && fwrite(zeros, 1, (size_t)padn, c->f) != (size_t)padn) return fail(TM_ELAUNCH, "comm_call: tape write failed");
  r.checksum = sum;
  const long end = ftell(c->f);
  if (fseek(c->f, rec_at, SEEK_SET) != 0 || fwrite(&r, sizeof(r), 1, c->f) != 1 || fseek(c->f, end, SEEK_SET) != 0)
    return fail(TM_ELAUNCH, "comm_call: tape write failed");
  c->stats.stored += 1;
  c->stats.stored_bytes += bytes;
  c->stats.tape_entries += 1;
  c->stats.tape_bytes += bytes;
  return TM_OK;
}

extern "C" int tm_comm_call(tm_comm_t *c, int kind, int scope, int site, int dtype, void *buf, int64_t bytes, void *stream) {
  if (!c) return fail(TM_EINVAL, "comm_call: NULL handle");
  if (kind < TM_COLL_ALL_REDUCE || kind > TM_COLL_BARRIER) return fail(TM_EINVAL, "comm_call: unknown kind %d", kind);
  if (scope != TM_SCOPE_TP && scope != TM_SCOPE_PP && scope != TM_SCOPE_DP)
    return fail(TM_EINVAL, "comm_call: scope must be exactly one of the TM_SCOPE_* bits");
  if (bytes < 0 || (bytes > 0 && !buf)) return fail(TM_EINVAL, "comm_call: NULL tensor of %lld bytes", (long long)bytes);
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "comm_call: unknown dtype %d", dtype);
  hipStream_t s = (hipStream_t)stream;
  c->stats.calls += 1;
  if (!comm_intercepts(c, scope)) {
    c->stats.native += 1;  // this rank's tensor is the result
    return TM_OK;
  }
  const bool carries = kind == TM_COLL_ALL_REDUCE || kind == TM_COLL_RECV;
  if (c->mode == TM_COMM_RECORD) {
    if (!carries) {
      c->stats.native += 1;
      return TM_OK;
    }
    return record_call(c, kind, scope, site, dtype, buf, bytes, s);
  }
  // replay
  if (!carries) {
    c->stats.skipped += 1;  // send / barrier: the caller's state does not depend on them
    return TM_OK;
  }
  if (c->at >= c->entries.size()) return fail(TM_ESTATE, "comm_call: the tape has no entry left (call %lld)", (long long)c->stats.calls);
  const Entry &e = c->entries[c->at];
  if (e.rec.kind != (uint32_t)kind || e.rec.scope != (uint32_t)scope || e.rec.site != (uint32_t)site ||
      e.rec.bytes != (uint64_t)bytes || e.rec.dtype != (uint32_t)dtype)
    return fail(TM_ESTATE, "comm_call: entry %zu of the tape is (kind %u, scope %u, site %u, dtype %u, %llu bytes), the program asks (%d, %d, %d, %d, %lld)",
                c->at, e.rec.kind, e.rec.scope, e.rec.site, e.rec.dtype, (unsigned long long)e.rec.bytes, kind, scope, site, dtype,
                (long long)bytes);
  if (bytes > 0 && hipMemcpyAsync(buf, c->arena + e.arena_off, (size_t)bytes, hipMemcpyHostToDevice, s) != hipSuccess) {
    (void)hipGetLastError();
    return fail(TM_ELAUNCH, "comm_call: copy from the tape failed");
  }
  c->at += 1;
  c->stats.stored += 1;
  c->stats.stored_bytes += bytes;
  return TM_OK;
}

extern "C" int tm_comm_rewind(tm_comm_t *c) {
  if (!c) return fail(TM_EINVAL, "comm_rewind: NULL handle");
  if (c->mode != TM_COMM_REPLAY) return fail(TM_ESTATE, "comm_rewind: not a replaying hook");
  c->at = 0;
  return TM_OK;
}

extern "C" int tm_comm_stats(const tm_comm_t *c, tm_comm_stats_t *out) {
  if (!c || !out) return fail(TM_EINVAL, "comm_stats: NULL argument");
  *out = c->stats;
  return TM_OK;
}

extern "C" int tm_comm_close(tm_comm_t *c) {
  if (!c) return TM_OK;
  int rc = TM_OK;
  if (c->mode == TM_COMM_RECORD && c->f) {
    const uint64_t count = (uint64_t)c->stats.tape_entries;
    if (fseek(c->f, 8, SEEK_SET) != 0 || fwrite(&count, 8, 1, c->f) != 1 || fflush(c->f) != 0)
      rc = fail(TM_ELAUNCH, "comm_close: cannot finish tape %s", c->path.c_str());
  }
  comm_free(c);
  return rc;
}

// ---- what follows an intercepted all-reduce of a row-parallel map ---------------------------------
namespace tmk {
template <typename T>
__global__ __launch_bounds__(256) void bias_residual_add_kernel(const T *__restrict__ part, const T *__restrict__ bias,
                                                                const T *__restrict__ residual, T *__restrict__ out,
                                                                int64_t nchunk, int chunks_per_row) {
  constexpr int VN = Vec<T>::N;
  const int64_t ch = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (ch >= nchunk) return;
  float a[VN], r[VN];
  load_vec<T>(part + ch * VN, a);
  load_vec<T>(residual + ch * VN, r);
  if (bias) {
    float b[VN];
    load_vec<T>(bias + (ch % chunks_per_row) * VN, b);
#pragma unroll
    for (int i = 0; i < VN; ++i) a[i] += b[i];
  }
#pragma unroll
  for (int i = 0; i < VN; ++i) a[i] += r[i];
  store_vec<T>(out + ch * VN, a);
}
}  // namespace tmk

extern "C" int tm_op_bias_residual_add(int dtype, int64_t T, int64_t h, const void *part, const void *bias,
                                       const void *residual, void *out, void *stream) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "bias_residual_add: unknown dtype %d", dtype);
  if (T <= 0 || h <= 0) return fail(TM_EINVAL, "bias_residual_add: empty shape");
  if (h % 8) return fail(TM_ESIZE, "bias_residual_add: row width %lld is not a multiple of 8", (long long)h);
  if (!part || !residual || !out) return fail(TM_EINVAL, "bias_residual_add: NULL pointer");
  const int vn = dtype == TM_DTYPE_BF16 ? 8 : 4;
  const int64_t nchunk = T * h / vn;
  const unsigned grid = (unsigned)ceil_div(nchunk, 256);
  hipStream_t s = (hipStream_t)stream;
  g_last_kernel = "bias_residual_add_kernel";
  if (dtype == TM_DTYPE_BF16)
    bias_residual_add_kernel<bf16><<<grid, 256, 0, s>>>((const bf16 *)part, (const bf16 *)bias, (const bf16 *)residual,
                                                        (bf16 *)out, nchunk, (int)(h / vn));
  else
    bias_residual_add_kernel<float><<<grid, 256, 0, s>>>((const float *)part, (const float *)bias, (const float *)residual,
                                                         (float *)out, nchunk, (int)(h / vn));
  return check_launch("bias_residual_add");
}

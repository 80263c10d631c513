// Flash-style causal attention on the CDNA4 matrix cores (bf16 in, fp32 accumulate), head size 128.
//
// The s x s score matrix is never stored: a block walks tiles of 64 rows, keeps running row maxima
// and sums in registers (online softmax) and accumulates its outputs in MFMA accumulators.
//
// Transposed products.  Everything is formed transposed (S^T = K Q^T, O^T = V^T P^T, ...), so that
// in every 32x32 accumulator tile the lane index is the row that owns the softmax statistics (a query
// row in the forward and dQ kernels, a key row in the dK/dV kernel) and the 16 accumulator registers
// run along the reduction axis of the NEXT product.  A lane's 8 consecutive accumulator registers are
// then exactly the 8 reduction-axis values the next MFMA expects from it, under a fixed permutation of
// that axis (slot (half h, e) <-> offset 8*(e/4) + 4*h + e%4).  Row statistics need one cross-half
// exchange per tile and no row-wise shuffles.
//
// One tile format.  Every staged tile is [64 rows][128] bf16, row-major as in global memory, fetched
// straight into LDS (buffer_load ... lds), double buffered.  An operand that is needed with the tile's
// rows as MFMA rows is read with plain 16-byte LDS reads; an operand that is needed TRANSPOSED (V in
// O^T = V^T P^T, K in dQ^T = K^T dS^T, Q and dO in the dK/dV kernel) is read from the same tile with
// the transposing LDS read ds_read_b64_tr_b16, which can also deliver the permuted reduction order
// directly.  The chunk placement inside a row is chosen so that both kinds of read are free of bank
// conflicts.
//
// Gradients are accumulated without atomics: dQ by a block that owns 128 query rows; dK/dV by a block
// that owns 128 key rows and loops over all later query tiles of ONE query head.  With grouped-query
// attention (several query heads per kv head) each head's block writes an fp32 partial and a small
// kernel adds the partials of a group in head order (a block looping over the whole group instead would
// leave a chip of 256 compute units with seq/128 * kv heads blocks: 32 for a 4096-token sequence and one
// kv head).
#include <math.h>
#include <stdlib.h>

#include "attn.h"

namespace tmk {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int D = 128;               // head size
constexpr int TILE = 64;             // rows of a staged tile
constexpr int ROWB = D * 2;          // bytes per tile row
constexpr int TILE_BYTES = TILE * ROWB;
constexpr float kLog2e = 1.4426950408889634f;

// Position of 16-byte chunk c (of 16) in tile row `row`.  row_key takes 16 distinct values over 16
// consecutive rows (plain reads of one chunk column by 16 lanes hit 16 different bank groups); its bits
// 2:1 are the row's low bits (the 4 rows of a transposing read land in 4 different 32-byte windows);
// and chunk bit 1 is folded into bit 3 (the two 16-lane groups of a half-wave use different 128-byte halves).
__device__ __forceinline__ int row_key(int row) { return ((row & 3) << 1) | ((row >> 2) & 1) | (((row >> 3) & 1) << 3); }
__device__ __forceinline__ int place(int c, int row) { return c ^ row_key(row) ^ (((c >> 1) & 1) << 3); }
__device__ __forceinline__ int unplace(int pc, int row) {
  const int t = pc ^ row_key(row);
  return t ^ (((t >> 1) & 1) << 3);
}

struct FlashParams {
  const bf16 *qkv;
  const bf16 *dctx;
  bf16 *ctx;
  bf16 *dqkv;
  float *lse;
  const float *lse_in;
  const float *dvec;
  float *part;                   // grouped-query dK/dV partials [batch][nq][seq][2][D] fp32, or NULL
  int seq, batch, nq, nkv, row;  // row = (nq + 2 nkv) * D
  float scale;                   // 1 / sqrt(D)
  uint32_t qkv_bytes, ctx_bytes;
};

// ---- global -> LDS: one [64][128] tile, 4 wave-wide loads per wave -------------------------------
template <int NW = 4> struct TileLoaderN {
  static constexpr int NL = 16 / NW;  // wave-wide loads per wave and tile
  uint32_t voff[NL];
  // row_stride: elements between consecutive tile rows in global memory
  __device__ __forceinline__ void init(int64_t row_stride, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int idx = (i * NW + wave) * 64 + lane;  // chunk position in the LDS tile
      const int row = idx >> 4, c = unplace(idx & 15, row);
      voff[i] = (uint32_t)(((int64_t)row * row_stride + c * 8) * 2);
    }
  }
  // rows0: element offset of tile row 0 (a multiple of the row stride), base: element offset of column 0
  // inside a row (below the row stride).  The row part travels in the per-lane offset, which the
  // hardware checks against the buffer size, so rows past the tensor read as zero.
  __device__ __forceinline__ void issue(rsrc_t rs, char *tile, int64_t rows0, int64_t base, int wave) const {
    const uint32_t roff = (uint32_t)(rows0 * 2), soff = (uint32_t)(base * 2);
#pragma unroll
    for (int i = 0; i < NL; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(tile + (i * NW + wave) * 1024), 16, voff[i] + roff, soff, 0,
                                               0);
  }
};
typedef TileLoaderN<4> TileLoader;

// A-operand fragment, tile rows as MFMA rows: row r32 + lane%32, reduction slots 16ks + 8hh + 0..7
__device__ __forceinline__ bf16x8 frag_rows(const char *tile, int r32, int ks, int lane) {
  const int r = r32 + (lane & 31), hh = lane >> 5;
  return *reinterpret_cast<const bf16x8 *>(tile + r * ROWB + (place(2 * ks + hh, r) << 4));
}
// A-operand fragment of the TRANSPOSED tile: MFMA row = tile column c32 + lane%32, reduction axis =
// tile rows 16kk .. 16kk+15 in the permuted order (slot (hh, e) <-> row 16kk + 8*(e/4) + 4hh + e%4).
// ds_read_b64_tr_b16: within 16 lanes, lane i receives element i%4 of the 8-byte pieces addressed by
// lanes i/4, i/4+4, i/4+8, i/4+12; lane s addresses tile[row0 + s/4][col0 + 4*(s%4) ..+3].
__device__ __forceinline__ bf16x8 frag_cols(const char *tile, int c32, int kk, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const int col = c32 + 16 * (g & 1) + 4 * (s & 3);
  const int c = col >> 3, half = (col >> 2) & 1;
  union { s16x4 h[2]; bf16x8 v; } x;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int row = 16 * kk + 8 * t + 4 * (g >> 1) + (s >> 2);
    const char *a = tile + row * ROWB + (place(c, row) << 4) + (half << 3);
    x.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(a));
  }
  return x.v;
}
// The same two fragment reads with the address arithmetic written out.  Every lane-dependent part of an address
// fits one per-lane base (relative to the tile, which must start on a 256-byte boundary); what changes with the
// reduction slice, the 32-column block and the row group is an XOR of the 16-byte chunk index with a compile-time
// constant plus a multiple of the row pitch, so that one register per kind of read serves all of them (written
// through place() the compiler keeps one address register per read, about forty of them).
__device__ __forceinline__ uint32_t rows_base(int lane) {  // for frag_rows: row lane%32 of a 32-row block
  const int l32 = lane & 31, hh = lane >> 5;
  return (uint32_t)(l32 * ROWB + ((hh ^ row_key(l32)) << 4));
}
__device__ __forceinline__ bf16x8 frag_rows_at(const char *tile, uint32_t base, int r32, int ks) {
  const uint32_t x = (uint32_t)(((2 * ks) ^ ((ks & 1) << 3)) << 4);  // place(2ks + hh, row) = hh ^ row_key ^ this
  return *reinterpret_cast<const bf16x8 *>(tile + ((base ^ x) + (uint32_t)(r32 * ROWB)));
}
__device__ __forceinline__ uint32_t cols_base(int lane) {  // for frag_cols: the lane's column piece and row inside a group of 8
  const int g = lane >> 4, s = lane & 15;
  const int col = 16 * (g & 1) + 4 * (s & 3), c = col >> 3, half = (col >> 2) & 1;
  const int r = 4 * (g >> 1) + (s >> 2);
  const int pl = c ^ row_key(r) ^ (((c >> 1) & 1) << 3);
  return (uint32_t)(r * ROWB + (pl << 4) + (half << 3));
}
__device__ __forceinline__ bf16x8 frag_cols_at(const char *tile, uint32_t base, int c32, int kk) {
  union { s16x4 h[2]; bf16x8 v; } x;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint32_t xr = (uint32_t)((((c32 >> 3)) ^ (t << 3)) << 4);  // chunk index: + 4 per 32 columns, row_key bit 3 = t
    const char *a = tile + ((base ^ xr) + (uint32_t)((16 * kk + 8 * t) * ROWB));
    x.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(a));
  }
  return x.v;
}
// B-operand fragments straight from global memory: 8 consecutive elements of row (lane%32) per step
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
// the same accumulators as fp32: part_row points at [D] floats of this lane's token
__device__ __forceinline__ void store_transposed_f32(const f32x16 (&acc)[D / 32], float mul, float *part_row, int hh) {
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = acc[dt][q4 * 4 + e] * mul;
      *reinterpret_cast<f32x4 *>(part_row + dt * 32 + 8 * q4 + 4 * hh) = o;
    }
}
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// =================================================================================================
// forward
// =================================================================================================
// One wave's work on one staged K / V tile of 64 keys for its 32 query rows (lane%32 = query row): S^T = K Q^T,
// online softmax, O^T += V^T P^T.  Only the last one or two tiles of a walk can hold a key index above a query
// index of the wave: only those pay for the mask.  The running maximum is kept in exponent units
// (m = max * scale * log2 e); the accumulators and the row sum are rescaled only when some row of the wave saw its
// maximum rise (the factor is exactly 1 otherwise).
struct FwdRow {
  f32x16 o[D / 32];
  float m, l;
};
__device__ __forceinline__ void fwd_tile(const char *kt, const char *vt, const bf16x8 (&qf)[D / 16], FwdRow &r, int j0,
                                         int q0w, int q, int hh, float sc2, uint32_t rb, uint32_t cb) {
  f32x16 s[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
      s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_at(kt, rb, t * 32, ks), qf[ks], s[t], 0, 0, 0);
  }
  if (j0 + TILE - 1 > q0w) {  // wave-uniform
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (j0 + t * 32 + acc_row(v, hh) > q) s[t][v] = -INFINITY;
  }
  float mraw = -INFINITY;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) mraw = fmaxf(mraw, s[t][v]);
  float mx = fmaxf(r.m, mraw * sc2);
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  if (__builtin_amdgcn_ballot_w64(mx > r.m) != 0) {  // wave-uniform
    const float alpha = __builtin_amdgcn_exp2f(r.m - mx);
    r.m = mx;
    r.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) r.o[dt][v] *= alpha;
  }
  float ps = 0.f;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][v], sc2, -r.m));
      s[t][v] = e;
      ps += e;
    }
  r.l += ps;
#pragma unroll
  for (int kk = 0; kk < TILE / 16; ++kk) {
    const bf16x8 pf = pack8(s[kk >> 1], 8 * (kk & 1));
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
      r.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_at(vt, cb, dt * 32, kk), pf, r.o[dt], 0, 0, 0);
  }
}
__device__ __forceinline__ void fwd_finish(const FlashParams &p, FwdRow &r, int q, int n, int g, int hh) {
  r.l += __shfl_xor(r.l, 32, 64);
  if (q < p.seq) {
    const int64_t trow = (int64_t)q * p.batch + n;
    store_transposed(r.o, 1.f / r.l, p.ctx + trow * (p.nq * D) + g * D, hh);
    if (hh == 0) p.lse[((int64_t)n * p.nq + g) * p.seq + q] = (r.m + log2f(r.l)) * 0.6931471805599453f;
  }
}

// block = 32 NW query rows of one (batch entry, query head); wave = 32 query rows.  Four waves, two blocks per
// compute unit; or eight waves, one block: the same waves per unit, but every staged K / V tile serves twice the query
// rows, which halves the bytes a unit pulls from L2 into LDS per MFMA (what bounds the walk of a long sequence).
template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void flash_fwd_kernel(const FlashParams p) {
  __shared__ __align__(1024) char lds[2][2][TILE_BYTES];  // [stage][K, V]
  constexpr int QB = 32 * NW;
  const int qt = gridDim.z - 1 - blockIdx.z, g = blockIdx.x, n = blockIdx.y;  // heads fastest, longest walks first
  const int kap = g / (p.nq / p.nkv);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, hh = lane >> 5;
  const int q0w = qt * QB + wave * 32;
  const int q = q0w + l32;
  const int64_t tstride = (int64_t)p.batch * p.row;  // elements between consecutive positions
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;
  const rsrc_t rs = make_rsrc(p.qkv, p.qkv_bytes);
  TileLoaderN<NW> ld;
  ld.init(tstride, wave, lane);

  bf16x8 qf[D / 16];
  load_row_frags(p.qkv + (int64_t)n * p.row + (int64_t)q * tstride + g * D, q < p.seq, hh, qf);

  FwdRow r;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) r.o[dt][v] = 0.f;
  r.m = -INFINITY;
  r.l = 0.f;
  const float sc2 = p.scale * kLog2e;
  const uint32_t rb = rows_base(lane), cb = cols_base(lane);

  const int kv_end = (qt * QB + QB < p.seq) ? qt * QB + QB : p.seq;
  const int ntile = (kv_end + TILE - 1) / TILE;
  ld.issue(rs, lds[0][0], 0, (int64_t)n * p.row + koff, wave);
  ld.issue(rs, lds[0][1], 0, (int64_t)n * p.row + voff, wave);
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * TILE, cur = jt & 1;
    wait_loads();
    __builtin_amdgcn_s_barrier();  // tile jt is in LDS; everyone is done with the other stage
    if (jt + 1 < ntile) {
      const int64_t r0 = (int64_t)(j0 + TILE) * tstride;
      ld.issue(rs, lds[cur ^ 1][0], r0, (int64_t)n * p.row + koff, wave);
      ld.issue(rs, lds[cur ^ 1][1], r0, (int64_t)n * p.row + voff, wave);
    }
    if (j0 > q0w + 31) continue;  // every key of this tile lies after every query row of the wave
    fwd_tile(lds[cur][0], lds[cur][1], qf, r, j0, q0w, q, hh, sc2, rb, cb);
  }
  wait_loads();
  fwd_finish(p, r, q, n, g, hh);
}
template __global__ void flash_fwd_kernel<4>(const FlashParams);
template __global__ void flash_fwd_kernel<8>(const FlashParams);

// The same for grids of at most one block per compute unit (short sequences, few heads), where the chain of tile
// steps of the last query rows bounds the kernel: eight waves; waves w and w + 4 share a SIMD and 32 query rows
// and take the even and the odd key tiles, each with its own maximum, row sum and accumulators; at the end the odd
// side's state goes through LDS and the even side merges it (o = o1 2^(m1-m) + o2 2^(m2-m), the row sum alike).
// Half as many steps, and the two waves of a SIMD overlap each other's softmax and MFMA phases.
__global__ __launch_bounds__(512, 1) void flash_fwd_split_kernel(const FlashParams p) {
  extern __shared__ __align__(1024) char smem[];  // [stage][parity][K, V] tiles
  const int qt = gridDim.z - 1 - blockIdx.z, g = blockIdx.x, n = blockIdx.y;  // heads fastest, longest walks first
  const int kap = g / (p.nq / p.nkv);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qg = wave & 3, par = wave >> 2;
  const int l32 = lane & 31, hh = lane >> 5;
  const int q0w = qt * 128 + qg * 32;
  const int q = q0w + l32;
  const int64_t tstride = (int64_t)p.batch * p.row;
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;
  const rsrc_t rs = make_rsrc(p.qkv, p.qkv_bytes);
  TileLoaderN<8> ld;
  ld.init(tstride, wave, lane);
  auto tile = [&](int stage, int parity, int which) { return smem + ((stage * 2 + parity) * 2 + which) * TILE_BYTES; };

  bf16x8 qf[D / 16];
  load_row_frags(p.qkv + (int64_t)n * p.row + (int64_t)q * tstride + g * D, q < p.seq, hh, qf);

  FwdRow r;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) r.o[dt][v] = 0.f;
  r.m = -INFINITY;
  r.l = 0.f;
  const float sc2 = p.scale * kLog2e;
  const uint32_t rb = rows_base(lane), cb = cols_base(lane);

  const int kv_end = (qt * 128 + 128 < p.seq) ? qt * 128 + 128 : p.seq;
  const int ntile = (kv_end + TILE - 1) / TILE, nstep = (ntile + 1) / 2;
  auto issue_step = [&](int step, int stage) {  // both parities' tiles; a tile past the walk's end is not fetched
#pragma unroll
    for (int parity = 0; parity < 2; ++parity) {
      const int jt = 2 * step + parity;
      if (jt < ntile) {
        const int64_t r0 = (int64_t)jt * TILE * tstride;
        ld.issue(rs, tile(stage, parity, 0), r0, (int64_t)n * p.row + koff, wave);
        ld.issue(rs, tile(stage, parity, 1), r0, (int64_t)n * p.row + voff, wave);
      }
    }
  };
  issue_step(0, 0);
  for (int step = 0; step < nstep; ++step) {
    const int cur = step & 1;
    wait_loads();
    __builtin_amdgcn_s_barrier();  // this step's tiles are in LDS; everyone is done with the other stage
    if (step + 1 < nstep) issue_step(step + 1, cur ^ 1);
    const int jt = 2 * step + par, j0 = jt * TILE;
    if (jt >= ntile || j0 > q0w + 31) continue;
    fwd_tile(tile(cur, par, 0), tile(cur, par, 1), qf, r, j0, q0w, q, hh, sc2, rb, cb);
  }
  wait_loads();
  __syncthreads();  // the tiles are no longer needed: the odd side's state goes where they were
  float *xch = reinterpret_cast<float *>(smem) + (size_t)qg * ((D / 32) * 16 + 2) * 64;  // [qg][o..., m, l][lane]
  if (par == 1) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) xch[(dt * 16 + v) * 64 + lane] = r.o[dt][v];
    xch[(D / 32) * 16 * 64 + lane] = r.m;
    xch[((D / 32) * 16 + 1) * 64 + lane] = r.l;
  }
  __syncthreads();
  if (par == 0) {
    const float m2 = xch[(D / 32) * 16 * 64 + lane], l2 = xch[((D / 32) * 16 + 1) * 64 + lane];
    const float mm = fmaxf(r.m, m2);  // r.m is finite: the even side always has key tile 0
    const float a1 = __builtin_amdgcn_exp2f(r.m - mm), a2 = __builtin_amdgcn_exp2f(m2 - mm);
    r.m = mm;
    r.l = r.l * a1 + l2 * a2;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) r.o[dt][v] = r.o[dt][v] * a1 + xch[(dt * 16 + v) * 64 + lane] * a2;
    fwd_finish(p, r, q, n, g, hh);
  }
}

// =================================================================================================
// dQ: same walk as the forward pass; dQ^T += K^T dS^T
// =================================================================================================
// one wave, one staged K / V tile: probabilities from the stored log-sum-exp, dS = P (dP - D), dQ^T += K^T dS^T
__device__ __forceinline__ void dq_tile(const char *kt, const char *vt, const bf16x8 (&qf)[D / 16],
                                        const bf16x8 (&dof)[D / 16], f32x16 (&acc)[D / 32], float lse2, float dq_d, int j0,
                                        int q0w, int q, int hh, float sc2, uint32_t rb, uint32_t cb) {
  f32x16 ds[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    f32x16 s, dp;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = dp[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_at(kt, rb, t * 32, ks), qf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_at(vt, rb, t * 32, ks), dof[ks], dp, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v)
      ds[t][v] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], sc2, -lse2)) * (dp[v] - dq_d);
  }
  if (j0 + TILE - 1 > q0w) {  // wave-uniform: only the last one or two tiles can hold a key above a query
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (j0 + t * 32 + acc_row(v, hh) > q) ds[t][v] = 0.f;
  }
#pragma unroll
  for (int kk = 0; kk < TILE / 16; ++kk) {
    const bf16x8 df = pack8(ds[kk >> 1], 8 * (kk & 1));
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
      acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_at(kt, cb, dt * 32, kk), df, acc[dt], 0, 0, 0);
  }
}

// block = 128 query rows (tile qt) of one (batch entry, query head), four waves; lds: [stage][K, V] tiles, 64 KB.
// In a block of eight waves the other four only keep the barrier count (one barrier per key tile).
template <int NW = 4>
__device__ __forceinline__ void dq_block(const FlashParams &p, char *lds_base, int qt, int g, int n) {
  char (*lds)[2][TILE_BYTES] = reinterpret_cast<char (*)[2][TILE_BYTES]>(lds_base);
  constexpr int QB = 32 * NW;  // query rows of the block (NW = 8: see the forward kernel)
  const int kap = g / (p.nq / p.nkv);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave >= NW) {
    const int kv_end_x = (qt * QB + QB < p.seq) ? qt * QB + QB : p.seq;
    const int ntile_x = (kv_end_x + TILE - 1) / TILE;
    for (int jt = 0; jt < ntile_x; ++jt) __builtin_amdgcn_s_barrier();
    return;
  }
  const int l32 = lane & 31, hh = lane >> 5;
  const int q0w = qt * QB + wave * 32;
  const int q = q0w + l32;
  const bool qvalid = q < p.seq;
  const int64_t tstride = (int64_t)p.batch * p.row;
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;
  const int64_t cstride = (int64_t)p.batch * p.nq * D;
  const rsrc_t rs = make_rsrc(p.qkv, p.qkv_bytes);
  TileLoaderN<NW> ld;
  ld.init(tstride, wave, lane);

  bf16x8 qf[D / 16], dof[D / 16];
  load_row_frags(p.qkv + (int64_t)n * p.row + (int64_t)q * tstride + g * D, qvalid, hh, qf);
  load_row_frags(p.dctx + (int64_t)n * p.nq * D + (int64_t)q * cstride + g * D, qvalid, hh, dof);
  const int64_t si = ((int64_t)n * p.nq + g) * p.seq + q;
  const float lse2 = qvalid ? p.lse_in[si] * kLog2e : 0.f;
  const float dq_d = qvalid ? p.dvec[si] : 0.f;

  f32x16 acc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.f;
  const float sc2 = p.scale * kLog2e;
  const uint32_t rb = rows_base(lane), cb = cols_base(lane);

  const int kv_end = (qt * QB + QB < p.seq) ? qt * QB + QB : p.seq;
  const int ntile = (kv_end + TILE - 1) / TILE;
  ld.issue(rs, lds[0][0], 0, (int64_t)n * p.row + koff, wave);
  ld.issue(rs, lds[0][1], 0, (int64_t)n * p.row + voff, wave);
  for (int jt = 0; jt < ntile; ++jt) {
    const int j0 = jt * TILE, cur = jt & 1;
    wait_loads();
    __builtin_amdgcn_s_barrier();
    if (jt + 1 < ntile) {
      const int64_t r0 = (int64_t)(j0 + TILE) * tstride;
      ld.issue(rs, lds[cur ^ 1][0], r0, (int64_t)n * p.row + koff, wave);
      ld.issue(rs, lds[cur ^ 1][1], r0, (int64_t)n * p.row + voff, wave);
    }
    if (j0 > q0w + 31) continue;
    dq_tile(lds[cur][0], lds[cur][1], qf, dof, acc, lse2, dq_d, j0, q0w, q, hh, sc2, rb, cb);
  }
  wait_loads();
  if (qvalid) store_transposed(acc, p.scale, p.dqkv + ((int64_t)q * p.batch + n) * p.row + g * D, hh);
}
template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void flash_bwd_dq_kernel(const FlashParams p) {
  __shared__ __align__(1024) char lds[4 * TILE_BYTES];
  dq_block<NW>(p, lds, gridDim.z - 1 - blockIdx.z, blockIdx.x, blockIdx.y);  // heads fastest, longest walks first
}
template __global__ void flash_bwd_dq_kernel<4>(const FlashParams);
template __global__ void flash_bwd_dq_kernel<8>(const FlashParams);

// =================================================================================================
// dK, dV: block = 128 key rows of one (batch entry, query head), eight waves: wave = 32 key rows x one 32-query
// half of every 64-row query tile (waves w and w + 4 share a SIMD and the key rows and take the two halves);
// loops over the query tiles from the diagonal to the end.  The two halves' sums over their queries are added
// through LDS at the end (first half + second half: a fixed order).  One query head per kv head: the block's
// result is the gradient.  Grouped heads: it is that head's fp32 partial.
// =================================================================================================
// smem: [stage][Q, dO] tiles, then [stage][lse, D] rows of floats, then the V fragments (kDkvLds bytes)
constexpr int kDkvLds = 4 * TILE_BYTES + 2 * 2 * TILE * (int)sizeof(float) + 128 * D * 2;
__device__ __forceinline__ void dkv_block(const FlashParams &p, char *smem, int kt, int g, int n) {
  const int group = p.nq / p.nkv, kap = g / group;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kr = wave & 3, t = wave >> 2;  // key-row group, query half
  const int l32 = lane & 31, hh = lane >> 5;
  const int j0w = kt * 128 + kr * 32;
  const int j = j0w + l32;
  const bool jvalid = j < p.seq;
  const int64_t tstride = (int64_t)p.batch * p.row;
  const int koff = p.nq * D + kap * D, voff = (p.nq + p.nkv) * D + kap * D;
  const int64_t cstride = (int64_t)p.batch * p.nq * D;
  const rsrc_t rq = make_rsrc(p.qkv, p.qkv_bytes), rdo = make_rsrc(p.dctx, p.ctx_bytes);
  TileLoaderN<8> lq, ldo;
  lq.init(tstride, wave, lane);
  ldo.init(cstride, wave, lane);
  auto tile = [&](int stage, int which) { return smem + (stage * 2 + which) * TILE_BYTES; };
  float *stats = reinterpret_cast<float *>(smem + 4 * TILE_BYTES);  // [stage][2][TILE]

  // The wave's K fragments stay in registers; its V fragments live in LDS ([key-row group][slice][lane], 16 bytes
  // each: 32 KB a block, written once by the first query half) and are read again at every use, which keeps the
  // kernel inside 256 registers without spills.
  bf16x8 kf[D / 16];
  load_row_frags(p.qkv + (int64_t)n * p.row + (int64_t)j * tstride + koff, jvalid, hh, kf);
  char *vl = smem + 4 * TILE_BYTES + 2 * 2 * TILE * (int)sizeof(float) + (kr * (D / 16) * 64 + lane) * 16;
  if (t == 0) {
    bf16x8 vf[D / 16];
    load_row_frags(p.qkv + (int64_t)n * p.row + (int64_t)j * tstride + voff, jvalid, hh, vf);
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) *reinterpret_cast<bf16x8 *>(vl + ks * 64 * 16) = vf[ks];
  }

  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dk[dt][v] = dv[dt][v] = 0.f;
  const float sc2 = p.scale * kLog2e;
  const uint32_t rb = rows_base(lane), cb = cols_base(lane);

  const int it_begin = (kt * 128) / TILE;
  const int it_end = (p.seq + TILE - 1) / TILE;
  const int total = it_end - it_begin;
  // the query tiles of this head, double buffered; the row statistics of a step are fetched into registers one
  // step ahead by the first wave and put into LDS just before the barrier that publishes the step's tiles
  float st_lse = 0.f, st_d = 0.f;
  auto issue_step = [&](int step, int stage) {
    const int i0 = (it_begin + step) * TILE;
    lq.issue(rq, tile(stage, 0), (int64_t)i0 * tstride, (int64_t)n * p.row + g * D, wave);
    ldo.issue(rdo, tile(stage, 1), (int64_t)i0 * cstride, (int64_t)n * p.nq * D + g * D, wave);
    if (threadIdx.x < TILE) {
      const int i = i0 + threadIdx.x;
      const int64_t sidx = ((int64_t)n * p.nq + g) * p.seq + i;
      st_lse = i < p.seq ? p.lse_in[sidx] * kLog2e : 0.f;
      st_d = i < p.seq ? p.dvec[sidx] : 0.f;
    }
  };
  issue_step(0, 0);
  for (int step = 0; step < total; ++step) {
    const int cur = step & 1;
    const int i0 = (it_begin + step) * TILE;
    wait_loads();
    if (threadIdx.x < TILE) {
      float *st = stats + cur * 2 * TILE;
      st[threadIdx.x] = st_lse;
      st[TILE + threadIdx.x] = st_d;
    }
    __syncthreads();  // tiles and statistics of this step are visible; the other stage is free
    if (step + 1 < total) issue_step(step + 1, cur ^ 1);
    if (i0 + t * 32 + 31 < j0w) continue;  // every query of this wave's half lies before every key row of the wave
    const char *qt = tile(cur, 0), *dot = tile(cur, 1);
    const float *lse_s = stats + cur * 2 * TILE, *dv_s = lse_s + TILE;

    const bool diag = i0 + t * 32 < j0w + 31;  // some query index may be below some key index
    f32x16 s, dp;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = dp[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_at(qt, rb, t * 32, ks), kf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_at(dot, rb, t * 32, ks), *reinterpret_cast<const bf16x8 *>(vl + ks * 64 * 16), dp, 0, 0, 0);
    }
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int ib = t * 32 + 8 * q4 + 4 * hh;  // four consecutive query rows of this lane
      const f32x4 l4 = *reinterpret_cast<const f32x4 *>(lse_s + ib);
      const f32x4 d4 = *reinterpret_cast<const f32x4 *>(dv_s + ib);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = q4 * 4 + e;
        const float x = __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], sc2, -l4[e]));
        s[v] = x;                     // P
        dp[v] = x * (dp[v] - d4[e]);  // dS
      }
    }
    if (diag) {  // wave-uniform: only the first tiles of the walk can hold a query below a key of the wave
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (i0 + t * 32 + acc_row(v, hh) < j) s[v] = dp[v] = 0.f;
    }
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      const int kk = 2 * t + k2;
      const bf16x8 pf = pack8(s, 8 * k2);
      const bf16x8 df = pack8(dp, 8 * k2);
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
        dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_at(dot, cb, dt * 32, kk), pf, dv[dt], 0, 0, 0);
        dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_at(qt, cb, dt * 32, kk), df, dk[dt], 0, 0, 0);
      }
    }
  }
  wait_loads();
  // the second query half hands its sums to the first through LDS (the tiles are no longer needed): dK, then dV
  float *xch = reinterpret_cast<float *>(smem) + (size_t)kr * (D / 32) * 16 * 64;  // [kr][dt][v][lane]
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    __syncthreads();
    if (t == 1) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) xch[(dt * 16 + v) * 64 + lane] = which == 0 ? dk[dt][v] : dv[dt][v];
    }
    __syncthreads();
    if (t == 0) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float other = xch[(dt * 16 + v) * 64 + lane];
          if (which == 0) dk[dt][v] += other;
          else dv[dt][v] += other;
        }
    }
  }
  if (jvalid && t == 0) {
    if (p.part) {
      float *out = p.part + (((int64_t)n * p.nq + g) * p.seq + j) * (2 * D);
      store_transposed_f32(dk, p.scale, out, hh);
      store_transposed_f32(dv, 1.f, out + D, hh);
    } else {
      bf16 *out = p.dqkv + ((int64_t)j * p.batch + n) * p.row;
      store_transposed(dk, p.scale, out + koff, hh);
      store_transposed(dv, 1.f, out + voff, hh);
    }
  }
}

__global__ __launch_bounds__(512, 1) void flash_bwd_dkv_kernel(const FlashParams p) {
  extern __shared__ __align__(1024) char smem[];
  dkv_block(p, smem, blockIdx.z, blockIdx.x, blockIdx.y);  // heads fastest, longest walks first
}

// Both backward kernels in one launch, for grids that leave compute units idle (at most one block of each kind per
// unit): the dK/dV block of key tile r and the dQ block of query tile last - r alternate in dispatch order, both
// kinds longest first, so that the chip works on the two independent halves of the backward pass at once instead of
// waiting twice for a longest walk (2048 tokens, 12 heads: 192 + 192 blocks on 256 units).  Blocks of eight waves;
// in a dQ block four of them only keep the barrier count.
__global__ __launch_bounds__(512, 1) void flash_bwd_both_kernel(const FlashParams p) {
  extern __shared__ __align__(1024) char smem[];
  const int rank = blockIdx.z >> 1, tiles = gridDim.z >> 1;
  if (blockIdx.z & 1) dq_block<4>(p, smem, tiles - 1 - rank, blockIdx.x, blockIdx.y);
  else dkv_block(p, smem, rank, blockIdx.x, blockIdx.y);
}

// dK, dV of a kv head = sum of its query heads' partials, added in head order; thread = 4 columns
__global__ __launch_bounds__(256) void flash_dkv_reduce_kernel(const FlashParams p) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // over [batch][nkv][seq][2 * D / 4]
  const int64_t total = (int64_t)p.batch * p.nkv * p.seq * (2 * D / 4);
  if (idx >= total) return;
  const int c4 = (int)(idx % (2 * D / 4));
  const int64_t r = idx / (2 * D / 4);
  const int j = (int)(r % p.seq);
  const int kap = (int)((r / p.seq) % p.nkv), n = (int)(r / ((int64_t)p.seq * p.nkv));
  const int group = p.nq / p.nkv;
  f32x4 sum = {0.f, 0.f, 0.f, 0.f};
  for (int gg = 0; gg < group; ++gg) {
    const float *src = p.part + (((int64_t)n * p.nq + kap * group + gg) * p.seq + j) * (2 * D) + c4 * 4;
    const f32x4 v = *reinterpret_cast<const f32x4 *>(src);
#pragma unroll
    for (int e = 0; e < 4; ++e) sum[e] += v[e];
  }
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16)sum[e];
  const int which = c4 / (D / 4), col = (c4 % (D / 4)) * 4;  // 0: dK, 1: dV
  bf16 *out = p.dqkv + ((int64_t)j * p.batch + n) * p.row + (p.nq + which * p.nkv + kap) * D + col;
  *reinterpret_cast<bf16x4 *>(out) = o;
}

bool attn_mfma_supported(int dtype, int64_t d) { return dtype == TM_DTYPE_BF16 && d == D; }

static FlashParams make_params(int64_t seq, int64_t batch, int64_t nq, int64_t nkv) {
  FlashParams p = {};
  p.seq = (int)seq;
  p.batch = (int)batch;
  p.nq = (int)nq;
  p.nkv = (int)nkv;
  p.row = (int)((nq + 2 * nkv) * D);
  p.scale = (float)(1.0 / sqrt((double)D));
  p.qkv_bytes = (uint32_t)(seq * batch * p.row * 2);
  p.ctx_bytes = (uint32_t)(seq * batch * nq * D * 2);
  return p;
}

// The eight-wave forward kernel that splits a query block's key tiles between two waves serves grids that leave
// compute units without a second block (at most one block per unit).  TM_ATTN_SPLIT=0 / 1 in the environment forces
// the choice (tuning and test aid).  (The same form of the dQ kernel was faster alone and slower inside the backward
// pass, where its 128 KB blocks wait for LDS beside the weight-gradient products of the other stream: not kept.)
static bool use_split(dim3 grid) {
  if (const char *e = getenv("TM_ATTN_SPLIT")) return e[0] == '1';
  static int units = 0;
  if (!units) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        units <= 0)
      units = 256;
  }
  return (int64_t)grid.x * grid.y * grid.z <= units;
}

// Blocks of 256 query rows (eight waves) for the forward and dQ walks of grids that still give every compute unit two
// such blocks.  TM_ATTN_WIDE=0 / 1 forces the choice.
static bool use_wide(int64_t seq, int64_t batch, int64_t nq) {
  if (const char *e = getenv("TM_ATTN_WIDE")) return e[0] == '1';
  int dev = 0, units = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      units <= 0)
    units = 256;
  return ceil_div(seq, 256) * batch * nq >= 2 * (int64_t)units;
}

// One launch for both backward kernels where neither fills the chip by itself.  TM_ATTN_BWD_BOTH=0 / 1 forces the choice.
static bool use_both(dim3 grid) {
  if (const char *e = getenv("TM_ATTN_BWD_BOTH")) return e[0] == '1';
  static int units = 0;
  if (!units) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        units <= 0)
      units = 256;
  }
  return (int64_t)grid.x * grid.y * grid.z <= units;
}

int attn_fwd_mfma_launch(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *qkv, void *ctx,
                         float *lse, hipStream_t s) {
  (void)d;
  if (seq * batch * (nq + 2 * nkv) * D * 2 >= (1LL << 31)) return fail(TM_ESIZE, "flash_fwd: qkv tensor above 2 GiB");
  FlashParams p = make_params(seq, batch, nq, nkv);
  p.qkv = (const bf16 *)qkv;
  p.ctx = (bf16 *)ctx;
  p.lse = lse;
  if (ceil_div(seq, 128) > 65535 || batch > 65535) return fail(TM_ESIZE, "flash_fwd: sequence or batch too long for the grid");
  // Block order = dispatch order: all heads of the longest walk (last query tile) first, then the next shorter one.
  // With the heads outermost instead, a long sequence's late heads start their longest walks when the chip is
  // already draining (16384 tokens, 8 heads, 512 block slots: 408 tile steps end to end against 258 balanced).
  dim3 grid((unsigned)nq, (unsigned)batch, (unsigned)ceil_div(seq, 128));
  if (use_split(grid)) {
    const int lds = 8 * TILE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
      if (hipFuncSetAttribute(reinterpret_cast<const void *>(&flash_fwd_split_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
        return fail(TM_ELAUNCH, "flash_fwd: cannot reserve LDS");
      attr_set = true;
    }
    g_last_kernel = "flash_fwd_split_kernel";
    flash_fwd_split_kernel<<<grid, 512, lds, s>>>(p);
  } else {
    g_last_kernel = "flash_fwd_kernel";
    if (use_wide(seq, batch, nq))
      flash_fwd_kernel<8><<<dim3((unsigned)nq, (unsigned)batch, (unsigned)ceil_div(seq, 256)), 512, 0, s>>>(p);
    else
      flash_fwd_kernel<4><<<grid, 256, 0, s>>>(p);
  }
  return check_launch("flash_fwd");
}

int64_t attn_bwd_mfma_partial_floats(int64_t seq, int64_t batch, int64_t nq, int64_t nkv) {
  return nq == nkv ? 0 : batch * nq * seq * 2 * D;
}

int attn_bwd_mfma_launch(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *qkv,
                         const void *dctx, const float *lse, const float *dvec, float *part, void *dqkv,
                         hipStream_t s) {
  (void)d;
  if (seq * batch * (nq + 2 * nkv) * D * 2 >= (1LL << 31)) return fail(TM_ESIZE, "flash_bwd: qkv tensor above 2 GiB");
  FlashParams p = make_params(seq, batch, nq, nkv);
  p.qkv = (const bf16 *)qkv;
  p.dctx = (const bf16 *)dctx;
  p.lse_in = lse;
  p.dvec = dvec;
  p.dqkv = (bf16 *)dqkv;
  p.part = nq == nkv ? nullptr : part;
  if (nq != nkv && !part) return fail(TM_EINVAL, "flash_bwd: grouped heads need the partial buffer");
  if (ceil_div(seq, 128) > 65535 || batch > 65535) return fail(TM_ESIZE, "flash_bwd: sequence or batch too long for the grid");
  const unsigned tiles = (unsigned)ceil_div(seq, 128);
  dim3 gq((unsigned)nq, (unsigned)batch, tiles);  // heads fastest: see the forward launch
  const int lds = kDkvLds;
  static_assert(kDkvLds >= 4 * TILE_BYTES, "the dQ block's tiles fit the dK/dV block's LDS");
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&flash_bwd_dkv_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void *>(&flash_bwd_both_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
      return fail(TM_ELAUNCH, "flash_bwd: cannot reserve LDS");
    attr_set = true;
  }
  g_last_kernel = "flash_bwd_dq_kernel+flash_bwd_dkv_kernel";
  if (use_both(gq) && 2 * tiles <= 65535) {
    g_last_kernel = "flash_bwd_both_kernel";
    flash_bwd_both_kernel<<<dim3((unsigned)nq, (unsigned)batch, 2 * tiles), 512, lds, s>>>(p);
  } else {
    if (use_wide(seq, batch, nq))
      flash_bwd_dq_kernel<8><<<dim3((unsigned)nq, (unsigned)batch, (unsigned)ceil_div(seq, 256)), 512, 0, s>>>(p);
    else
      flash_bwd_dq_kernel<4><<<gq, 256, 0, s>>>(p);
    flash_bwd_dkv_kernel<<<gq, 512, lds, s>>>(p);
  }
  if (p.part) {
    const int64_t total = batch * nkv * seq * (2 * D / 4);
    flash_dkv_reduce_kernel<<<(unsigned)ceil_div(total, (int64_t)256), 256, 0, s>>>(p);
  }
  return check_launch("flash_bwd");
}

}  // namespace tmk
